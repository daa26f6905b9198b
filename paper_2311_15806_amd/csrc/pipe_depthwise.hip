// Expanded depthwise convolution (App. H: a convolution whose filters see one input channel;
// the separable blocks of MobileNet / EfficientNet).  Not a dense contraction: every output is
// kh*kw multiply-adds per order, so the layer is bound by reading Q(x) and writing y, and runs
// on the vector ALUs: a thread owns one (pixel, channel), reads its window once and applies
// every stored order of the channel to it.  Arithmetic as everywhere: exact integer sums,
// fp32 sum over the orders of a member in ascending order, activation scale, bias.
#include <hip/hip_runtime.h>

#include "pipe_internal.h"

namespace {

constexpr int BLK = 256;
constexpr int MAX_WIN = 49;   // up to 7 x 7

// codes[k][i][o] (tap-major, channel-minor: the codes of four neighbouring channels for one
// tap are one 32-bit word) and scales[k][o] of one order, from its unpacked stored rows
__global__ void dense_order_kernel(const int8_t* __restrict__ rows_codes, const float* __restrict__ scales_all,
                                   const int32_t* __restrict__ pos, const int32_t* __restrict__ gids, int group, int in,
                                   int C, int8_t* __restrict__ codes_k, float* __restrict__ scales_k) {
  const int r = blockIdx.x;   // stored row
  const int slot = r / group;
  const int o = gids[slot] * group + (r - slot * group);
  for (int i = threadIdx.x; i < in; i += blockDim.x) codes_k[(size_t)i * C + o] = rows_codes[(size_t)r * in + i];
  if (threadIdx.x == 0) scales_k[o] = scales_all[(size_t)pos[r >> 4] * 16 + (r & 15)];
}

// fp32 [N,C,H,W] -> int8 codes [N,H,W,C]: 32 channels x 32 pixels per workgroup through LDS, so
// that reads run along the pixels and writes along the channels
__global__ __launch_bounds__(256) void quantize_to_nhwc_kernel(const float* __restrict__ x, int C, int HW, float s_static,
                                                               const uint32_t* __restrict__ amax_bits, float qmax,
                                                               int8_t* __restrict__ q8, float* __restrict__ scale_out) {
  __shared__ int8_t tile[32][33];
  const float s = s_static > 0.f ? s_static : __fdiv_rn(__uint_as_float(*amax_bits), qmax);
  if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x == 0 && scale_out) *scale_out = s;
  const int n = blockIdx.z, c0 = blockIdx.y * 32, p0 = blockIdx.x * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int c = c0 + ty + 8 * j, pp = p0 + tx;
    int v = 0;
    if (c < C && pp < HW && s > 0.f) {
      float q = rintf(__fdiv_rn(x[((size_t)n * C + c) * HW + pp], s));
      q = fminf(fmaxf(q, -qmax), qmax);
      v = (int)q;
    }
    tile[ty + 8 * j][tx] = (int8_t)v;
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int pp = p0 + ty + 8 * j, c = c0 + tx;
    if (c < C && pp < HW) q8[((size_t)n * HW + pp) * C + c] = tile[tx][ty + 8 * j];
  }
}

struct DwParams {
  const int8_t* q8;        // Q(x), channels last [N,H,W,C]
  const float* s_x;
  const int8_t* codes;     // [K][kk][C]
  const float* scales;     // [K][C]
  const float* bias;
  float* y;                // [T, C] or [M, T, C]
  int N, C, H, W, kh, kw, stride, pad, Ho, Wo;
  int K, M, reduce;
  int member_lo[PIPE_MAX_K], member_hi[PIPE_MAX_K];
};

__device__ __forceinline__ int byte_of(uint32_t w, int j) { return (int)(int8_t)(w >> (8 * j)); }

// A thread owns one pixel and four neighbouring channels (C is a multiple of 16): one 32-bit
// load per window tap, one per tap and order for the codes, 16-byte stores.  KH, KW > 0: the
// window is a compile-time size and lives in registers; 0: any size up to MAX_WIN.
template <int KH, int KW>
__global__ __launch_bounds__(BLK) void depthwise_kernel(const DwParams p) {
  const int C4 = p.C >> 2;
  const long long idx = (long long)blockIdx.x * BLK + threadIdx.x;   // (pixel, channel quad), quad fastest
  const long long n_pix = (long long)p.N * p.Ho * p.Wo;
  if (idx >= n_pix * C4) return;
  const int c = (int)(idx % C4) * 4;
  const long long pix = idx / C4;
  const int wo = (int)(pix % p.Wo), ho = (int)((pix / p.Wo) % p.Ho), n = (int)(pix / ((long long)p.Wo * p.Ho));
  const int kh = KH > 0 ? KH : p.kh, kw = KW > 0 ? KW : p.kw;
  const int kk = kh * kw;
  uint32_t win[KH > 0 ? KH * KW : MAX_WIN];
#pragma unroll
  for (int r = 0; r < (KH > 0 ? KH : MAX_WIN); ++r) {
    if (r >= kh) break;
#pragma unroll
    for (int q = 0; q < (KW > 0 ? KW : MAX_WIN); ++q) {
      if (q >= kw) break;
      const int hi = ho * p.stride - p.pad + r, wi = wo * p.stride - p.pad + q;
      uint32_t v = 0;
      if (hi >= 0 && hi < p.H && wi >= 0 && wi < p.W)
        v = *reinterpret_cast<const uint32_t*>(p.q8 + (((size_t)n * p.H + hi) * p.W + wi) * p.C + c);
      win[r * kw + q] = v;
    }
  }
  const float sx = p.s_x[0];
  float4 bias = make_float4(0.f, 0.f, 0.f, 0.f);
  if (p.bias != nullptr) bias = *reinterpret_cast<const float4*>(p.bias + c);
  float ysum[4] = {0.f, 0.f, 0.f, 0.f};
  for (int m = 0; m < p.M; ++m) {
    float yacc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int k = p.member_lo[m]; k <= p.member_hi[m]; ++k) {
      const float4 s4 = *reinterpret_cast<const float4*>(p.scales + (size_t)k * p.C + c);
      if (s4.x == 0.f && s4.y == 0.f && s4.z == 0.f && s4.w == 0.f) continue;   // all four pruned at this order
      const int8_t* w = p.codes + (size_t)k * kk * p.C + c;
      int acc[4] = {0, 0, 0, 0};
      auto tap = [&](int i) __attribute__((always_inline)) {
        const uint32_t cw = *reinterpret_cast<const uint32_t*>(w + (size_t)i * p.C);
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] += byte_of(win[i], j) * byte_of(cw, j);
      };
      if (KH > 0) {
#pragma unroll
        for (int i = 0; i < KH * KW; ++i) tap(i);
      } else {
        for (int i = 0; i < kk; ++i) tap(i);
      }
      const float sv[4] = {s4.x, s4.y, s4.z, s4.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) yacc[j] = fmaf(sv[j], (float)acc[j], yacc[j]);   // a pruned channel has scale 0 and codes 0
    }
    const float bv[4] = {bias.x, bias.y, bias.z, bias.w};
    float v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      v[j] = fmaf(sx, yacc[j], m == 0 ? bv[j] : 0.f);
      ysum[j] = m == 0 ? v[j] : ysum[j] + v[j];
    }
    if (!p.reduce) *reinterpret_cast<float4*>(p.y + ((size_t)m * n_pix + pix) * p.C + c) = make_float4(v[0], v[1], v[2], v[3]);
  }
  if (p.reduce) *reinterpret_cast<float4*>(p.y + (size_t)pix * p.C + c) = make_float4(ysum[0], ysum[1], ysum[2], ysum[3]);
}

}  // namespace

int pipe_depthwise_prepare(pipe_expansion* e, hipStream_t st) {
  if (e->dw_codes_dev != nullptr) return PIPE_OK;
  const size_t n_codes = (size_t)e->K * e->out * e->in;
  PIPE_HIP(hipMalloc(&e->dw_codes_dev, n_codes));
  PIPE_HIP(hipMalloc(&e->dw_scales_dev, (size_t)e->K * e->out * sizeof(float)));
  PIPE_HIP(hipMemsetAsync(e->dw_codes_dev, 0, n_codes, st));
  PIPE_HIP(hipMemsetAsync(e->dw_scales_dev, 0, (size_t)e->K * e->out * sizeof(float), st));
  for (int k = 0; k < e->K; ++k) {
    const PipeOrder& o = e->orders[k];
    const int rows = o.n_kept * e->group;
    if (rows == 0) continue;
    int8_t* tmp = (int8_t*)pipe_ws_get(WS_DIAG_CODES, (size_t)rows * e->in);
    if (!tmp) return pipe_ws_error();
    int rc = launch_unpack_codes(e->codes_dev, o.pos_dev, e->bits, rows, e->in, e->in_pad, tmp, st);
    if (rc) return rc;
    PIPE_KLAUNCH(dense_order_kernel, dim3(rows), dim3(64), 0, st, tmp, e->scales_all_dev, o.pos_dev, o.gids_dev,
                       e->group, e->in, e->out, e->dw_codes_dev + (size_t)k * e->out * e->in, e->dw_scales_dev + (size_t)k * e->out);
    PIPE_HIP(hipGetLastError());
  }
  PIPE_HIP(hipStreamSynchronize(st));   // the scratch rows are reused by other calls
  return PIPE_OK;
}

int launch_quantize_to_nhwc(const float* x, int N, int C, int HW, float s_static, const uint32_t* amax_bits, float qmax,
                            int8_t* q8, float* scale_out, hipStream_t st) {
  PIPE_KLAUNCH(quantize_to_nhwc_kernel, dim3(ceil_div(HW, 32), ceil_div(C, 32), N), dim3(256), 0, st, x, C, HW, s_static,
                     amax_bits, qmax, q8, scale_out);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

int launch_depthwise(const pipe_expansion* e, const int8_t* q8, const float* s_x, int N, int C, int H, int W, int kh, int kw,
                     int stride, int pad, int Ho, int Wo, int M, const int* lo, const int* hi,
                     const float* bias, int reduce, float* y, hipStream_t st) {
  if (kh * kw > MAX_WIN || (C & 3) != 0) return PIPE_ESHAPE;
  DwParams p;
  p.q8 = q8; p.s_x = s_x; p.codes = e->dw_codes_dev; p.scales = e->dw_scales_dev; p.bias = bias; p.y = y;
  p.N = N; p.C = C; p.H = H; p.W = W; p.kh = kh; p.kw = kw; p.stride = stride; p.pad = pad; p.Ho = Ho; p.Wo = Wo;
  p.K = e->K; p.M = M; p.reduce = reduce;
  for (int m = 0; m < PIPE_MAX_K; ++m) { p.member_lo[m] = m < M ? lo[m] : 0; p.member_hi[m] = m < M ? hi[m] : -1; }
  const long long total = (long long)N * Ho * Wo * (C / 4);
  if (total <= 0) return PIPE_OK;
  const dim3 grid((unsigned)((total + BLK - 1) / BLK));
  if (kh == 3 && kw == 3) PIPE_KLAUNCH((depthwise_kernel<3, 3>), grid, dim3(BLK), 0, st, p);
  else if (kh == 5 && kw == 5) PIPE_KLAUNCH((depthwise_kernel<5, 5>), grid, dim3(BLK), 0, st, p);
  else if (kh == 7 && kw == 7) PIPE_KLAUNCH((depthwise_kernel<7, 7>), grid, dim3(BLK), 0, st, p);
  else PIPE_KLAUNCH((depthwise_kernel<0, 0>), grid, dim3(BLK), 0, st, p);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}
