// Weight-streaming kernel of the expanded layer for decode-sized batches (T <= 16), where the
// path is bound by reading the packed codes from HBM once (App. B, Eq. (define_dre), same
// arithmetic as the tiled kernel).
//
// Work item = one stored row block (16 rows of one order, all of in_features).  A workgroup
// owns a bin of items that together hold every order of a few output row blocks; its waves
// split the k dimension (wave w takes packed tiles w, w+NW, ...), so each wave streams its
// own 1-KiB tiles straight from HBM into registers with fully coalesced 16-byte loads, widens
// them with a shift and a mask and feeds v_mfma_i32_16x16x64_i8 against the 16-token
// activation fragments (also read straight from L2: waves use disjoint k, nothing is shared,
// so the k loop has no LDS traffic and no barrier).  The waves' partial int32 tiles are summed
// with LDS integer adds (exact, order independent); the epilogue then applies offsets, row
// scales, activation scale, bias and the member sum in a fixed order, so results are
// bit-reproducible.
#include "pipe_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int R = 4;  // items processed concurrently by a wave (independent load streams)

struct StreamParams {
  const uint8_t* qx;
  int64_t qx_mstride;
  const int32_t* rowsum;
  int64_t rowsum_mstride;
  const float* s_x;
  int sx_mstride;
  const uint8_t* packed[PIPE_MAX_K];
  const float* scales[PIPE_MAX_K];
  const StreamBin* bins;
  const float* bias;
  float* y;
  int32_t* acc_out;
  uint32_t* amax_out;
  int T, out, K, nks, M, reduce, act;
  int member_lo[PIPE_MAX_K];
  int member_hi[PIPE_MAX_K];
  int member_of[PIPE_MAX_K];
};

__device__ __forceinline__ float gelu_erf(float a) {
  return 0.5f * a * (1.f + erff(a * 0.70710678118654752440f));
}

template <int BITS>
__device__ __forceinline__ void unpack_step(const uint4& w, int j, v4i& o) {
  if (BITS == 8) {
    o = v4i{(int)w.x, (int)w.y, (int)w.z, (int)w.w};
  } else if (BITS == 4) {
    const uint32_t a = j == 0 ? w.x : w.z, b = j == 0 ? w.y : w.w;
    o = v4i{(int)(a & 0x0F0F0F0Fu), (int)((a >> 4) & 0x0F0F0F0Fu), (int)(b & 0x0F0F0F0Fu), (int)((b >> 4) & 0x0F0F0F0Fu)};
  } else {
    const uint32_t a = j == 0 ? w.x : (j == 1 ? w.y : (j == 2 ? w.z : w.w));
    o = v4i{(int)(a & 0x03030303u), (int)((a >> 2) & 0x03030303u), (int)((a >> 4) & 0x03030303u), (int)((a >> 6) & 0x03030303u)};
  }
}

template <int BITS, int NW, bool SHARED_X, bool ACC_OUT>
__global__ __launch_bounds__(NW * 64) void gemm_stream_kernel(const StreamParams p) {
  constexpr int OFF = BITS == 8 ? 0 : (BITS == 4 ? 8 : 1);
  constexpr int KSUP = 512 / BITS;
  constexpr int STEPS = KSUP / 64;      // 64-k steps per packed tile
  __shared__ int fin[STREAM_BIN_CAP][256];

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const StreamBin& bin = p.bins[blockIdx.x];
  const int n_items = bin.n_items;
  const int n_tiles = (p.nks * 64) / KSUP;

  for (int i = threadIdx.x; i < STREAM_BIN_CAP * 256; i += NW * 64) (&fin[0][0])[i] = 0;
  __syncthreads();

  for (int c0 = 0; c0 < n_items; c0 += R) {
    const uint4* wp[R];
    const uint4* xp[R];
    bool on[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      on[r] = c0 + r < n_items;
      const int it = on[r] ? c0 + r : c0;
      const int k = bin.k[it];
      wp[r] = reinterpret_cast<const uint4*>(p.packed[k] + (size_t)bin.crb[it] * n_tiles * 1024) + lane;
      xp[r] = reinterpret_cast<const uint4*>(p.qx + (SHARED_X ? (size_t)0 : (size_t)p.member_of[k] * p.qx_mstride)) + lane;
    }
    v4i acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = v4i{0, 0, 0, 0};

    for (int t = wave; t < n_tiles; t += NW) {
      uint4 w[R];
#pragma unroll
      for (int r = 0; r < R; ++r)
        if (on[r]) w[r] = wp[r][(size_t)t * 64];
      if (SHARED_X) {
        uint4 x[STEPS];
#pragma unroll
        for (int j = 0; j < STEPS; ++j) x[j] = xp[0][(size_t)(t * STEPS + j) * 64];
#pragma unroll
        for (int j = 0; j < STEPS; ++j) {
          const v4i xf = v4i{(int)x[j].x, (int)x[j].y, (int)x[j].z, (int)x[j].w};
#pragma unroll
          for (int r = 0; r < R; ++r) {
            if (!on[r]) continue;
            v4i wf;
            unpack_step<BITS>(w[r], j, wf);
            acc[r] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf, xf, acc[r], 0, 0, 0);
          }
        }
      } else {
#pragma unroll
        for (int r = 0; r < R; ++r) {
          if (!on[r]) continue;
#pragma unroll
          for (int j = 0; j < STEPS; ++j) {
            const uint4 x = xp[r][(size_t)(t * STEPS + j) * 64];
            const v4i xf = v4i{(int)x.x, (int)x.y, (int)x.z, (int)x.w};
            v4i wf;
            unpack_step<BITS>(w[r], j, wf);
            acc[r] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf, xf, acc[r], 0, 0, 0);
          }
        }
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if (!on[r]) continue;
#pragma unroll
      for (int i = 0; i < 4; ++i) atomicAdd(&fin[c0 + r][lane * 4 + i], acc[r][i]);
    }
  }
  __syncthreads();

  // epilogue: 256 threads per output row block, thread = (token t, channel ch)
  const int e = threadIdx.x & 255;
  const int t = e >> 4, ch = e & 15;
  const int fidx = ((ch >> 2) * 16 + t) * 4 + (ch & 3);   // lane*4 + i of the MFMA result layout
  for (int o = threadIdx.x >> 8; o < bin.n_out; o += (NW * 64) / 256) {
    const int orb = bin.out_rb[o];
    const int col = orb * 16 + ch;
    // Evaluation order (same as the tiled kernel): one member, or members kept apart:
    // y_m = s_x,m * (sum_k s_k * a_k) + b;  members summed: y = sum_m sum_k (s_k * s_x,m) * a_k + b.
    const bool fold_sx = p.reduce && p.M > 1;
    float yacc = 0.f;
    for (int m = 0; m < p.M; ++m) {
      const int rs = OFF ? p.rowsum[(size_t)m * p.rowsum_mstride + t] : 0;
      const float sx = p.s_x[m * p.sx_mstride];
      for (int it = 0; it < n_items; ++it) {      // items of a row block are stored in ascending order k
        const int k = bin.k[it];
        if (bin.slot[it] != o || k < p.member_lo[m] || k > p.member_hi[m]) continue;
        const int a = fin[it][fidx] - OFF * rs;
        float sc = p.scales[k][(size_t)bin.crb[it] * 16 + ch];
        if (fold_sx) sc *= sx;
        yacc = fmaf(sc, (float)a, yacc);
        if (ACC_OUT) {
          if (t < p.T) p.acc_out[((size_t)k * p.T + t) * p.out + col] = a;
        }
      }
      if (ACC_OUT) continue;
      if (fold_sx && m + 1 < p.M) continue;
      float v = (fold_sx ? yacc : sx * yacc) + (((m == 0 || fold_sx) && p.bias != nullptr) ? p.bias[col] : 0.f);
      yacc = 0.f;
      if (p.act == PIPE_ACT_GELU) v = gelu_erf(v);
      if (p.amax_out != nullptr) {
        float mx = t < p.T ? fabsf(v) : 0.f;
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) mx = fmaxf(mx, __shfl_xor(mx, s, 64));
        if (lane == 0) atomicMax(&p.amax_out[m], __float_as_uint(mx));
      }
      if (t < p.T) p.y[((size_t)(p.reduce ? 0 : m) * p.T + t) * p.out + col] = v;
    }
  }
}

template <int BITS, int NW>
int launch_nw(const StreamParams& p, int n_bins, bool shared_x, bool acc_out, hipStream_t st) {
  const dim3 grid((unsigned)n_bins), blk(NW * 64);
  if (acc_out) {
    if (shared_x) hipLaunchKernelGGL((gemm_stream_kernel<BITS, NW, true, true>), grid, blk, 0, st, p);
    else hipLaunchKernelGGL((gemm_stream_kernel<BITS, NW, false, true>), grid, blk, 0, st, p);
  } else {
    if (shared_x) hipLaunchKernelGGL((gemm_stream_kernel<BITS, NW, true, false>), grid, blk, 0, st, p);
    else hipLaunchKernelGGL((gemm_stream_kernel<BITS, NW, false, false>), grid, blk, 0, st, p);
  }
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

}  // namespace

int launch_gemm_stream(const GemmArgs& a, hipStream_t st) {
  const pipe_expansion* e = a.e;
  if (a.T <= 0) return PIPE_OK;
  if (a.T > 16 || a.T_pad != 16) return PIPE_ESHAPE;
  StreamParams p;
  p.qx = a.qx; p.qx_mstride = a.qx_mstride;
  p.rowsum = a.rowsum; p.rowsum_mstride = a.rowsum_mstride;
  p.s_x = a.s_x; p.sx_mstride = a.sx_mstride;
  for (int k = 0; k < PIPE_MAX_K; ++k) {
    p.packed[k] = k < e->K ? e->orders[k].packed_dev : nullptr;
    p.scales[k] = k < e->K ? e->orders[k].scales_dev : nullptr;
  }
  p.bins = e->bins_dev;
  p.bias = a.bias; p.y = a.y; p.acc_out = a.acc_out; p.amax_out = a.amax_out;
  p.T = a.T; p.out = e->out; p.K = e->K; p.nks = e->nks; p.M = a.M; p.reduce = a.reduce; p.act = a.act;
  for (int m = 0; m < PIPE_MAX_K; ++m) { p.member_lo[m] = a.member_lo[m]; p.member_hi[m] = a.member_hi[m]; p.member_of[m] = 0; }
  for (int m = 0; m < a.M; ++m)
    for (int k = a.member_lo[m]; k <= a.member_hi[m]; ++k) p.member_of[k] = m;
  const bool shared_x = a.qx_mstride == 0;
  const bool acc_out = a.acc_out != nullptr;
  switch (e->bits) {
    case 8: return launch_nw<8, 8>(p, e->n_bins, shared_x, acc_out, st);
    case 4: return launch_nw<4, 8>(p, e->n_bins, shared_x, acc_out, st);
    default: return launch_nw<2, 8>(p, e->n_bins, shared_x, acc_out, st);
  }
}
