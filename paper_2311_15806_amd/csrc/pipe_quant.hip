// Activation quantization (App. B, Eq. (define_dre): Q(x) with a per-tensor scale lambda_x):
// absmax reduction, fp32 -> int8 into the fragment layout with per-token code sums, the
// im2col variant for convolutions, and the element-wise hidden activation of the MLP call.
//
// Q(x) = clamp(rint(x / s_x), -127, 127) with an IEEE fp32 division and round-half-to-even;
// this file is compiled with floating-point contraction off.
#include "pipe_internal.h"

#include <algorithm>

namespace {

constexpr int BLK = 256;

__global__ void zero_u32_kernel(uint32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

__device__ __forceinline__ float block_max(float v) {
  __shared__ float sm[BLK / 64];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = sm[0];
#pragma unroll
  for (int i = 1; i < BLK / 64; ++i) r = fmaxf(r, sm[i]);
  __syncthreads();
  return r;
}

// max|x| over n elements; the maximum is order independent, so the result is exact.
// Also clears the per-token code sums the quantizer that follows accumulates into.
__global__ __launch_bounds__(BLK) void absmax_kernel(const float* __restrict__ x, int64_t n,
                                                     uint32_t* __restrict__ amax_bits,
                                                     int32_t* __restrict__ zero_me, int n_zero) {
  for (int i = blockIdx.x * BLK + threadIdx.x; i < n_zero; i += gridDim.x * BLK) zero_me[i] = 0;
  float m = 0.f;
  const int64_t stride = (int64_t)gridDim.x * BLK;
  const int64_t i0 = (int64_t)blockIdx.x * BLK + threadIdx.x;
  if ((reinterpret_cast<uintptr_t>(x) & 15) == 0) {
    const int64_t n4 = n >> 2;
    const float4* x4 = reinterpret_cast<const float4*>(x);
    int64_t i = i0;
    for (; i + 7 * stride < n4; i += 8 * stride) {   // eight independent 16-byte loads in flight
      float4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = x4[i + u * stride];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        m = fmaxf(m, fmaxf(fmaxf(fabsf(v[u].x), fabsf(v[u].y)), fmaxf(fabsf(v[u].z), fabsf(v[u].w))));
    }
    for (; i < n4; i += stride) {
      const float4 v = x4[i];
      m = fmaxf(m, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
    }
    for (int64_t i = (n4 << 2) + i0; i < n; i += stride) m = fmaxf(m, fabsf(x[i]));
  } else {
    for (int64_t i = i0; i < n; i += stride) m = fmaxf(m, fabsf(x[i]));
  }
  m = block_max(m);
  if (threadIdx.x == 0) amax_raise(amax_bits, m);
}

// Largest activation code 2^(a-1)-1: 127 for int8 activations, 31 / 7 for 6 / 4 bits (the codes
// still travel as bytes).  Set by pipe_set_activation_bits through set_act_qmax below.
__constant__ float c_act_qmax = 127.f;

__device__ __forceinline__ float act_scale(float s_static, const uint32_t* amax_bits) {
  if (s_static > 0.f) return s_static;
  return __fdiv_rn(__uint_as_float(*amax_bits), c_act_qmax);
}

__device__ __forceinline__ int quant1(float v, float s) {
  float q = rintf(__fdiv_rn(v, s));
  q = fminf(fmaxf(q, -c_act_qmax), c_act_qmax);
  return (int)q;
}

__device__ __forceinline__ uint32_t pack4(int a, int b, int c, int d) {
  return (uint32_t)(uint8_t)a | ((uint32_t)(uint8_t)b << 8) | ((uint32_t)(uint8_t)c << 16) |
         ((uint32_t)(uint8_t)d << 24);
}

// One block: token block blockIdx.x (16 tokens), a range of 16-wide k-chunks given by
// blockIdx.y (whole 64-k steps).  FETCH(t, k) returns the fp32 activation (0 outside the valid
// region).  Rows that can be read 16 bytes at a time (xvec) take the wide path for every 64-k step
// that lies inside the row: a wave owns 16 tokens x 64 k, lane = (token lane >> 2, quarter
// lane & 3), so one load instruction reads 64 contiguous bytes of each of the 16 rows (and the
// four loads of a step 256 contiguous bytes per row) and one store instruction writes 256
// contiguous bytes of the fragment layout.  Everything else (ragged tail, padding, gathers) goes
// through the generic path: thread = (token tid & 15, chunk slot tid >> 4).
template <class Fetch>
__device__ __forceinline__ void quantize_block(Fetch fetch, int T, int in, int in_pad, float s,
                                               uint8_t* __restrict__ qx_frag, int32_t* __restrict__ rowsum,
                                               int8_t* __restrict__ qx_rowmajor, const float* __restrict__ xvec = nullptr) {
  const int tb = blockIdx.x;
  const int nks = in_pad >> 6;
  const int nchunk = in_pad >> 4;
  const int per = ((nchunk + (int)gridDim.y - 1) / (int)gridDim.y + 3) & ~3;
  const int c_lo = min(nchunk, (int)blockIdx.y * per);
  const int c_hi = min(nchunk, c_lo + per);
  const bool live = s > 0.f;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int NWAVE = BLK / 64;

  // wide path
  int c_wide = c_lo;
  int sum_w = 0;
  if (xvec != nullptr && qx_rowmajor == nullptr) {
    c_wide = max(c_lo, min(c_hi, (in >> 6) << 2));
    const int nw = lane >> 2, sub = lane & 3;
    const int tw = tb * 16 + nw;
    const bool row_ok = live && tw < T;
    const float* row = xvec + (size_t)min(tw, T - 1) * in + sub * 4;
    uint8_t* dst = qx_frag + (size_t)tb * nks * 1024 + lane * 4;
    auto load_step = [&](int ks, float4(&f)[4]) {
#pragma unroll
      for (int e = 0; e < 4; ++e) f[e] = *reinterpret_cast<const float4*>(row + ks * 64 + e * 16);
    };
    auto put_step = [&](int ks, const float4(&f)[4]) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        int q0 = 0, q1 = 0, q2 = 0, q3 = 0;
        if (row_ok) {
          q0 = quant1(f[e].x, s); q1 = quant1(f[e].y, s); q2 = quant1(f[e].z, s); q3 = quant1(f[e].w, s);
        }
        sum_w += q0 + q1 + q2 + q3;
        *reinterpret_cast<uint32_t*>(dst + (size_t)ks * 1024 + e * 256) = pack4(q0, q1, q2, q3);
      }
    };
    const int ks_hi = c_wide >> 2;
    int ks = (c_lo >> 2) + wave;
    for (; ks + NWAVE < ks_hi; ks += 2 * NWAVE) {   // two steps = eight 16-byte loads in flight
      float4 f0[4], f1[4];
      load_step(ks, f0);
      load_step(ks + NWAVE, f1);
      put_step(ks, f0);
      put_step(ks + NWAVE, f1);
    }
    for (; ks < ks_hi; ks += NWAVE) {
      float4 f0[4];
      load_step(ks, f0);
      put_step(ks, f0);
    }
  }

  // generic path
  const int n = threadIdx.x & 15;
  const int t = tb * 16 + n;
  int sum = 0;
  for (int c = c_wide + (threadIdx.x >> 4); c < c_hi; c += BLK / 16) {
    int q[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int k = c * 16 + e;
      int v = 0;
      if (live && t < T && k < in) v = quant1(fetch(t, k), s);
      q[e] = v;
      sum += v;
    }
    const int ks = c >> 2, kc = c & 3;
    uint4 w = make_uint4(pack4(q[0], q[1], q[2], q[3]), pack4(q[4], q[5], q[6], q[7]),
                         pack4(q[8], q[9], q[10], q[11]), pack4(q[12], q[13], q[14], q[15]));
    *reinterpret_cast<uint4*>(qx_frag + (((size_t)tb * nks + ks) * 64 + kc * 16 + n) * 16) = w;
    if (qx_rowmajor != nullptr && t < T) {
#pragma unroll
      for (int e = 0; e < 16; ++e)
        if (c * 16 + e < in) qx_rowmajor[(size_t)t * in + c * 16 + e] = (int8_t)q[e];
    }
  }
  // one atomic per token and workgroup.  Generic path: threads 16 apart hold the same token
  // (lane bits 4 and 5); wide path: the four lanes of a quarter group; then the waves through LDS.
  sum += __shfl_xor(sum, 16, 64);
  sum += __shfl_xor(sum, 32, 64);
  sum_w += __shfl_xor(sum_w, 1, 64);
  sum_w += __shfl_xor(sum_w, 2, 64);
  __shared__ int wsum[2][NWAVE][16];
  if (lane < 16) wsum[0][wave][lane] = sum;
  if ((lane & 3) == 0) wsum[1][wave][lane >> 2] = sum_w;
  __syncthreads();
  if (threadIdx.x < 16) {
    int tot = 0;
#pragma unroll
    for (int w = 0; w < NWAVE; ++w) tot += wsum[0][w][threadIdx.x] + wsum[1][w][threadIdx.x];
    if (t < T && tot != 0) atomicAdd(&rowsum[t], tot);
  }
}

// blockIdx.z = ensemble member: member m reads x + m*x_mstride with the scale slot m, and writes
// its own fragment buffer, code sums and scale.
__global__ __launch_bounds__(BLK) void quantize_act_kernel(const float* __restrict__ x_all, int64_t x_mstride, int T, int in,
                                                           int in_pad, float s_static,
                                                           const uint32_t* __restrict__ amax_bits,
                                                           uint8_t* __restrict__ qx_all, int64_t qx_mstride,
                                                           int32_t* __restrict__ rowsum_all, int rowsum_mstride,
                                                           int8_t* __restrict__ qx_rowmajor,
                                                           float* __restrict__ scale_out) {
  const int m = blockIdx.z;
  const float* x = x_all + (size_t)m * x_mstride;
  const float s = act_scale(s_static, amax_bits + m);
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0 && scale_out) scale_out[m] = s;
  auto fetch = [=](int t, int k) { return x[(size_t)t * in + k]; };
  const bool vec = (in & 3) == 0 && (reinterpret_cast<uintptr_t>(x) & 15) == 0;
  quantize_block(fetch, T, in, in_pad, s, qx_all + (size_t)m * qx_mstride, rowsum_all + (size_t)m * rowsum_mstride,
                 qx_rowmajor, vec ? x : nullptr);
}

// Decode-sized batches (up to 64 tokens): ONE launch does max|x|, scale, codes and code sums, so the
// forward path is two launches (this one and the contraction).  Workgroup (n, m) owns token n
// of member m: it first reduces max|x| over the member's whole input (every workgroup does,
// redundantly -- the input is a few hundred KiB and L2 resident, and it spares a grid-wide
// synchronization), then quantizes its own token and sums its codes without atomics.
constexpr int SBLK = 1024;   // a large workgroup: the scan for the maximum is the long part
__global__ __launch_bounds__(SBLK) void quantize_small_kernel(const float* __restrict__ x_all, int64_t x_mstride,
                                                              int T, int in, int in_pad, float s_static,
                                                              const uint32_t* __restrict__ amax_bits,
                                                              uint8_t* __restrict__ qx_all, int64_t qx_mstride,
                                                              int32_t* __restrict__ rowsum_all,
                                                              int8_t* __restrict__ qx_rowmajor,
                                                              float* __restrict__ scale_out) {
  const int n = blockIdx.x;      // token 0..T_pad-1 (T_pad = gridDim.x, a multiple of 16)
  const int nks = in_pad >> 6;
  const int m = blockIdx.y;
  const float* x = x_all + (size_t)m * x_mstride;
  uint8_t* qx_frag = qx_all + (size_t)m * qx_mstride;
  __shared__ float smax[SBLK / 64];
  __shared__ int ssum[SBLK / 64];
  float s = s_static;
  if (!(s_static > 0.f) && amax_bits != nullptr) {
    // the producer of x already reduced max|x| of member m
    s = __fdiv_rn(__uint_as_float(amax_bits[m]), c_act_qmax);
  } else if (!(s_static > 0.f)) {
    float mx = 0.f;
    const int64_t cnt = (int64_t)T * in;
    if ((reinterpret_cast<uintptr_t>(x) & 15) == 0) {
      const float4* x4 = reinterpret_cast<const float4*>(x);
      const int64_t n4 = cnt >> 2;
      int64_t i = threadIdx.x;
      for (; i + 7 * SBLK < n4; i += 8 * SBLK) {   // eight independent 16-byte loads in flight
        float4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = x4[i + u * SBLK];
#pragma unroll
        for (int u = 0; u < 8; ++u)
          mx = fmaxf(mx, fmaxf(fmaxf(fabsf(v[u].x), fabsf(v[u].y)), fmaxf(fabsf(v[u].z), fabsf(v[u].w))));
      }
      for (; i < n4; i += SBLK) {
        const float4 v = x4[i];
        mx = fmaxf(mx, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
      }
      for (int64_t j = (n4 << 2) + threadIdx.x; j < cnt; j += SBLK) mx = fmaxf(mx, fabsf(x[j]));
    } else {
      for (int64_t j = threadIdx.x; j < cnt; j += SBLK) mx = fmaxf(mx, fabsf(x[j]));
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    if ((threadIdx.x & 63) == 0) smax[threadIdx.x >> 6] = mx;
    __syncthreads();
    mx = smax[0];
#pragma unroll
    for (int i = 1; i < SBLK / 64; ++i) mx = fmaxf(mx, smax[i]);
    s = __fdiv_rn(mx, c_act_qmax);
  }
  if (n == 0 && threadIdx.x == 0 && scale_out) scale_out[m] = s;
  const bool live = s > 0.f && n < T;
  const int nchunk = in_pad >> 4;
  const bool vec = (in & 3) == 0 && (reinterpret_cast<uintptr_t>(x) & 15) == 0;
  int sum = 0;
  for (int c = threadIdx.x; c < nchunk; c += SBLK) {
    int q[16];
    if (live && vec && c * 16 + 15 < in) {
      const float4* row = reinterpret_cast<const float4*>(x + (size_t)n * in + c * 16);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float4 v = row[e];
        q[4 * e] = quant1(v.x, s); q[4 * e + 1] = quant1(v.y, s); q[4 * e + 2] = quant1(v.z, s); q[4 * e + 3] = quant1(v.w, s);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 16; ++e) q[e] = (live && c * 16 + e < in) ? quant1(x[(size_t)n * in + c * 16 + e], s) : 0;
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) sum += q[e];
    const int ks = c >> 2, kc = c & 3;
    const uint4 w = make_uint4(pack4(q[0], q[1], q[2], q[3]), pack4(q[4], q[5], q[6], q[7]),
                               pack4(q[8], q[9], q[10], q[11]), pack4(q[12], q[13], q[14], q[15]));
    *reinterpret_cast<uint4*>(qx_frag + (((size_t)(n >> 4) * nks + ks) * 64 + kc * 16 + (n & 15)) * 16) = w;
    if (qx_rowmajor != nullptr && n < T) {
#pragma unroll
      for (int e = 0; e < 16; ++e)
        if (c * 16 + e < in) qx_rowmajor[(size_t)n * in + c * 16 + e] = (int8_t)q[e];
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
  if ((threadIdx.x & 63) == 0) ssum[threadIdx.x >> 6] = sum;
  __syncthreads();
  if (threadIdx.x == 0) {
    int tot = 0;
#pragma unroll
    for (int i = 0; i < SBLK / 64; ++i) tot += ssum[i];
    rowsum_all[(size_t)m * gridDim.x + n] = tot;
  }
}

struct ConvGeom {
  int N, C, H, W, kh, kw, stride, pad, nhwc, Ho, Wo;
};

// Convolution input, step 1: every input element is quantized once, in the input's own layout
// (an element appears in up to kh*kw patches; the IEEE division is paid once, not per patch).
__global__ __launch_bounds__(BLK) void quantize_elem_kernel(const float* __restrict__ x, int64_t n, float s_static,
                                                            const uint32_t* __restrict__ amax_bits,
                                                            int8_t* __restrict__ q8, float* __restrict__ scale_out,
                                                            int32_t* __restrict__ zero_me, int n_zero) {
  // also clears the token code sums the gather that follows adds into
  for (int i = blockIdx.x * BLK + threadIdx.x; i < n_zero; i += gridDim.x * BLK) zero_me[i] = 0;
  const float s = act_scale(s_static, amax_bits);
  if (blockIdx.x == 0 && threadIdx.x == 0 && scale_out) *scale_out = s;
  const bool live = s > 0.f;
  for (int64_t i = (int64_t)blockIdx.x * BLK + threadIdx.x; i < n; i += (int64_t)gridDim.x * BLK)
    q8[i] = live ? (int8_t)quant1(x[i], s) : (int8_t)0;
}

// Step 2: patches of codes -> fragment layout and token code sums.  Token t = (n, ho, wo); column
// k = (c, r, q) as in a weight row flattened [C, kh, kw].  A thread owns 16 consecutive k of one
// token; (c, r, q) is split once per chunk and then stepped, not divided, element by element.
// pad_neg: nullptr (taps outside the image read code 0), or a device word whose negation is the code
// of the real value 0 (asymmetric codes: the zero point minus 2^(a-1)).
__global__ __launch_bounds__(BLK) void im2col_codes_kernel(const int8_t* __restrict__ q8, ConvGeom g, int T, int in,
                                                           int in_pad, uint8_t* __restrict__ qx_frag,
                                                           int32_t* __restrict__ rowsum, const int32_t* __restrict__ pad_neg) {
  const int padv = pad_neg != nullptr ? -pad_neg[0] : 0;
  const int tb = blockIdx.x;
  const int n16 = threadIdx.x & 15;
  const int t = tb * 16 + n16;
  const int nks = in_pad >> 6;
  const int nchunk = in_pad >> 4;
  const int per = (nchunk + gridDim.y - 1) / gridDim.y;
  const int c_lo = blockIdx.y * per;
  const int c_hi = min(nchunk, c_lo + per);
  const bool tok = t < T;
  const int wo = tok ? t % g.Wo : 0, ho = tok ? (t / g.Wo) % g.Ho : 0, nimg = tok ? t / (g.Wo * g.Ho) : 0;
  const int hi0 = ho * g.stride - g.pad, wi0 = wo * g.stride - g.pad;
  // offset = base_n + c * step_c + h * step_r + w * step_q in either layout
  const int step_q = g.nhwc ? g.C : 1, step_r = g.nhwc ? g.W * g.C : g.W, step_c = g.nhwc ? 1 : g.H * g.W;
  const int base_n = nimg * g.C * g.H * g.W;
  int sum = 0;
  for (int c = c_lo + (threadIdx.x >> 4); c < c_hi; c += BLK / 16) {
    int k = c * 16;
    int qq = k % g.kw, rr = (k / g.kw) % g.kh, cc = k / (g.kw * g.kh);
    // The element offset is stepped, not recomputed (32-bit: the input has fewer than 2^31 elements), and
    // all 16 byte loads are issued before the first one is used: offsets of taps that are not read are
    // clamped to element 0 and the value is replaced afterwards.
    int off = base_n + cc * step_c + (hi0 + rr) * step_r + (wi0 + qq) * step_q;
    int q[16];
    int offs[16];
    int kind[16];   // 0: code 0 (beyond the row or the batch), 1: read, 2: outside the image
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int hi = hi0 + rr, wi = wi0 + qq;
      const bool inside = hi >= 0 && hi < g.H && wi >= 0 && wi < g.W;
      kind[e] = (tok && k < in) ? (inside ? 1 : 2) : 0;
      offs[e] = kind[e] == 1 ? off : 0;
      ++k;
      off += step_q;
      if (++qq == g.kw) {
        qq = 0;
        off += step_r - g.kw * step_q;
        if (++rr == g.kh) { rr = 0; ++cc; off += step_c - g.kh * step_r; }
      }
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) q[e] = q8[offs[e]];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      q[e] = kind[e] == 1 ? q[e] : (kind[e] == 2 ? padv : 0);
      sum += q[e];
    }
    const int ks = c >> 2, kc = c & 3;
    const uint4 w = make_uint4(pack4(q[0], q[1], q[2], q[3]), pack4(q[4], q[5], q[6], q[7]),
                               pack4(q[8], q[9], q[10], q[11]), pack4(q[12], q[13], q[14], q[15]));
    *reinterpret_cast<uint4*>(qx_frag + (((size_t)tb * nks + ks) * 64 + kc * 16 + n16) * 16) = w;
  }
  if (tok && sum != 0) atomicAdd(&rowsum[t], sum);
}

// h = act(y1) for every member, and max|h| per member (amax_neg set: max(h, 0) and max(-h, 0) apart, the range
// an asymmetric quantizer needs).
__global__ __launch_bounds__(BLK) void mlp_act_kernel(const float* __restrict__ y1, int T, int H, int act,
                                                      float* __restrict__ h, uint32_t* __restrict__ amax_bits,
                                                      uint32_t* __restrict__ amax_neg) {
  const int m = blockIdx.y;
  const int64_t n = (int64_t)T * H;
  const int O1 = act == PIPE_ACT_SILU_GATED ? 2 * H : H;
  const float* src = y1 + (size_t)m * T * O1;
  float* dst = h + (size_t)m * n;
  float mx = 0.f, mn = 0.f;
  const bool two_sided = amax_neg != nullptr;
  auto gelu1 = [](float a) { return 0.5f * a * (1.f + erff(a * 0.70710678118654752440f)); };
  auto gate1 = [](float gte, float up) { return gte / (1.f + expf(-gte)) * up; };
  auto take = [&](float v) { mx = fmaxf(mx, two_sided ? v : fabsf(v)); mn = fmaxf(mn, -v); };
  if ((H & 3) == 0 && ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) == 0) {
    // four neighbouring channels of a token per step: 16-byte loads and stores, 32-bit index arithmetic
    // (the host keeps T * H below 2^31), the same expression per element as below
    const int H4 = H >> 2, n4 = T * H4, O4 = O1 >> 2;
    const float4* s4 = reinterpret_cast<const float4*>(src);
    float4* d4 = reinterpret_cast<float4*>(dst);
    for (int i = blockIdx.x * BLK + threadIdx.x; i < n4; i += gridDim.x * BLK) {
      const int t = i / H4, c4 = i - t * H4;
      float4 v;
      if (act == PIPE_ACT_SILU_GATED) {
        const float4 g = s4[t * O4 + c4], u = s4[t * O4 + H4 + c4];
        v = make_float4(gate1(g.x, u.x), gate1(g.y, u.y), gate1(g.z, u.z), gate1(g.w, u.w));
      } else {
        const float4 a = s4[i];
        v = make_float4(gelu1(a.x), gelu1(a.y), gelu1(a.z), gelu1(a.w));
      }
      d4[i] = v;
      take(v.x); take(v.y); take(v.z); take(v.w);
    }
  } else {
    for (int64_t i = (int64_t)blockIdx.x * BLK + threadIdx.x; i < n; i += (int64_t)gridDim.x * BLK) {
      float v;
      if (act == PIPE_ACT_SILU_GATED) {
        const int64_t t = i / H;
        const int c = (int)(i - t * H);
        v = gate1(src[t * O1 + c], src[t * O1 + H + c]);
      } else {
        v = gelu1(src[i]);
      }
      dst[i] = v;
      take(v);
    }
  }
  mx = block_max(mx);
  if (threadIdx.x == 0) amax_raise(&amax_bits[m], mx);
  if (two_sided) {
    mn = block_max(mn);
    if (threadIdx.x == 0) amax_raise(&amax_neg[m], mn);
  }
}


// ---------------------------------------------------------------- asymmetric activation codes
// Sec. 4.3 compares under asymmetric quantization; the affine quantizer over [min(x,0), max(x,0)]:
//   s = (hi - lo) / (2^a - 1),  z = clamp(rint(-lo / s), 0, 2^a - 1),  Q(x) = clamp(rint(x / s) + z, 0, 2^a - 1).
// The contraction kernels multiply signed bytes, so the stored code is Q(x) - 2^(a-1); the exact
// accumulator is then acc' + (2^(a-1) - z) * (sum of the row's weight codes), a term without the
// token that the entry point folds into the bias.

// slots[0] = max(x, 0), slots[1] = max(-x, 0) (bit patterns; both order independent, hence exact)
__global__ __launch_bounds__(BLK) void minmax_kernel(const float* __restrict__ x, int64_t n, uint32_t* __restrict__ slots) {
  float hi = 0.f, nlo = 0.f;
  for (int64_t i = (int64_t)blockIdx.x * BLK + threadIdx.x; i < n; i += (int64_t)gridDim.x * BLK) {
    const float v = x[i];
    hi = fmaxf(hi, v);
    nlo = fmaxf(nlo, -v);
  }
  hi = block_max(hi);
  nlo = block_max(nlo);
  if (threadIdx.x == 0) {
    amax_raise(slots, hi);
    amax_raise(slots + 1, nlo);
  }
}

// thread = (token tid & 15, chunk slot tid >> 4) of token block blockIdx.x; blockIdx.y splits k.
// qa = 2^a - 1, shift = 2^(a-1).  Writes the fragment layout, adds the token code sums (zero on
// entry), optionally the unsigned codes row-major, and (block 0,0) the scale and shift - z.
__global__ __launch_bounds__(BLK) void quantize_asym_kernel(const float* __restrict__ x, int T, int in, int in_pad,
                                                            const uint32_t* __restrict__ hi_slot,
                                                            const uint32_t* __restrict__ nlo_slot, float qa, int shift,
                                                            uint8_t* __restrict__ qx_frag, int32_t* __restrict__ rowsum,
                                                            uint8_t* __restrict__ qx_rowmajor, float* __restrict__ scale_out,
                                                            int32_t* __restrict__ dz_out) {
  const float hi = __uint_as_float(hi_slot[0]), nlo = __uint_as_float(nlo_slot[0]);
  const float s = __fdiv_rn(__fadd_rn(hi, nlo), qa);
  const bool live = s > 0.f;
  const float zf = live ? fminf(fmaxf(rintf(__fdiv_rn(nlo, s)), 0.f), qa) : 0.f;
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
    scale_out[0] = s;
    dz_out[0] = live ? shift - (int)zf : 0;
  }
  const int tb = blockIdx.x;
  const int nks = in_pad >> 6, nchunk = in_pad >> 4;
  const int per = ((nchunk + (int)gridDim.y - 1) / (int)gridDim.y + 3) & ~3;
  const int c_lo = min(nchunk, (int)blockIdx.y * per), c_hi = min(nchunk, c_lo + per);
  const int n = threadIdx.x & 15, t = tb * 16 + n;
  int sum = 0;
  for (int c = c_lo + (threadIdx.x >> 4); c < c_hi; c += BLK / 16) {
    int q[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int k = c * 16 + e;
      int v = 0;
      if (live && t < T && k < in) {
        const float u = fminf(fmaxf(__fadd_rn(rintf(__fdiv_rn(x[(size_t)t * in + k], s)), zf), 0.f), qa);
        if (qx_rowmajor != nullptr) qx_rowmajor[(size_t)t * in + k] = (uint8_t)(int)u;
        v = (int)u - shift;
      } else if (qx_rowmajor != nullptr && t < T && k < in) {
        qx_rowmajor[(size_t)t * in + k] = 0;
      }
      q[e] = v;
      sum += v;
    }
    const int ks = c >> 2, kc = c & 3;
    uint4 w = make_uint4(pack4(q[0], q[1], q[2], q[3]), pack4(q[4], q[5], q[6], q[7]),
                         pack4(q[8], q[9], q[10], q[11]), pack4(q[12], q[13], q[14], q[15]));
    *reinterpret_cast<uint4*>(qx_frag + (((size_t)tb * nks + ks) * 64 + kc * 16 + n) * 16) = w;
  }
  sum += __shfl_xor(sum, 16, 64);
  sum += __shfl_xor(sum, 32, 64);
  __shared__ int wsum[BLK / 64][16];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane < 16) wsum[wave][lane] = sum;
  __syncthreads();
  if (threadIdx.x < 16) {
    int tot = 0;
#pragma unroll
    for (int w = 0; w < BLK / 64; ++w) tot += wsum[w][threadIdx.x];
    if (t < T && tot != 0) atomicAdd(&rowsum[t], tot);
  }
}

// every element of a tensor once, in its own layout (the convolution's first step): code minus shift
__global__ __launch_bounds__(BLK) void quantize_elem_asym_kernel(const float* __restrict__ x, int64_t n,
                                                                 const uint32_t* __restrict__ hi_slot,
                                                                 const uint32_t* __restrict__ nlo_slot, float qa, int shift,
                                                                 int8_t* __restrict__ q8, float* __restrict__ scale_out,
                                                                 int32_t* __restrict__ dz_out, int32_t* __restrict__ zero_me,
                                                                 int n_zero) {
  for (int i = blockIdx.x * BLK + threadIdx.x; i < n_zero; i += gridDim.x * BLK) zero_me[i] = 0;
  const float hi = __uint_as_float(hi_slot[0]), nlo = __uint_as_float(nlo_slot[0]);
  const float s = __fdiv_rn(__fadd_rn(hi, nlo), qa);
  const bool live = s > 0.f;
  const float zf = live ? fminf(fmaxf(rintf(__fdiv_rn(nlo, s)), 0.f), qa) : 0.f;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    scale_out[0] = s;
    dz_out[0] = live ? shift - (int)zf : 0;
  }
  for (int64_t i = (int64_t)blockIdx.x * BLK + threadIdx.x; i < n; i += (int64_t)gridDim.x * BLK) {
    int v = 0;
    if (live) v = (int)fminf(fmaxf(__fadd_rn(rintf(__fdiv_rn(x[i], s)), zf), 0.f), qa) - shift;
    q8[i] = (int8_t)v;
  }
}

// bias_eff[o] = b[o] + (s * dz) * C[o], C[o] = sum_k s_k[o] * (sum_i q_k[o,i]); also clears the
// two range slots for the next call
__global__ void asym_bias_kernel(const float* __restrict__ bias, const float* __restrict__ C, const float* __restrict__ scale,
                                 const int32_t* __restrict__ dz, float* __restrict__ out, int n, uint32_t* __restrict__ slots) {
  const int o = blockIdx.x * blockDim.x + threadIdx.x;
  if (o == 0) { slots[0] = 0u; slots[1] = 0u; }
  if (o >= n) return;
  const float f = scale[0] * (float)dz[0];
  out[o] = (bias != nullptr ? bias[o] : 0.f) + f * C[o];
}

// Members of a chain, each with its own scale and zero point: member m's offset vector is
// (s_m * dz_m) * sum_{k in member m, ascending} P[k][o], P[k][o] = s_k[o] * (sum_i q_k[o,i]); the layer's
// bias joins the first member.  reduce: one vector, the members' sum (ascending m) plus the bias.
__global__ void asym_bias_members_kernel(const float* __restrict__ bias, const float* __restrict__ P, const float* __restrict__ scale,
                                         int scale_stride, const int32_t* __restrict__ dz, int dz_stride, MemberRanges mr,
                                         int reduce, float* __restrict__ outv, int n, uint32_t* __restrict__ clear, int n_clear) {
  const int o = blockIdx.x * blockDim.x + threadIdx.x;
  if (o < n_clear) clear[o] = 0u;
  if (o >= n) return;
  float tot = bias != nullptr ? bias[o] : 0.f;
  for (int m = 0; m < mr.M; ++m) {
    float c = 0.f;
    for (int k = mr.lo[m]; k <= mr.hi[m]; ++k) c += P[(size_t)k * n + o];
    const float f = scale[m * scale_stride] * (float)dz[m * dz_stride];
    if (reduce) {
      tot = fmaf(f, c, tot);
    } else {
      outv[(size_t)m * n + o] = fmaf(f, c, m == 0 ? tot : 0.f);
    }
  }
  if (reduce) outv[o] = tot;
}

// exact accumulators of the debug export: acc[k][t][o] += dz * wsum[k][o]
__global__ void asym_acc_fix_kernel(int32_t* __restrict__ acc, const int32_t* __restrict__ wsum, const int32_t* __restrict__ dz,
                                    int K, int T, int out) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)K * T * out) return;
  const int o = (int)(i % out), k = (int)(i / ((int64_t)T * out));
  acc[i] += dz[0] * wsum[(size_t)k * out + o];
}

// sum of the codes of every stored row of one order -> wsum[o] (dense over output channels)
__global__ __launch_bounds__(BLK) void row_code_sums_kernel(const int8_t* __restrict__ codes, int in, int group,
                                                            const int32_t* __restrict__ gids, int32_t* __restrict__ wsum) {
  const int r = blockIdx.x, slot = r / group;
  const int o = gids[slot] * group + (r - slot * group);
  int s = 0;
  for (int i = threadIdx.x; i < in; i += BLK) s += codes[(size_t)r * in + i];
  __shared__ int sm[BLK];
  sm[threadIdx.x] = s;
  __syncthreads();
  for (int w = BLK / 2; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) sm[threadIdx.x] += sm[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) wsum[o] = sm[0];
}

// Convolution input for the implicit GEMM: channels-last int8 codes [N, H, W, C] and, per pixel,
// the sum of its C codes (added into csum, zero on entry).  NCHW input: 32 channels x 32 pixels per
// workgroup through LDS, so that reads run along the pixels and writes along the channels; NHWC input:
// element-wise, a group of 32 consecutive threads holds 32 consecutive channels of one pixel (C is a
// multiple of 64).
__global__ __launch_bounds__(BLK) void quantize_nhwc_sums_kernel(const float* __restrict__ x, int C, int HW, int nhwc,
                                                                 float s_static, const uint32_t* __restrict__ amax_bits,
                                                                 int8_t* __restrict__ q8, int32_t* __restrict__ csum,
                                                                 float* __restrict__ scale_out) {
  __shared__ int8_t tile[32][33];
  const float s = act_scale(s_static, amax_bits);
  if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x == 0 && scale_out) *scale_out = s;
  const bool live = s > 0.f;
  const int n = blockIdx.z, c0 = blockIdx.y * 32, p0 = blockIdx.x * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
  if (!nhwc) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int c = c0 + ty + 8 * j, pp = p0 + tx;
      int v = 0;
      if (c < C && pp < HW && live) v = quant1(x[((size_t)n * C + c) * HW + pp], s);
      tile[ty + 8 * j][tx] = (int8_t)v;
    }
    __syncthreads();
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int pp = p0 + ty + 8 * j, c = c0 + tx;
    int v = 0;
    if (c < C && pp < HW) {
      v = nhwc ? (live ? quant1(x[((size_t)n * HW + pp) * C + c], s) : 0) : (int)tile[tx][ty + 8 * j];
      q8[((size_t)n * HW + pp) * C + c] = (int8_t)v;
    }
    // the 32 threads of a half wave hold 32 channels of one pixel
    int sum = v;
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    if (tx == 0 && pp < HW && sum != 0) atomicAdd(&csum[(size_t)n * HW + pp], sum);
  }
}

}  // namespace

int launch_quantize_nhwc_sums(const float* x, int N, int C, int HW, int nhwc, float s_static, const uint32_t* amax_bits,
                              int8_t* q8, int32_t* csum, float* scale_out, hipStream_t st) {
  PIPE_KLAUNCH(quantize_nhwc_sums_kernel, dim3(ceil_div(HW, 32), ceil_div(C, 32), N), dim3(BLK), 0, st, x, C, HW, nhwc, s_static,
               amax_bits, q8, csum, scale_out);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

int set_act_qmax(float qmax) {
  PIPE_HIP(hipMemcpyToSymbol(HIP_SYMBOL(c_act_qmax), &qmax, sizeof(float)));
  return PIPE_OK;
}

int launch_zero_u32(uint32_t* p, int n, hipStream_t st) {
  if (n <= 0) return PIPE_OK;
  PIPE_KLAUNCH(zero_u32_kernel, dim3(ceil_div(n, 256)), dim3(256), 0, st, p, n);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

int launch_absmax(const float* x, int64_t n, uint32_t* amax_bits, int32_t* zero_me, int n_zero, hipStream_t st) {
  if (n <= 0) return PIPE_OK;
  int64_t blocks = (n / 4 + BLK - 1) / BLK;
  if (blocks < 1) blocks = 1;
  if (blocks > 256) blocks = 256;   // 1 per CU: every thread keeps 8 loads (128 B) in flight
  PIPE_KLAUNCH(absmax_kernel, dim3((unsigned)blocks), dim3(BLK), 0, st, x, n, amax_bits, zero_me, n_zero);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

static int ksplit_for(int T_pad, int in_pad) {
  // enough blocks to fill the chip when there are few token blocks
  const int tbs = T_pad / 16;
  int ks = 1;
  const int nchunk = in_pad / 16;
  while (tbs * ks < 1024 && ks * 2 * 16 <= nchunk) ks *= 2;
  return ks;
}

int launch_quantize_act(const float* x, int T, int in, int in_pad, int T_pad, float s_static,
                        const uint32_t* amax_bits, uint8_t* qx_frag, int32_t* rowsum, bool rowsum_is_zero,
                        int8_t* qx_rowmajor, float* scale_out, hipStream_t st) {
  if (!rowsum_is_zero) {
    int rc = launch_zero_u32(reinterpret_cast<uint32_t*>(rowsum), T_pad, st);
    if (rc) return rc;
  }
  dim3 grid(T_pad / 16, ksplit_for(T_pad, in_pad));
  PIPE_KLAUNCH(quantize_act_kernel, grid, dim3(BLK), 0, st, x, (int64_t)0, T, in, in_pad, s_static, amax_bits,
                     qx_frag, (int64_t)0, rowsum, 0, qx_rowmajor, scale_out);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

int launch_quantize_members(const float* x, int64_t x_mstride, int M, int T, int in, int in_pad, int T_pad,
                            const uint32_t* amax_bits, uint8_t* qx_frag, int64_t qx_mstride, int32_t* rowsum,
                            bool rowsum_is_zero, float* scale_out, hipStream_t st) {
  if (!rowsum_is_zero) {
    int rc = launch_zero_u32(reinterpret_cast<uint32_t*>(rowsum), M * T_pad, st);
    if (rc) return rc;
  }
  dim3 grid(T_pad / 16, ksplit_for(T_pad * M, in_pad), M);
  PIPE_KLAUNCH(quantize_act_kernel, grid, dim3(BLK), 0, st, x, x_mstride, T, in, in_pad, 0.f, amax_bits,
                     qx_frag, qx_mstride, rowsum, T_pad, (int8_t*)nullptr, scale_out);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

int launch_quantize_small(const float* x, int64_t x_mstride, int M, int T, int in, int in_pad, float s_static,
                          const uint32_t* amax_bits, uint8_t* qx_frag, int64_t qx_mstride, int32_t* rowsum,
                          int8_t* qx_rowmajor, float* scale_out, hipStream_t st) {
  PIPE_KLAUNCH(quantize_small_kernel, dim3((unsigned)round_up64(T, 16), M), dim3(SBLK), 0, st, x, x_mstride, T, in, in_pad, s_static,
                     amax_bits, qx_frag, qx_mstride, rowsum, qx_rowmajor, scale_out);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

int launch_quantize_elem(const float* x, int64_t n, float s_static, const uint32_t* amax_bits, int8_t* q8,
                         float* scale_out, hipStream_t st) {
  int64_t blocks = (n + BLK - 1) / BLK;
  if (blocks > 2048) blocks = 2048;
  if (blocks < 1) blocks = 1;
  PIPE_KLAUNCH(quantize_elem_kernel, dim3((unsigned)blocks), dim3(BLK), 0, st, x, n, s_static, amax_bits, q8, scale_out,
                     (int32_t*)nullptr, 0);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

int launch_quantize_im2col(const float* x, int N, int C, int H, int W, int kh, int kw, int stride,
                           int pad, int nhwc, int Ho, int Wo, int in_pad, int T_pad,
                           float s_static, const uint32_t* amax_bits, int8_t* q8_scratch, uint8_t* qx_frag,
                           int32_t* rowsum, float* scale_out, hipStream_t st) {
  const int64_t n = (int64_t)N * C * H * W;
  if (n >= ((int64_t)1 << 31)) return PIPE_ESHAPE;   // the gather steps 32-bit element offsets
  int64_t blocks = (n + BLK - 1) / BLK;
  if (blocks > 2048) blocks = 2048;
  if (blocks < 1) blocks = 1;
  PIPE_KLAUNCH(quantize_elem_kernel, dim3((unsigned)blocks), dim3(BLK), 0, st, x, n, s_static, amax_bits,
                     q8_scratch, scale_out, rowsum, T_pad);
  ConvGeom g{N, C, H, W, kh, kw, stride, pad, nhwc, Ho, Wo};
  const int T = N * Ho * Wo, in = C * kh * kw;
  dim3 grid(T_pad / 16, ksplit_for(T_pad, in_pad));
  PIPE_KLAUNCH(im2col_codes_kernel, grid, dim3(BLK), 0, st, q8_scratch, g, T, in, in_pad, qx_frag, rowsum,
                     (const int32_t*)nullptr);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

// the same with asymmetric codes: every element once (code minus 2^(a-1), scale and 2^(a-1) - z to device
// memory), then the patches, whose taps outside the image hold the code of the real value 0
int launch_quantize_im2col_asym(const float* x, int N, int C, int H, int W, int kh, int kw, int stride, int pad, int nhwc,
                                int Ho, int Wo, int in_pad, int T_pad, const uint32_t* hi_slot, const uint32_t* nlo_slot,
                                int act_bits, int8_t* q8_scratch, uint8_t* qx_frag, int32_t* rowsum, float* scale_out,
                                int32_t* dz_out, hipStream_t st) {
  const int64_t n = (int64_t)N * C * H * W;
  if (n >= ((int64_t)1 << 31)) return PIPE_ESHAPE;   // the gather steps 32-bit element offsets
  int64_t blocks = (n + BLK - 1) / BLK;
  if (blocks > 2048) blocks = 2048;
  if (blocks < 1) blocks = 1;
  PIPE_KLAUNCH(quantize_elem_asym_kernel, dim3((unsigned)blocks), dim3(BLK), 0, st, x, n, hi_slot, nlo_slot,
                     (float)((1 << act_bits) - 1), 1 << (act_bits - 1), q8_scratch, scale_out, dz_out, rowsum, T_pad);
  ConvGeom g{N, C, H, W, kh, kw, stride, pad, nhwc, Ho, Wo};
  const int T = N * Ho * Wo, in = C * kh * kw;
  dim3 grid(T_pad / 16, ksplit_for(T_pad, in_pad));
  PIPE_KLAUNCH(im2col_codes_kernel, grid, dim3(BLK), 0, st, q8_scratch, g, T, in, in_pad, qx_frag, rowsum,
                     (const int32_t*)dz_out);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

int launch_mlp_act(const float* y1, int M, int T, int H, int act, float* h, uint32_t* amax_bits, uint32_t* amax_neg,
                   hipStream_t st) {
  const int64_t n = (int64_t)T * H;
  if (n <= 0) return PIPE_OK;
  if (n >= ((int64_t)1 << 31)) return PIPE_ESHAPE;   // the kernel's fast path indexes with 32 bits
  int64_t blocks = (n + BLK * 4 - 1) / (BLK * 4);
  if (blocks > 4096) blocks = 4096;
  PIPE_KLAUNCH(mlp_act_kernel, dim3((unsigned)blocks, M), dim3(BLK), 0, st, y1, T, H, act, h, amax_bits, amax_neg);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

// ---- asymmetric activation codes (host side) ----------------------------------------------
int launch_minmax(const float* x, int64_t n, uint32_t* slots, hipStream_t st) {
  int64_t blocks = std::min<int64_t>((n + BLK - 1) / BLK, 2048);
  if (blocks < 1) blocks = 1;
  PIPE_KLAUNCH(minmax_kernel, dim3((unsigned)blocks), dim3(BLK), 0, st, x, n, slots);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

int launch_quantize_asym(const float* x, int T, int in, int in_pad, int T_pad, const uint32_t* hi_slot, const uint32_t* nlo_slot,
                         int act_bits, uint8_t* qx_frag, int32_t* rowsum, uint8_t* qx_rowmajor, float* scale_out, int32_t* dz_out,
                         hipStream_t st) {
  int rc = launch_zero_u32(reinterpret_cast<uint32_t*>(rowsum), T_pad, st);
  if (rc) return rc;
  dim3 grid(T_pad / 16, ksplit_for(T_pad, in_pad));
  PIPE_KLAUNCH(quantize_asym_kernel, grid, dim3(BLK), 0, st, x, T, in, in_pad, hi_slot, nlo_slot, (float)((1 << act_bits) - 1),
                     1 << (act_bits - 1), qx_frag, rowsum, qx_rowmajor, scale_out, dz_out);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

int launch_asym_bias(const float* bias, const float* C, const float* scale, const int32_t* dz, float* out, int n,
                     uint32_t* slots, hipStream_t st) {
  PIPE_KLAUNCH(asym_bias_kernel, dim3((n + 255) / 256), dim3(256), 0, st, bias, C, scale, dz, out, n, slots);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

int launch_asym_bias_members(const float* bias, const float* P, const float* scale, int scale_stride, const int32_t* dz,
                             int dz_stride, int M, const int* lo, const int* hi, int reduce, float* outv, int n, uint32_t* clear,
                             int n_clear, hipStream_t st) {
  MemberRanges mr{};
  mr.M = M;
  for (int m = 0; m < M; ++m) { mr.lo[m] = lo[m]; mr.hi[m] = hi[m]; }
  PIPE_KLAUNCH(asym_bias_members_kernel, dim3((std::max(n, n_clear) + 255) / 256), dim3(256), 0, st, bias, P, scale, scale_stride,
               dz, dz_stride, mr, reduce, outv, n, clear, n_clear);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

int launch_asym_acc_fix(int32_t* acc, const int32_t* wsum, const int32_t* dz, int K, int T, int out, hipStream_t st) {
  const int64_t n = (int64_t)K * T * out;
  if (n == 0) return PIPE_OK;
  PIPE_KLAUNCH(asym_acc_fix_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, acc, wsum, dz, K, T, out);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

int launch_row_code_sums(const int8_t* codes, int rows, int in, int group, const int32_t* gids, int32_t* wsum, hipStream_t st) {
  if (rows == 0) return PIPE_OK;
  PIPE_KLAUNCH(row_code_sums_kernel, dim3(rows), dim3(BLK), 0, st, codes, in, group, gids, wsum);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}
