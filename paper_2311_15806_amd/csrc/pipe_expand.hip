// Residual-expansion builder (Sec. 3.1, Eq. (2)-(3) and the masked form; quantizer: Sec. 3,
// Eq. (1)).  Row-parallel kernels: residual energy per row (fp64), top-gamma group selection,
// per-row quantization with in-place residual update and packing into the tile layout.
// Unstructured masks (Sec. 3.1: M^k a sparse tensor): the magnitude of the keep-th largest
// residual entry is found exactly by a three-level radix select over the entries' bit patterns,
// entries of that magnitude are kept in flat-index order up to a cut, and the row quantizer
// skips the entries the mask prunes.
//
// The integer codes depend on the fp32 arithmetic, so every operation that feeds a rounding
// decision is written with an explicitly rounded intrinsic (IEEE division, separate multiply
// and subtract) and this file is compiled with floating-point contraction off.
#include "pipe_internal.h"

#include <algorithm>
#include <vector>

namespace {

constexpr int BLK = 256;

// ---- residual energy of every row: sum_i E[o,i]^2 in fp64, fixed reduction tree ----------
__global__ __launch_bounds__(BLK) void row_energy_kernel(const float* __restrict__ E, int in,
                                                         double* __restrict__ out) {
  const int row = blockIdx.x;
  const float* p = E + (size_t)row * in;
  double s = 0.0;
  for (int i = threadIdx.x; i < in; i += BLK) {
    const double v = (double)p[i];
    s += v * v;  // the square of an fp32 value is exact in fp64
  }
  __shared__ double sm[BLK];
  sm[threadIdx.x] = s;
  __syncthreads();
  for (int o = BLK / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) sm[threadIdx.x] += sm[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[row] = sm[0];
}

// ---- group score = sum of its rows' energies, rows ascending ------------------------------
__global__ void group_score_kernel(const double* __restrict__ row_energy, int n_groups, int group,
                                   double* __restrict__ score) {
  const int g = blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= n_groups) return;
  double s = 0.0;
  for (int r = 0; r < group; ++r) s += row_energy[(size_t)g * group + r];
  score[g] = s;
}

// ---- keep flag: a group is kept if fewer than n_keep groups beat it (higher score, or equal
//      score and lower index) --------------------------------------------------------------
__global__ void group_rank_kernel(const double* __restrict__ score, int n_groups, int n_keep,
                                  int32_t* __restrict__ flag) {
  const int g = blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= n_groups) return;
  const double sg = score[g];
  int rank = 0;
  for (int j = 0; j < n_groups; ++j) {
    const double sj = score[j];
    rank += (sj > sg) || (sj == sg && j < g);
  }
  flag[g] = rank < n_keep ? 1 : 0;
}

// ---- compaction: kept groups in ascending order -------------------------------------------
__global__ void group_compact_kernel(const int32_t* __restrict__ flag, int n_groups,
                                     int32_t* __restrict__ gids) {
  const int g = blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= n_groups || !flag[g]) return;
  int idx = 0;
  for (int j = 0; j < g; ++j) idx += flag[j];
  gids[idx] = g;
}

// ---- unstructured mask: histogram of one digit of the magnitudes' bit patterns ------------
// key = bits of |e| (monotone in |e| for finite values); entries whose key >> prefix_shift equals
// prefix (all entries if prefix_shift is 32) are counted in bin (key >> shift) & (bins - 1).
constexpr int SEL_BINS = 2048;
__global__ __launch_bounds__(BLK) void key_histogram_kernel(const float* __restrict__ E, long long n, int shift, int bins,
                                                            int prefix_shift, uint32_t prefix, uint32_t* __restrict__ hist) {
  __shared__ uint32_t h[SEL_BINS];
  for (int i = threadIdx.x; i < bins; i += BLK) h[i] = 0u;
  __syncthreads();
  for (long long i = (long long)blockIdx.x * BLK + threadIdx.x; i < n; i += (long long)gridDim.x * BLK) {
    const uint32_t key = __float_as_uint(fabsf(E[i]));
    if (prefix_shift >= 32 || (key >> prefix_shift) == prefix) atomicAdd(&h[(key >> shift) & (uint32_t)(bins - 1)], 1u);
  }
  __syncthreads();
  for (int i = threadIdx.x; i < bins; i += BLK)
    if (h[i]) atomicAdd(&hist[i], h[i]);
}

// ---- entries of magnitude exactly thr_key with flat index <= cut ---------------------------
__global__ __launch_bounds__(BLK) void count_ties_kernel(const float* __restrict__ E, long long n, uint32_t thr_key,
                                                         long long cut, uint32_t* __restrict__ count) {
  uint32_t c = 0;
  const long long hi = cut + 1 < n ? cut + 1 : n;
  for (long long i = (long long)blockIdx.x * BLK + threadIdx.x; i < hi; i += (long long)gridDim.x * BLK)
    c += __float_as_uint(fabsf(E[i])) == thr_key;
  __shared__ uint32_t sm[BLK];
  sm[threadIdx.x] = c;
  __syncthreads();
  for (int s = BLK / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) sm[threadIdx.x] += sm[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0 && sm[0]) atomicAdd(count, sm[0]);
}

// ---- quantize one stored row, update its residual in place, pack its codes ----------------
// An entry takes part if its magnitude's bit pattern exceeds thr_key, or equals it with a flat
// index of at most tie_cut (thr_key = 0 with the largest tie_cut: every entry, the structured case).
template <int BITS>
__global__ __launch_bounds__(BLK) void quantize_rows_kernel(float* __restrict__ E, int in, int in_pad,
                                                            int group, const int32_t* __restrict__ gids,
                                                            float* __restrict__ scales,
                                                            uint8_t* __restrict__ packed, int QMAX,
                                                            const int8_t* __restrict__ given,
                                                            uint32_t thr_key, long long tie_cut) {
  // BITS is the width of the stored code (8, 4 or 2); QMAX = 2^(b-1)-1 of the quantizer, which
  // may be narrower (3-bit codes in 4-bit fields, 5..7-bit codes in bytes).  given: NULL, or the
  // codes [rows, in] another rounding operator chose for these rows (clamped here)
  constexpr int KSUP = 512 / BITS;       // k-values per tile
  constexpr int STEPS = KSUP / 64;       // 64-k steps per tile
  constexpr int OFF = BITS == 8 ? 0 : (BITS == 4 ? 8 : 1);
  const int r = blockIdx.x;              // stored (compact) row
  const int slot = r / group;
  const int o = gids[slot] * group + (r - slot * group);
  float* e = E + (size_t)o * in;
  const long long flat0 = (long long)o * in;
  auto kept = [&](float v, int k) {
    const uint32_t key = __float_as_uint(fabsf(v));
    return key > thr_key || (key == thr_key && flat0 + k <= tie_cut);
  };

  float amax = 0.f;
  for (int i = threadIdx.x; i < in; i += BLK) {
    const float v = e[i];
    amax = fmaxf(amax, kept(v, i) ? fabsf(v) : 0.f);
  }
  __shared__ float sm[BLK];
  sm[threadIdx.x] = amax;
  __syncthreads();
  for (int s = BLK / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) sm[threadIdx.x] = fmaxf(sm[threadIdx.x], sm[threadIdx.x + s]);
    __syncthreads();
  }
  amax = sm[0];
  const float s = __fdiv_rn(amax, (float)QMAX);
  const bool live = s > 0.f;
  if (threadIdx.x == 0) scales[r] = s;

  const int crb = r >> 4, rr = r & 15;
  const int nksup = in_pad / KSUP;
  const int nchunk = in_pad >> 4;
  for (int c = threadIdx.x; c < nchunk; c += BLK) {
    int code[16];
#pragma unroll
    for (int t = 0; t < 16; ++t) {
      const int k = c * 16 + t;
      int q = 0;
      if (live && k < in && kept(e[k], k)) {
        const float v = e[k];
        float qf = given != nullptr ? (float)given[(size_t)r * in + k]
                                    : rintf(__fdiv_rn(v, s));   // round half to even
        qf = fminf(fmaxf(qf, (float)-QMAX), (float)QMAX);
        e[k] = __fsub_rn(v, __fmul_rn(s, qf));             // Q^-1 then residual: two roundings
        q = (int)qf;
      }
      code[t] = q;
    }
    const int ks = c >> 2, kc = c & 3;
    const int ksup = ks / STEPS, j = ks - ksup * STEPS;
    const int lane = kc * 16 + rr;
    uint32_t* dst = reinterpret_cast<uint32_t*>(packed + ((size_t)crb * nksup + ksup) * 1024 + lane * 16);
    if (BITS == 8) {
      uint32_t w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        w[i] = (uint32_t)(uint8_t)code[4 * i] | ((uint32_t)(uint8_t)code[4 * i + 1] << 8) |
               ((uint32_t)(uint8_t)code[4 * i + 2] << 16) | ((uint32_t)(uint8_t)code[4 * i + 3] << 24);
      *reinterpret_cast<uint4*>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
    } else if (BITS == 4) {
      uint32_t w0 = 0, w1 = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const uint32_t v = (uint32_t)(code[4 * i + b] + OFF) << (8 * b + 4 * (i & 1));
          if (i < 2) w0 |= v; else w1 |= v;
        }
      dst[2 * j] = w0;
      dst[2 * j + 1] = w1;
    } else {
      uint32_t w = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int b = 0; b < 4; ++b) w |= (uint32_t)(code[4 * i + b] + OFF) << (8 * b + 2 * i);
      dst[j] = w;
    }
  }
}

// ---- operator hook: the rows an order quantizes, compact, with their scales ---------------
__global__ __launch_bounds__(BLK) void gather_rows_kernel(const float* __restrict__ E, int in, int group,
                                                          const int32_t* __restrict__ gids, int QMAX,
                                                          float* __restrict__ rows_out, float* __restrict__ scales_out) {
  const int r = blockIdx.x;
  const int slot = r / group;
  const float* e = E + (size_t)(gids[slot] * group + (r - slot * group)) * in;
  float amax = 0.f;
  for (int i = threadIdx.x; i < in; i += BLK) {
    const float v = e[i];
    rows_out[(size_t)r * in + i] = v;
    amax = fmaxf(amax, fabsf(v));
  }
  __shared__ float sm[BLK];
  sm[threadIdx.x] = amax;
  __syncthreads();
  for (int s = BLK / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) sm[threadIdx.x] = fmaxf(sm[threadIdx.x], sm[threadIdx.x + s]);
    __syncthreads();
  }
  if (threadIdx.x == 0) scales_out[r] = __fdiv_rn(sm[0], (float)QMAX);
}

// ---- introspection: tile layout -> one signed code per byte, [rows, in] -------------------
// rb_map (optional): stored position of compact row block crb inside `packed`.
__global__ void unpack_codes_kernel(const uint8_t* __restrict__ packed, const int32_t* __restrict__ rb_map, int bits,
                                    int rows, int in, int in_pad, int8_t* __restrict__ codes) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)rows * in) return;
  const int r = (int)(idx / in), k = (int)(idx - (int64_t)r * in);
  const int ksupw = 512 / bits, steps = ksupw / 64;
  const int crb = r >> 4, rr = r & 15;
  const int c = k >> 4, t = k & 15, ks = c >> 2, kc = c & 3;
  const int ksup = ks / steps, j = ks - ksup * steps;
  const int nksup = in_pad / ksupw;
  const int pos = rb_map ? rb_map[crb] : crb;
  const uint32_t* src = reinterpret_cast<const uint32_t*>(packed + ((size_t)pos * nksup + ksup) * 1024 +
                                                          (kc * 16 + rr) * 16);
  const int i = t >> 2, b = t & 3;
  int v;
  if (bits == 8) v = (int8_t)((src[i] >> (8 * b)) & 0xFF);
  else if (bits == 4) v = (int)((src[2 * j + (i >> 1)] >> (8 * b + 4 * (i & 1))) & 0xF) - 8;
  else v = (int)((src[j] >> (8 * b + 2 * i)) & 0x3) - 1;
  codes[idx] = (int8_t)v;
}

// ---- stored row blocks of one order -> their positions in the schedule-ordered buffers --------
// One workgroup per row block: rb_bytes of codes (16-byte units) and 16 row scales.
__global__ __launch_bounds__(256) void gather_row_blocks_kernel(const uint8_t* __restrict__ codes_k,
                                                                const float* __restrict__ scales_k,
                                                                const int32_t* __restrict__ pos_of, int64_t rb_bytes,
                                                                uint8_t* __restrict__ codes_all,
                                                                float* __restrict__ scales_all) {
  const int crb = blockIdx.x;
  const int64_t pos = pos_of[crb];
  const uint4* s = reinterpret_cast<const uint4*>(codes_k + (size_t)crb * rb_bytes);
  uint4* d = reinterpret_cast<uint4*>(codes_all + (size_t)pos * rb_bytes);
  for (int64_t i = threadIdx.x; i < rb_bytes / 16; i += 256) d[i] = s[i];
  if (threadIdx.x < 16) scales_all[pos * 16 + threadIdx.x] = scales_k[(size_t)crb * 16 + threadIdx.x];
}

// A convolution weight row flattened [C, kh, kw] -> flattened [kh, kw, C] (tap-major, channel-minor):
// the k axis the implicit-GEMM convolution walks (one tap's channels are contiguous in a channels-last input)
__global__ void permute_conv_weight_kernel(const float* __restrict__ W, int C, int taps, float* __restrict__ W_out) {
  const size_t row = blockIdx.x;
  const int in = C * taps;
  for (int i = threadIdx.x; i < in; i += blockDim.x) {
    const int tap = i / C, c = i - tap * C;
    W_out[row * in + i] = W[row * in + (size_t)c * taps + tap];
  }
}

}  // namespace

int launch_gather_row_blocks(const uint8_t* codes_k, const float* scales_k, const int32_t* pos_of_dev, int n_crb,
                             int64_t rb_bytes, uint8_t* codes_all, float* scales_all, hipStream_t st) {
  if (n_crb <= 0) return PIPE_OK;
  PIPE_KLAUNCH(gather_row_blocks_kernel, dim3((unsigned)n_crb), dim3(256), 0, st, codes_k, scales_k, pos_of_dev,
                     rb_bytes, codes_all, scales_all);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

int launch_row_energy(const float* E, int out, int in, double* row_energy, hipStream_t st) {
  PIPE_KLAUNCH(row_energy_kernel, dim3(out), dim3(BLK), 0, st, E, in, row_energy);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

// row_energy holds [out] doubles followed by scratch for [n_groups] scores (doubles) and
// [n_groups] flags (int32); the caller sizes it with out + n_groups doubles + n_groups ints.
int launch_group_select(const double* row_energy, int n_groups, int group, int n_keep,
                        int32_t* gids_out, hipStream_t st) {
  double* score = const_cast<double*>(row_energy) + (size_t)n_groups * group;
  int32_t* flag = reinterpret_cast<int32_t*>(score + n_groups);
  const int g = ceil_div(n_groups, 128);
  PIPE_KLAUNCH(group_score_kernel, dim3(g), dim3(128), 0, st, row_energy, n_groups, group, score);
  PIPE_KLAUNCH(group_rank_kernel, dim3(g), dim3(128), 0, st, score, n_groups, n_keep, flag);
  PIPE_KLAUNCH(group_compact_kernel, dim3(g), dim3(128), 0, st, flag, n_groups, gids_out);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

// Sec. 4.1: y = BN(W x + b) as one affine layer (the folded weight is what gets quantized, so
// every rounding is fixed): g = gamma / sqrt(var + eps) in fp64 rounded once to fp32, then
// W' = W * g, b' = (b - mean) * g + beta in explicitly rounded fp32.
__global__ __launch_bounds__(BLK) void fold_batchnorm_kernel(const float* __restrict__ W, const float* __restrict__ b,
                                                             const float* __restrict__ gamma, const float* __restrict__ beta,
                                                             const float* __restrict__ mean, const float* __restrict__ var,
                                                             float eps, int in, float* __restrict__ W_out,
                                                             float* __restrict__ b_out) {
  const int o = blockIdx.x;
  // the scale in fp64, rounded once (fp32 sqrt is not correctly rounded on this target)
  const float g = (float)((double)gamma[o] / sqrt((double)var[o] + (double)eps));
  for (int i = threadIdx.x; i < in; i += BLK) W_out[(size_t)o * in + i] = __fmul_rn(W[(size_t)o * in + i], g);
  if (threadIdx.x == 0 && b_out != nullptr)
    b_out[o] = __fadd_rn(__fmul_rn(__fsub_rn(b != nullptr ? b[o] : 0.f, mean[o]), g), beta[o]);
}

int launch_fold_batchnorm(const float* W, const float* b, const float* gamma, const float* beta, const float* mean,
                          const float* var, float eps, int out, int in, float* W_out, float* b_out, hipStream_t st) {
  PIPE_KLAUNCH(fold_batchnorm_kernel, dim3(out), dim3(BLK), 0, st, W, b, gamma, beta, mean, var, eps, in, W_out, b_out);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

// The keep-th largest magnitude of the n entries of E and the cut among the entries that share
// it: *thr_key = its bit pattern, *tie_cut = the flat index up to which entries of exactly that
// magnitude are kept (ties go to the lower flat index).  hist_dev: SEL_BINS + 1 words of scratch.
// Synchronizes the stream several times (an offline step).
int select_entry_threshold(const float* E, long long n, long long keep, uint32_t* hist_dev, uint32_t* thr_key,
                           long long* tie_cut, hipStream_t st) {
  if (keep < 1 || keep > n) return PIPE_EINVAL;
  const unsigned grid = (unsigned)std::min<long long>((n + BLK - 1) / BLK, 4096);
  std::vector<uint32_t> h(SEL_BINS);
  // digits of the 31-bit key, most significant first: 11, 11 and 9 bits
  const int shifts[3] = {20, 9, 0}, nbins[3] = {2048, 2048, 512};
  uint32_t prefix = 0;
  long long want = keep;   // entries still to take from the current prefix class, largest first
  uint32_t ties = 0;
  for (int lvl = 0; lvl < 3; ++lvl) {
    PIPE_HIP(hipMemsetAsync(hist_dev, 0, SEL_BINS * sizeof(uint32_t), st));
    PIPE_KLAUNCH(key_histogram_kernel, dim3(grid), dim3(BLK), 0, st, E, n, shifts[lvl], nbins[lvl],
                       lvl == 0 ? 32 : shifts[lvl - 1], prefix, hist_dev);
    PIPE_HIP(hipGetLastError());
    PIPE_HIP(hipMemcpyAsync(h.data(), hist_dev, SEL_BINS * sizeof(uint32_t), hipMemcpyDeviceToHost, st));
    PIPE_HIP(hipStreamSynchronize(st));
    int b = nbins[lvl] - 1;
    for (; b > 0 && (long long)h[b] < want; --b) want -= h[b];
    prefix = lvl == 0 ? (uint32_t)b : ((prefix << (shifts[lvl - 1] - shifts[lvl])) | (uint32_t)b);
    ties = h[b];
  }
  *thr_key = prefix;
  if (want >= (long long)ties) {   // every entry of the threshold magnitude is kept
    *tie_cut = n;
    return PIPE_OK;
  }
  // the smallest flat index c with `want` entries of the threshold magnitude at or below it
  long long lo = 0, hi = n - 1;
  uint32_t* cnt_dev = hist_dev + SEL_BINS;
  while (lo < hi) {
    const long long mid = lo + (hi - lo) / 2;
    uint32_t c = 0;
    PIPE_HIP(hipMemsetAsync(cnt_dev, 0, sizeof(uint32_t), st));
    PIPE_KLAUNCH(count_ties_kernel, dim3(grid), dim3(BLK), 0, st, E, n, prefix, mid, cnt_dev);
    PIPE_HIP(hipGetLastError());
    PIPE_HIP(hipMemcpyAsync(&c, cnt_dev, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
    PIPE_HIP(hipStreamSynchronize(st));
    if ((long long)c >= want) hi = mid; else lo = mid + 1;
  }
  *tie_cut = lo;
  return PIPE_OK;
}

int launch_quantize_rows(float* E, int out, int in, int in_pad, int bits, int qbits, int group,
                         const int32_t* gids, int n_kept, float* scales, uint8_t* packed,
                         const int8_t* given, uint32_t thr_key, long long tie_cut, hipStream_t st) {
  const int qmax = (1 << (qbits - 1)) - 1;
  (void)out;
  const int rows = n_kept * group;
  if (rows == 0) return PIPE_OK;
  if (bits == 8)
    PIPE_KLAUNCH(quantize_rows_kernel<8>, dim3(rows), dim3(BLK), 0, st, E, in, in_pad, group, gids, scales, packed, qmax, given, thr_key, tie_cut);
  else if (bits == 4)
    PIPE_KLAUNCH(quantize_rows_kernel<4>, dim3(rows), dim3(BLK), 0, st, E, in, in_pad, group, gids, scales, packed, qmax, given, thr_key, tie_cut);
  else
    PIPE_KLAUNCH(quantize_rows_kernel<2>, dim3(rows), dim3(BLK), 0, st, E, in, in_pad, group, gids, scales, packed, qmax, given, thr_key, tie_cut);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

int launch_gather_rows(const float* E, int in, int qbits, int group, const int32_t* gids, int n_kept,
                       float* rows_out, float* scales_out, hipStream_t st) {
  const int rows = n_kept * group;
  if (rows == 0) return PIPE_OK;
  PIPE_KLAUNCH(gather_rows_kernel, dim3(rows), dim3(BLK), 0, st, E, in, group, gids, (1 << (qbits - 1)) - 1, rows_out,
                     scales_out);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

int launch_unpack_codes(const uint8_t* packed, const int32_t* rb_map_dev, int bits, int rows, int in, int in_pad,
                        int8_t* codes, hipStream_t st) {
  const int64_t n = (int64_t)rows * in;
  if (n == 0) return PIPE_OK;
  PIPE_KLAUNCH(unpack_codes_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, packed, rb_map_dev,
                     bits, rows, in, in_pad, codes);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

int launch_permute_conv_weight(const float* W, int out, int C, int taps, float* W_out, hipStream_t st) {
  PIPE_KLAUNCH(permute_conv_weight_kernel, dim3(out), dim3(BLK), 0, st, W, C, taps, W_out);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}
