// Data-free error diagnostics (App. C): spectral norms by power iteration, the dequantized
// expansion, element-wise error bounds from the stored scales, and the bound U of Theorems 1-2.
// Not on the forward path: plain HBM-bound kernels, fp64 accumulation.
#include <hip/hip_runtime.h>

#include <cmath>
#include <vector>

#include "pipe_internal.h"

namespace {

constexpr int BLK = 256;
constexpr int ROW_CHUNKS = 64;   // row ranges of the transposed product (partial sums per range)

// +-1/sqrt(n) by a multiplicative hash of the index (bit 15 of i * 2654435761 mod 2^32)
__global__ void start_vector_kernel(float* v, int n) {
  const int i = blockIdx.x * BLK + threadIdx.x;
  if (i >= n) return;
  const uint32_t h = (uint32_t)i * 2654435761u;
  const double s = 1.0 / sqrt((double)n);
  v[i] = (float)(((h >> 15) & 1u) ? s : -s);
}

// y[r] = sum_i W[r,i] v[i]: one wave per row, 16-byte loads when the row allows
__global__ __launch_bounds__(BLK) void matvec_kernel(const float* __restrict__ W, int out, int in,
                                                     const float* __restrict__ v, double* __restrict__ y) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * (BLK / 64) + (threadIdx.x >> 6);
  if (r >= out) return;
  const float* row = W + (size_t)r * in;
  double acc = 0.0;
  if ((in & 3) == 0 && (reinterpret_cast<uintptr_t>(W) & 15) == 0 && (reinterpret_cast<uintptr_t>(v) & 15) == 0) {
    const float4* r4 = reinterpret_cast<const float4*>(row);
    const float4* v4 = reinterpret_cast<const float4*>(v);
    for (int i = lane; i < in / 4; i += 64) {
      const float4 a = r4[i], b = v4[i];
      acc += (double)a.x * b.x + (double)a.y * b.y + (double)a.z * b.z + (double)a.w * b.w;
    }
  } else {
    for (int i = lane; i < in; i += 64) acc += (double)row[i] * v[i];
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
  if (lane == 0) y[r] = acc;
}

// partial[c][i] = sum over the rows of chunk c of W[r,i] y[r]: a thread owns a column, a workgroup
// reads 1 KiB of each row
__global__ __launch_bounds__(BLK) void matvec_t_kernel(const float* __restrict__ W, int out, int in,
                                                       const double* __restrict__ y, double* __restrict__ partial) {
  const int i = blockIdx.x * BLK + threadIdx.x;
  const int per = (out + ROW_CHUNKS - 1) / ROW_CHUNKS;
  const int r_lo = blockIdx.y * per, r_hi = min(out, r_lo + per);
  if (i >= in) return;
  // eight rows in flight per thread, each with its own running sum
  double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  int r = r_lo;
  for (; r + 8 <= r_hi; r += 8) {
    float w[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) w[j] = W[(size_t)(r + j) * in + i];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] += (double)w[j] * y[r + j];
  }
  for (; r < r_hi; ++r) acc[0] += (double)W[(size_t)r * in + i] * y[r];
  partial[(size_t)blockIdx.y * in + i] = ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
}

// z = sum of the partial rows, and each workgroup's share of ||z||^2
__global__ __launch_bounds__(BLK) void reduce_partials_kernel(const double* __restrict__ partial, int in,
                                                              double* __restrict__ z, double* __restrict__ nz_part) {
  const int i = blockIdx.x * BLK + threadIdx.x;
  double t = 0.0;
  if (i < in) {
#pragma unroll 8
    for (int c = 0; c < ROW_CHUNKS; ++c) t += partial[(size_t)c * in + i];
    z[i] = t;
  }
  double a = t * t;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o, 64);
  __shared__ double sm[BLK / 64];
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) nz_part[blockIdx.x] = (sm[0] + sm[1]) + (sm[2] + sm[3]);
}

// One workgroup: sigma = ||y||; ||z|| from the workgroups' shares; v = z / ||z|| (left alone if
// z = 0).  With nz_part == nullptr only sigma is produced.
__global__ __launch_bounds__(1024) void normalize_kernel(const double* __restrict__ y, int out,
                                                         const double* __restrict__ nz_part, int n_part, int in,
                                                         float* __restrict__ v, const double* __restrict__ z,
                                                         double* __restrict__ sigma) {
  __shared__ double sm[16];
  auto block_sum = [&](double a) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = a;
    __syncthreads();
    double t = 0.0;
    for (int w = 0; w < 16; ++w) t += sm[w];
    return t;
  };
  double a = 0.0;
  for (int r = threadIdx.x; r < out; r += 1024) a += y[r] * y[r];
  const double ny = sqrt(block_sum(a));
  if (threadIdx.x == 0) *sigma = ny;
  if (nz_part == nullptr) return;
  double b = 0.0;
  for (int i = threadIdx.x; i < n_part; i += 1024) b += nz_part[i];
  const double nz = sqrt(block_sum(b));
  if (nz > 0.0)
    for (int i = threadIdx.x; i < in; i += 1024) v[i] = (float)(z[i] / nz);
}

// W_out[o, i] += s[r] * code[r, i] for the stored rows of one order (fp32, product then sum)
__global__ __launch_bounds__(BLK) void add_order_kernel(const int8_t* __restrict__ codes, const float* __restrict__ scales_all,
                                                        const int32_t* __restrict__ pos, const int32_t* __restrict__ gids,
                                                        int group, int in, float* __restrict__ W_out) {
  const int r = blockIdx.x;   // stored (compact) row
  const float s = scales_all[(size_t)pos[r >> 4] * 16 + (r & 15)];
  const int slot = r / group;
  const int o = gids[slot] * group + (r - slot * group);
  const int8_t* c = codes + (size_t)r * in;
  float* w = W_out + (size_t)o * in;
  for (int i = threadIdx.x; i < in; i += BLK) w[i] = __fadd_rn(w[i], __fmul_rn(s, (float)c[i]));
}

// R[r, i] = s[r] * code[r, i] for the stored rows of one order, compact (pruned rows left out:
// zero rows do not change a matrix's singular values)
__global__ __launch_bounds__(BLK) void scale_rows_kernel(const int8_t* __restrict__ codes, const float* __restrict__ scales_all,
                                                         const int32_t* __restrict__ pos, int in, float* __restrict__ R) {
  const int r = blockIdx.x;
  const float s = scales_all[(size_t)pos[r >> 4] * 16 + (r & 15)];
  const int8_t* c = codes + (size_t)r * in;
  float* w = R + (size_t)r * in;
  for (int i = threadIdx.x; i < in; i += BLK) w[i] = __fmul_rn(s, (float)c[i]);
}

int spectral_norm_dev(const float* W_dev, int out, int in, int iters, double* sigma_host, hipStream_t st) {
  // v [in] fp32 | y [out] fp64 | z [in] fp64 | sigma fp64 | ||z||^2 shares | partial [ROW_CHUNKS][in] fp64
  const int n_part = ceil_div(in, BLK);
  const size_t off_y = ((size_t)in * 4 + 255) & ~(size_t)255;
  const size_t off_z = off_y + (((size_t)out * 8 + 255) & ~(size_t)255);
  const size_t off_s = off_z + (((size_t)in * 8 + 255) & ~(size_t)255);
  const size_t off_n = off_s + 256;
  const size_t off_p = off_n + (((size_t)n_part * 8 + 255) & ~(size_t)255);
  uint8_t* ws = (uint8_t*)pipe_ws_get(WS_DIAG, off_p + (size_t)ROW_CHUNKS * in * 8);
  if (!ws) return pipe_ws_error();
  float* v = (float*)ws;
  double* y = (double*)(ws + off_y);
  double* z = (double*)(ws + off_z);
  double* sigma = (double*)(ws + off_s);
  double* nz_part = (double*)(ws + off_n);
  double* partial = (double*)(ws + off_p);
  PIPE_KLAUNCH(start_vector_kernel, dim3(ceil_div(in, BLK)), dim3(BLK), 0, st, v, in);
  const dim3 g_mv(ceil_div(out, BLK / 64)), g_mt(ceil_div(in, BLK), ROW_CHUNKS);
  for (int it = 0; it < iters; ++it) {
    PIPE_KLAUNCH(matvec_kernel, g_mv, dim3(BLK), 0, st, W_dev, out, in, v, y);
    PIPE_KLAUNCH(matvec_t_kernel, g_mt, dim3(BLK), 0, st, W_dev, out, in, y, partial);
    PIPE_KLAUNCH(reduce_partials_kernel, dim3(n_part), dim3(BLK), 0, st, partial, in, z, nz_part);
    PIPE_KLAUNCH(normalize_kernel, dim3(1), dim3(1024), 0, st, y, out, nz_part, n_part, in, v, z, sigma);
  }
  PIPE_KLAUNCH(matvec_kernel, g_mv, dim3(BLK), 0, st, W_dev, out, in, v, y);
  PIPE_KLAUNCH(normalize_kernel, dim3(1), dim3(1024), 0, st, y, out, (const double*)nullptr, 0, in, v, z, sigma);
  PIPE_HIP(hipGetLastError());
  double s = 0.0;
  PIPE_HIP(hipMemcpyAsync(&s, sigma, sizeof(double), hipMemcpyDeviceToHost, st));
  PIPE_HIP(hipStreamSynchronize(st));
  *sigma_host = s;
  return PIPE_OK;
}

}  // namespace

extern "C" int pipe_spectral_norm(const float* W_dev, int out, int in, int iters, float* sigma_host, void* stream) {
  if (!W_dev || !sigma_host || iters < 1) return PIPE_EINVAL;
  if (out < 1 || in < 1) return PIPE_ESHAPE;
  double s = 0.0;
  const int rc = spectral_norm_dev(W_dev, out, in, iters, &s, (hipStream_t)stream);
  if (rc == PIPE_OK) *sigma_host = (float)s;
  return rc;
}

extern "C" int pipe_expansion_order_norms(const pipe_expansion* e, int iters, double* norms_host, void* stream) {
  if (!e || !norms_host || iters < 1) return PIPE_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  for (int k = 0; k < e->K; ++k) {
    const PipeOrder& o = e->orders[k];
    const int rows = o.n_kept * e->group;
    norms_host[k] = 0.0;
    if (rows == 0) continue;
    int8_t* tmp = (int8_t*)pipe_ws_get(WS_DIAG_CODES, (size_t)rows * e->in);
    float* R = (float*)pipe_ws_get(WS_DIAG_DENSE, (size_t)rows * e->in * sizeof(float));
    if (!tmp || !R) return pipe_ws_error();
    int rc = launch_unpack_codes(e->codes_dev, o.pos_dev, e->bits, rows, e->in, e->in_pad, tmp, st);
    if (rc) return rc;
    PIPE_KLAUNCH(scale_rows_kernel, dim3(rows), dim3(BLK), 0, st, tmp, e->scales_all_dev, o.pos_dev, e->in, R);
    PIPE_HIP(hipGetLastError());
    rc = spectral_norm_dev(R, rows, e->in, iters, &norms_host[k], st);
    if (rc) return rc;
  }
  return PIPE_OK;
}

extern "C" int pipe_expansion_reconstruct(const pipe_expansion* e, int upto, float* W_out_dev, void* stream) {
  if (!e || !W_out_dev) return PIPE_EINVAL;
  if (upto < 1 || upto > e->K) return PIPE_EINVAL;
  if (e->conv_C > 0) return PIPE_EINVAL;   // stored tap-major: its rows are not laid out as the weight was given
  hipStream_t st = (hipStream_t)stream;
  PIPE_HIP(hipMemsetAsync(W_out_dev, 0, (size_t)e->out * e->in * sizeof(float), st));
  for (int k = 0; k < upto; ++k) {
    const PipeOrder& o = e->orders[k];
    const int rows = o.n_kept * e->group;
    if (rows == 0) continue;
    int8_t* tmp = (int8_t*)pipe_ws_get(WS_DIAG_CODES, (size_t)rows * e->in);
    if (!tmp) return pipe_ws_error();
    int rc = launch_unpack_codes(e->codes_dev, o.pos_dev, e->bits, rows, e->in, e->in_pad, tmp, st);
    if (rc) return rc;
    PIPE_KLAUNCH(add_order_kernel, dim3(rows), dim3(BLK), 0, st, tmp, e->scales_all_dev, o.pos_dev, o.gids_dev,
                       e->group, e->in, W_out_dev);
    PIPE_HIP(hipGetLastError());
  }
  return PIPE_OK;
}

extern "C" int pipe_expansion_error_bound(const pipe_expansion* e, double* u_lemma, double* u_stored) {
  if (!e) return PIPE_EINVAL;
  if (e->unstructured) return PIPE_EINVAL;   // a pruned entry keeps an earlier order's residual: the row scales do not bound it
  PIPE_HIP(hipDeviceSynchronize());
  const size_t n_pos = (size_t)e->n_pos;
  std::vector<float> all(n_pos * 16);
  PIPE_HIP(hipMemcpy(all.data(), e->scales_all_dev, all.size() * sizeof(float), hipMemcpyDeviceToHost));
  std::vector<double> last((size_t)e->out, 0.0);
  double s1 = 0.0;
  for (int k = 0; k < e->K; ++k) {
    const PipeOrder& o = e->orders[k];
    for (int slot = 0; slot < o.n_kept; ++slot)
      for (int j = 0; j < e->group; ++j) {
        const int r = slot * e->group + j;
        const double s = all[(size_t)o.pos[r >> 4] * 16 + (r & 15)];
        last[(size_t)o.gids[slot] * e->group + j] = s;
        if (k == 0) s1 = std::max(s1, s);
      }
  }
  double lmax = 0.0;
  for (double s : last) lmax = std::max(lmax, s);
  const double qm = (double)((1 << (e->qbits - 1)) - 1);
  if (u_lemma) *u_lemma = std::pow(1.0 / qm, e->K - 1) * s1 / 2.0;
  if (u_stored) *u_stored = lmax / 2.0;
  return PIPE_OK;
}

extern "C" int pipe_error_bound_U(const double* s, const double* u, int L, double* U_out) {
  if (!s || !u || !U_out || L < 1) return PIPE_EINVAL;
  double U = 1.0, run = 0.0;
  for (int l = 0; l < L; ++l) {
    run += s[l] * u[l];
    U *= run + 1.0;
  }
  *U_out = U - 1.0;
  return PIPE_OK;
}

static int u_ens(const double* norms, const double* lam, int L, int K, const int* split, int M, double* out) {
  int lo = 0;
  double head = 0.0, tail = 0.0;
  for (int m = 0; m < M; ++m) {
    const int hi = lo + split[m];
    if (m == 0) {
      for (int k = lo; k < hi; ++k) head += norms[(size_t)(L - 1) * K + k];
      head /= std::ldexp(1.0, L - 1);
    } else {
      double prod = 1.0;
      for (int l = 0; l + 1 < L; ++l) {
        double sum = 0.0;
        for (int k = lo; k < hi; ++k) sum += norms[(size_t)l * K + k] * (lam ? lam[(size_t)l * K + k] : 1.0);
        prod *= sum;
      }
      tail += prod;
    }
    lo = hi;
  }
  *out = head * (1.0 + tail);
  return PIPE_OK;
}

extern "C" int pipe_error_bound_U_ens(const double* norms, const double* lam, int L, int K, const int* split, int M,
                                      double* U_out) {
  if (!norms || !U_out || L < 1 || K < 1 || K > PIPE_MAX_K) return PIPE_EINVAL;
  const int whole[1] = {K};
  if (!split) { split = whole; M = 1; }
  if (M < 1) return PIPE_ESPLIT;
  int sum = 0;
  for (int m = 0; m < M; ++m) {
    if (split[m] < 1) return PIPE_ESPLIT;
    sum += split[m];
  }
  if (sum != K) return PIPE_ESPLIT;
  return u_ens(norms, lam, L, K, split, M, U_out);
}

extern "C" int pipe_first_predictor_size(const double* norms, const double* lam, int L, int K, double logit_norm,
                                         double ratio, int* K1_out) {
  if (!norms || !K1_out || L < 1 || K < 1 || K > PIPE_MAX_K) return PIPE_EINVAL;
  *K1_out = K;
  for (int K1 = 1; K1 < K; ++K1) {
    const int split[2] = {K1, K - K1};
    double U = 0.0;
    u_ens(norms, lam, L, K, split, 2, &U);
    if (U <= ratio * logit_norm) { *K1_out = K1; break; }
  }
  return PIPE_OK;
}
