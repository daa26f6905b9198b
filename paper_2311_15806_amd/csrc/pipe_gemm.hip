// Tiled int8-MFMA kernel of the expanded layer (App. B, Eq. (define_dre)):
//   y[t,o] = sum_m ( s_x,m * sum_{k in member m} s_k[o] * acc_k[t,o]  (+ b[o] if m = 0) )
//   acc_k[t,o] = sum_i Qx[t,i] * q_k[o,i]          (exact, int32)
//
// One workgroup (4 waves) owns 128 tokens x 8 row blocks (128 stored channels).  The row
// blocks of a column tile were sorted at expansion time by the set of orders that hold them,
// so the loop over orders does uniform work; a row block that an order pruned is skipped
// (no load, no MFMA).  Packed 4-bit / ternary codes are streamed from HBM with 16-byte
// coalesced loads, widened to int8 with a shift and a mask, and staged in LDS in the
// register layout of v_mfma_i32_16x16x64_i8 (A operand = 16 channels x 64 k, B operand = 16
// tokens x 64 k, D = 4 consecutive channels x 1 token per lane).  Codes are stored
// offset-binary; the offset is removed exactly in the epilogue with the token's code sum.
// Per order the int32 accumulators are folded into an fp32 running sum with the row-wise
// scale; the activation scale, the bias, the optional GELU and the member sum are applied once.
#include "pipe_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int TT = 128;               // tokens per tile
constexpr int NTB = TT / 16;          // token blocks per tile
constexpr int STAGE_STEPS = 2;        // 64-k steps per LDS stage
constexpr int FRAG = 64;              // uint4 per fragment

struct TiledParams {
  const uint8_t* qx;
  int64_t qx_mstride;
  const int32_t* rowsum;
  int64_t rowsum_mstride;
  const float* s_x;
  int sx_mstride;
  const uint8_t* const* packed;   // [K]
  const float* const* scales;     // [K]
  const int32_t* ct_rb_out;       // [n_ct][NRB_TILE]
  const int32_t* ct_src;          // [n_ct][K][NRB_TILE]
  const float* bias;
  float* y;
  int32_t* acc_out;
  uint32_t* amax_out;
  int T, out, K, nks, n_tt, n_ct, M, reduce, act;
  int member_lo[PIPE_MAX_K];
  int member_hi[PIPE_MAX_K];
};

__device__ __forceinline__ float gelu_erf(float a) {
  return 0.5f * a * (1.f + erff(a * 0.70710678118654752440f));
}

template <int BITS, bool ACC_OUT>
__global__ __launch_bounds__(256) void gemm_tiled_kernel(const TiledParams p) {
  constexpr int OFF = BITS == 8 ? 0 : (BITS == 4 ? 8 : 1);
  constexpr int KSUP = 512 / BITS;
  __shared__ uint4 Xs[2][NTB * STAGE_STEPS * FRAG];       // 2 x 16 KiB
  __shared__ uint4 Ws[2][NRB_TILE * STAGE_STEPS * FRAG];  // 2 x 16 KiB

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wm = wave & 1;   // token half: token blocks 4*wm .. 4*wm+3
  const int wn = wave >> 1;  // row-block half: row blocks 4*wn .. 4*wn+3
  const int ct = blockIdx.x / p.n_tt;
  const int tt = blockIdx.x - ct * p.n_tt;
  const int t0 = tt * TT;
  const int nksup = (p.nks * 64) / KSUP;
  const int n_stage = p.nks / STAGE_STEPS;

  int rb_out[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) rb_out[r] = p.ct_rb_out[ct * NRB_TILE + 4 * wn + r];

  float ytot[4][4][4];
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int i = 0; i < 4; ++i) ytot[r][b][i] = 0.f;

  for (int m = 0; m < p.M; ++m) {
    const uint8_t* qx = p.qx + (size_t)m * p.qx_mstride;
    const int32_t* rowsum = p.rowsum + (size_t)m * p.rowsum_mstride;
    float yacc[4][4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int i = 0; i < 4; ++i) yacc[r][b][i] = 0.f;
    int rs[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) rs[b] = OFF ? rowsum[t0 + (4 * wm + b) * 16 + (lane & 15)] : 0;

    for (int k = p.member_lo[m]; k <= p.member_hi[m]; ++k) {
      // which row blocks of this column tile does order k hold?
      const int32_t* srcp = p.ct_src + ((size_t)ct * p.K + k) * NRB_TILE;
      int src_ld[2];   // the two row blocks this wave loads: 2*wave, 2*wave+1
      src_ld[0] = srcp[2 * wave];
      src_ld[1] = srcp[2 * wave + 1];
      int src_mm[4];   // the four row blocks this wave multiplies
      bool any = false;
#pragma unroll
      for (int r = 0; r < 4; ++r) src_mm[r] = srcp[4 * wn + r];
#pragma unroll
      for (int r = 0; r < NRB_TILE; ++r) any |= srcp[r] >= 0;
      if (!any) continue;   // uniform over the workgroup
      const uint8_t* pk = p.packed[k];

      v4i acc[4][4];
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[r][b] = v4i{0, 0, 0, 0};

      uint4 xr[4];
      uint4 wr[2][2];
      auto gload = [&](int s) {
        // activations: 16 fragments per stage, 4 per wave
#pragma unroll
        for (int f = 0; f < 4; ++f) {
          const int idx = wave * 4 + f;             // = tb*2 + j
          const int tb = idx >> 1, j = idx & 1;
          const uint4* g = reinterpret_cast<const uint4*>(
              qx + ((size_t)(t0 / 16 + tb) * p.nks + (s * STAGE_STEPS + j)) * 1024);
          xr[f] = g[lane];
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          if (src_ld[q] < 0) continue;
          if (BITS == 8) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
              wr[q][j] = reinterpret_cast<const uint4*>(pk + ((size_t)src_ld[q] * nksup + (s * 2 + j)) * 1024)[lane];
          } else if (BITS == 4) {
            wr[q][0] = reinterpret_cast<const uint4*>(pk + ((size_t)src_ld[q] * nksup + s) * 1024)[lane];
          } else {
            const uint2 v = reinterpret_cast<const uint2*>(pk + ((size_t)src_ld[q] * nksup + (s >> 1)) * 1024)[lane * 2 + (s & 1)];
            wr[q][0].x = v.x;
            wr[q][0].y = v.y;
          }
        }
      };
      auto lstore = [&](int buf) {
#pragma unroll
        for (int f = 0; f < 4; ++f) Xs[buf][(wave * 4 + f) * FRAG + lane] = xr[f];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          if (src_ld[q] < 0) continue;
          const int rb = 2 * wave + q;
          uint4 o0, o1;
          if (BITS == 8) {
            o0 = wr[q][0];
            o1 = wr[q][1];
          } else if (BITS == 4) {
            const uint4 w = wr[q][0];
            o0 = make_uint4(w.x & 0x0F0F0F0Fu, (w.x >> 4) & 0x0F0F0F0Fu, w.y & 0x0F0F0F0Fu, (w.y >> 4) & 0x0F0F0F0Fu);
            o1 = make_uint4(w.z & 0x0F0F0F0Fu, (w.z >> 4) & 0x0F0F0F0Fu, w.w & 0x0F0F0F0Fu, (w.w >> 4) & 0x0F0F0F0Fu);
          } else {
            const uint32_t a = wr[q][0].x, b = wr[q][0].y;
            o0 = make_uint4(a & 0x03030303u, (a >> 2) & 0x03030303u, (a >> 4) & 0x03030303u, (a >> 6) & 0x03030303u);
            o1 = make_uint4(b & 0x03030303u, (b >> 2) & 0x03030303u, (b >> 4) & 0x03030303u, (b >> 6) & 0x03030303u);
          }
          Ws[buf][(rb * 2 + 0) * FRAG + lane] = o0;
          Ws[buf][(rb * 2 + 1) * FRAG + lane] = o1;
        }
      };

      gload(0);
      for (int s = 0; s < n_stage; ++s) {
        const int buf = s & 1;
        lstore(buf);
        __syncthreads();
        if (s + 1 < n_stage) gload(s + 1);
#pragma unroll
        for (int j = 0; j < STAGE_STEPS; ++j) {
          v4i xf[4];
#pragma unroll
          for (int b = 0; b < 4; ++b) {
            const uint4 v = Xs[buf][((4 * wm + b) * 2 + j) * FRAG + lane];
            xf[b] = v4i{(int)v.x, (int)v.y, (int)v.z, (int)v.w};
          }
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            if (src_mm[r] < 0) continue;
            const uint4 v = Ws[buf][((4 * wn + r) * 2 + j) * FRAG + lane];
            const v4i wf = v4i{(int)v.x, (int)v.y, (int)v.z, (int)v.w};
#pragma unroll
            for (int b = 0; b < 4; ++b)
              acc[r][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf, xf[b], acc[r][b], 0, 0, 0);
          }
        }
      }
      __syncthreads();

      // fold this order: yacc += s_k[o] * float(acc - OFF * rowsum)
      const float* sck = p.scales[k];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if (src_mm[r] < 0) continue;
        const float4 sc = *reinterpret_cast<const float4*>(sck + (size_t)src_mm[r] * 16 + 4 * (lane >> 4));
        const float scv[4] = {sc.x, sc.y, sc.z, sc.w};
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const int t = t0 + (4 * wm + b) * 16 + (lane & 15);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int a = acc[r][b][i] - OFF * rs[b];
            yacc[r][b][i] = fmaf(scv[i], (float)a, yacc[r][b][i]);
            if (ACC_OUT) {
              if (t < p.T && rb_out[r] >= 0)
                p.acc_out[((size_t)k * p.T + t) * p.out + rb_out[r] * 16 + 4 * (lane >> 4) + i] = a;
            }
          }
        }
      }
    }  // orders of the member

    if (ACC_OUT) continue;
    // member epilogue
    const float sx = p.s_x[m * p.sx_mstride];
    float mx = 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if (rb_out[r] < 0) continue;
      const int ch = rb_out[r] * 16 + 4 * (lane >> 4);
      float bv[4] = {0.f, 0.f, 0.f, 0.f};
      if (m == 0 && p.bias != nullptr) {
        const float4 b4 = *reinterpret_cast<const float4*>(p.bias + ch);
        bv[0] = b4.x; bv[1] = b4.y; bv[2] = b4.z; bv[3] = b4.w;
      }
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const int t = t0 + (4 * wm + b) * 16 + (lane & 15);
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          v[i] = sx * yacc[r][b][i] + bv[i];
          if (p.act == PIPE_ACT_GELU) v[i] = gelu_erf(v[i]);
          if (t < p.T) mx = fmaxf(mx, fabsf(v[i]));
        }
        if (p.reduce) {
#pragma unroll
          for (int i = 0; i < 4; ++i) ytot[r][b][i] = (m == 0) ? v[i] : ytot[r][b][i] + v[i];
        } else if (t < p.T) {
          *reinterpret_cast<float4*>(p.y + ((size_t)m * p.T + t) * p.out + ch) = make_float4(v[0], v[1], v[2], v[3]);
        }
      }
    }
    if (p.amax_out != nullptr) {
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
      if (lane == 0) atomicMax(&p.amax_out[m], __float_as_uint(mx));
    }
  }  // members

  if (!ACC_OUT && p.reduce) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if (rb_out[r] < 0) continue;
      const int ch = rb_out[r] * 16 + 4 * (lane >> 4);
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const int t = t0 + (4 * wm + b) * 16 + (lane & 15);
        if (t < p.T)
          *reinterpret_cast<float4*>(p.y + (size_t)t * p.out + ch) =
              make_float4(ytot[r][b][0], ytot[r][b][1], ytot[r][b][2], ytot[r][b][3]);
      }
    }
  }
}

template <int BITS>
int launch_bits(const TiledParams& p, bool acc_out, hipStream_t st) {
  const dim3 grid((unsigned)(p.n_ct * p.n_tt));
  if (acc_out)
    hipLaunchKernelGGL((gemm_tiled_kernel<BITS, true>), grid, dim3(256), 0, st, p);
  else
    hipLaunchKernelGGL((gemm_tiled_kernel<BITS, false>), grid, dim3(256), 0, st, p);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

}  // namespace

int launch_gemm_tiled(const GemmArgs& a, hipStream_t st) {
  const pipe_expansion* e = a.e;
  if (a.T <= 0) return PIPE_OK;
  if (a.T_pad % TT != 0) return PIPE_ESHAPE;
  TiledParams p;
  p.qx = a.qx; p.qx_mstride = a.qx_mstride;
  p.rowsum = a.rowsum; p.rowsum_mstride = a.rowsum_mstride;
  p.s_x = a.s_x; p.sx_mstride = a.sx_mstride;
  p.packed = e->packed_ptrs_dev; p.scales = e->scale_ptrs_dev;
  p.ct_rb_out = e->ct_rb_out_dev; p.ct_src = e->ct_src_dev;
  p.bias = a.bias; p.y = a.y; p.acc_out = a.acc_out; p.amax_out = a.amax_out;
  p.T = a.T; p.out = e->out; p.K = e->K; p.nks = e->nks;
  p.n_tt = ceil_div(a.T, TT); p.n_ct = e->n_ct; p.M = a.M; p.reduce = a.reduce; p.act = a.act;
  for (int m = 0; m < PIPE_MAX_K; ++m) { p.member_lo[m] = a.member_lo[m]; p.member_hi[m] = a.member_hi[m]; }
  const bool acc_out = a.acc_out != nullptr;
  switch (e->bits) {
    case 8: return launch_bits<8>(p, acc_out, st);
    case 4: return launch_bits<4>(p, acc_out, st);
    default: return launch_bits<2>(p, acc_out, st);
  }
}

// The weight-streaming small-batch kernel lives in pipe_gemv.hip.
