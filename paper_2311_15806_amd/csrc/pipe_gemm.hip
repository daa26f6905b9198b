// Tiled int8-MFMA kernel of the expanded layer (App. B, Eq. (define_dre)):
//   y[t,o] = sum_m ( s_x,m * sum_{k in member m} s_k[o] * acc_k[t,o]  (+ b[o] if m = 0) )
//   acc_k[t,o] = sum_i Qx[t,i] * q_k[o,i]          (exact, int32)
//
// One workgroup (4 waves) owns MT = 16*MTB tokens x 4*NRW row blocks (16 stored channels
// each).  Every wave multiplies ALL MT tokens with its OWN NRW row blocks, so
//   - packed 4-bit / ternary codes never pass through LDS: each wave streams the 1-KiB tiles
//     of its row blocks from L2/HBM with one coalesced 16-byte load per lane, keeps them
//     packed in registers and widens them to int8 (shift + mask, offset-binary codes) right
//     before the MFMA that consumes them;
//   - only the int8 activation tile is staged in LDS (double buffered, one barrier per 256 k),
//     already in the register layout of the B operand of v_mfma_i32_16x16x64_i8, so LDS reads
//     are lane-linear 16-byte reads without bank conflicts.
// The row blocks of a column tile were sorted at expansion time by the set of orders that
// hold them, so the loop over orders does uniform work; a row block that an order pruned is
// skipped (no load, no MFMA).  Per order the int32 accumulators (minus offset * token code
// sum, exact) are folded into an fp32 running sum with the row-wise scale; activation scale,
// bias, optional GELU and the member sum are applied once in the epilogue.
// Workgroups are mapped to (column tile, token tile) in super-tiles of 64 tiles per XCD (8 x 8, or
// 16 x 4 when that deals every XCD a share of every column-tile row) so that the 64 workgroups
// resident on one XCD share a few weight strips and activation strips in its L2.
#include <type_traits>

#include "pipe_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int S = 4;       // 64-k steps per LDS stage (256 k)
constexpr int FRAG = 64;   // uint4 per fragment

struct TiledParams {
  const uint8_t* qx;
  int64_t qx_mstride;
  const int32_t* rowsum;
  int64_t rowsum_mstride;
  const float* s_x;
  int sx_mstride;
  const uint8_t* codes;           // stored row blocks of all orders, schedule order
  const float* scales;            // their row scales, 16 per position
  const int32_t* rb_out;          // [n_sorted] output row block of sorted position i, or -1
  const int32_t* rb_src;          // [M][p_max][n_sorted] position of the row block's j-th stored order of member m, or -1
  const uint8_t* ct_cnt;          // [n_ct][16] passes member m runs in the column tile
  int n_sorted;                   // padded to a multiple of 64
  int p_max;
  const float* bias;
  long long bias_mstride;         // 0: the first member's (or the sum's) vector; else one vector per member
  float* y;
  int32_t* acc_out;
  uint32_t* amax_out;
  uint32_t* amax_neg;             // if set: positive and negative parts of the range apart
  uint32_t* zero_after;
  int zero_n;
  uint32_t* zero_big;
  int zero_big_n;
  int T, out, K, nks, n_tt, n_ct, M, reduce, act;
  const float* res;               // MODE_CHAIN: skip tensor [res_members, T, out] or nullptr
  long long res_mstride;
  int res_members, res_pre_act;
  int hidden;                     // MODE_GATED: H; the layer's rows are gate [0,H) and up [H,2H), y is [M,T,H]
  int n_st_t;                     // super-tiles along tokens
  int st_c_log2;                  // a super-tile is 2^st_c_log2 column tiles x 64 / 2^st_c_log2 token tiles
  // CONV (implicit GEMM: the expansion's k runs tap-major, channel-minor): the activation stage gathers
  // each 64-channel chunk of a tap straight from the channels-last codes of the input tensor
  const int8_t* cq8;              // Q(x) [N, H, W, C]
  const int32_t* ccsum;           // per input pixel: sum of its C codes
  const uint8_t* czero;           // 16 zero bytes: what a tap outside the image (or beyond in_features) reads
  int cC, cH, cW, ckh, ckw, cstride, cpad, cHo, cWo;
};

__device__ __forceinline__ float gelu_erf(float a) {
  return 0.5f * a * (1.f + erff(a * 0.70710678118654752440f));
}

template <int BITS>
struct WRegs {
  static constexpr int N = BITS == 2 ? 1 : (BITS == 4 ? 2 : 4);   // uint4 per row block per stage
  uint4 v[N];
};

// Hand-issued LDS reads: N fragments (16 bytes per lane each) at byte offsets BASE + b*STRIDE
// from `addr` (LDS byte address of this lane's slot in fragment 0).  The results may be used
// only after lds_wait on the same registers.
template <int N, int BASE, int STRIDE>
__device__ __forceinline__ void lds_read_frags(unsigned addr, v4i (&x)[N]) {
#pragma unroll
  for (int b = 0; b < N; ++b)
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(x[b]) : "v"(addr), "n"(BASE + b * STRIDE) : "memory");
}
// Waits until at most PENDING later LDS reads are outstanding (LDS reads return in order), i.e.
// until the N fragments of x, issued before them, have arrived.
template <int N, int PENDING>
__device__ __forceinline__ void lds_wait(v4i (&x)[N]) {
  static_assert((N == 1 || N == 2 || N == 4) && (PENDING == 0 || PENDING == N), "token blocks per tile");
  if constexpr (N == 4) {
    if constexpr (PENDING == 0)
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3])::"memory");
    else
      asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3])::"memory");
  } else if constexpr (N == 2) {
    if constexpr (PENDING == 0)
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(x[0]), "+v"(x[1])::"memory");
    else
      asm volatile("s_waitcnt lgkmcnt(2)" : "+v"(x[0]), "+v"(x[1])::"memory");
  } else {
    if constexpr (PENDING == 0)
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(x[0])::"memory");
    else
      asm volatile("s_waitcnt lgkmcnt(1)" : "+v"(x[0])::"memory");
  }
}

template <int BITS>
__device__ __forceinline__ v4i widen(const WRegs<BITS>& w, int j) {
  if (BITS == 8) {
    const uint4 a = w.v[j & (WRegs<BITS>::N - 1)];
    return v4i{(int)a.x, (int)a.y, (int)a.z, (int)a.w};
  } else if (BITS == 4) {
    const uint4 q = w.v[(j >> 1) & (WRegs<BITS>::N - 1)];
    const uint32_t a = (j & 1) ? q.z : q.x, b = (j & 1) ? q.w : q.y;
    return v4i{(int)(a & 0x0F0F0F0Fu), (int)((a >> 4) & 0x0F0F0F0Fu), (int)(b & 0x0F0F0F0Fu), (int)((b >> 4) & 0x0F0F0F0Fu)};
  } else {
    const uint4 q = w.v[0];
    const uint32_t a = j == 0 ? q.x : (j == 1 ? q.y : (j == 2 ? q.z : q.w));
    return v4i{(int)(a & 0x03030303u), (int)((a >> 2) & 0x03030303u), (int)((a >> 4) & 0x03030303u), (int)((a >> 6) & 0x03030303u)};
  }
}

// A load known to hit global memory.  Pointers rebuilt from integers are "generic" to the
// compiler, which would emit FLAT loads: those also count as LDS operations (every wait on the
// LDS fragment reads would then wait for the weight prefetch as well) and are ordered against
// the LDS-direct loads.
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 gload16(const void* p) {
  typedef const __attribute__((address_space(1))) v4u* gptr;
  const v4u v = *(gptr)(unsigned long long)p;
  return make_uint4(v.x, v.y, v.z, v.w);
}

// Loads of schedule tables at wave-uniform addresses through the constant address space: the
// compiler then uses scalar loads (the tables are written once, by the host, when the expansion
// is built; no kernel ever stores to them), which cost no vector registers and no vector wait.
template <class T>
__device__ __forceinline__ T cload(const T* base, size_t idx) {
  typedef const __attribute__((address_space(4))) T* cptr;
  return ((cptr)(unsigned long long)base)[idx];
}

// MODE_CHAIN: activation chosen at run time (none, ReLU, GELU) and a skip tensor added before or
// after it (a layer inside a member chain)
enum { MODE_PLAIN = 0, MODE_ACC_OUT = 1, MODE_GELU = 2, MODE_GATED = 3, MODE_CHAIN = 4 };

}  // namespace

int g_tiled_mtb = 0;   // 16-token blocks per tile of the tiled kernel: 0 = automatic, else 1, 2 or 4

namespace {

template <int BITS, int MTB, int NRW, int MINW, int MODE, bool CONV = false>
__global__ __launch_bounds__(256, MINW) void gemm_tiled_kernel(const TiledParams p) {
  constexpr bool ACC_OUT = MODE == MODE_ACC_OUT;
  constexpr int OFF = BITS == 8 ? 0 : (BITS == 4 ? 8 : 1);
  constexpr int KSUP = 512 / BITS;
  constexpr int WN = WRegs<BITS>::N;
  constexpr int NRB_WG = 4 * NRW;
  constexpr int XCOPY = MTB * S / 4;              // activation fragments per wave per stage
  static_assert(TOK_TILE % (16 * MTB) == 0 || (16 * MTB) % TOK_TILE == 0, "token tile");
  __shared__ uint4 Xs[2][MTB * S * FRAG];
  __shared__ uint4 Stg[MTB == 4 ? 1 : 4 * 256];   // output staging of narrow token tiles (wide ones reuse Xs[1])
  __shared__ float Scl[4][16 * NRW];   // per wave: row scales of the current order

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform

  // ---- (column tile, token tile) from blockIdx: super-tiles of 64 tiles, one per XCD at a time ----
  if (p.zero_big != nullptr)
    for (int i = blockIdx.x * 256 + threadIdx.x; i < p.zero_big_n; i += gridDim.x * 256) p.zero_big[i] = 0u;
  int ct, tt;
  {
    const int i = blockIdx.x;
    const int xcd = i & 7, j = i >> 3;
    const int sidx = (j >> 6) * 8 + xcd, local = j & 63;
    const int sc = sidx / p.n_st_t, st = sidx - sc * p.n_st_t;
    const int tl2 = 6 - p.st_c_log2;
    ct = (sc << p.st_c_log2) + (local >> tl2);
    tt = (st << tl2) + (local & ((1 << tl2) - 1));
    if (ct >= p.n_ct || tt >= p.n_tt) return;
  }
  if (blockIdx.x == 0 && (int)threadIdx.x < p.zero_n && p.zero_after != nullptr) p.zero_after[threadIdx.x] = 0u;
  const int t0 = tt * (16 * MTB);
  // LDS byte address of this lane's 16 bytes inside fragment 0 of buffer 0
  const unsigned xs_lane = (unsigned)(uintptr_t)(__attribute__((address_space(3))) uint4*)&Xs[0][0] + lane * 16;
  const int nksup = (p.nks * 64) / KSUP;
  const int n_stage = p.nks / S;

  // CONV: this lane's token (output pixel) of each of the fragments it loads: element offset of the
  // window's first tap and channel 0 in Q(x), and the tap's row and column in the input (may lie
  // outside the image; a token beyond the batch lies outside for every tap)
  constexpr int NCB = CONV ? XCOPY : 1;
  int c_off[NCB], c_h0[NCB], c_w0[NCB];
  int c_r[NCB], c_q[NCB], c_c0[NCB];   // wave-uniform: tap (row, column) and first channel of the 64-k step each fragment loads next
  if constexpr (CONV) {
#pragma unroll
    for (int f = 0; f < XCOPY; ++f) {
      const int b = (wave * XCOPY + f) / S;
      const int t = t0 + b * 16 + (lane & 15);
      const int wo = t % p.cWo, ho = (t / p.cWo) % p.cHo, img = t / (p.cWo * p.cHo);
      const int h0 = ho * p.cstride - p.cpad;
      c_h0[f] = t < p.T ? h0 : -(1 << 20);   // a token beyond the batch: every tap outside
      c_w0[f] = wo * p.cstride - p.cpad;
      c_off[f] = ((img * p.cH + h0) * p.cW + c_w0[f]) * p.cC + (lane >> 4) * 16;   // used only for taps inside the image
    }
  }
  // ---- tile descriptors, fetched once (one memory round trip) -------------------------------
  // the first activation stage does not depend on them: request it first
  auto xload = [&](const uint8_t* qx, int s, int buf) __attribute__((always_inline)) {
    // activations: global -> LDS without passing through registers; one 1-KiB fragment per
    // wave-wide load, XCOPY fragments per wave and stage
#pragma unroll
    for (int f = 0; f < XCOPY; ++f) {
      const int idx = wave * XCOPY + f;          // fragment (b, j) = (idx / S, idx % S)
      const int b = idx / S, j = idx - b * S;
      if constexpr (CONV) {
        // 64-k step s*S + j of the tap-major k axis: tap (r, q), channels c0 .. c0 + 63 (C is a multiple of
        // 64).  The stages of a pass are requested in order, so the position is stepped, not divided out.
        if (s == 0) {
          const int tap = (j * 64) / p.cC;
          c_c0[f] = j * 64 - tap * p.cC;
          c_r[f] = tap / p.ckw;
          c_q[f] = tap - c_r[f] * p.ckw;
        } else {
          c_c0[f] += S * 64;
          while (c_c0[f] >= p.cC) {
            c_c0[f] -= p.cC;
            if (++c_q[f] == p.ckw) { c_q[f] = 0; ++c_r[f]; }
          }
        }
        const int r = c_r[f], q = c_q[f], c0 = c_c0[f];
        const bool inside = r < p.ckh && (unsigned)(c_h0[f] + r) < (unsigned)p.cH && (unsigned)(c_w0[f] + q) < (unsigned)p.cW;
        const int8_t* g = inside ? p.cq8 + (c_off[f] + (r * p.cW + q) * p.cC + c0) : reinterpret_cast<const int8_t*>(p.czero);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                         (__attribute__((address_space(3))) void*)&Xs[buf][idx * FRAG], 16, 0, 0);
      } else {
        const uint4* g = reinterpret_cast<const uint4*>(qx + ((size_t)(t0 / 16 + b) * p.nks + (size_t)s * S + j) * 1024) + lane;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                         (__attribute__((address_space(3))) void*)&Xs[buf][idx * FRAG], 16, 0, 0);
      }
    }
  };
  xload(p.qx, 0, 0);   // member 0 owns order 1, which every tile holds
  // tile_cnt: passes each member runs in this column tile (one byte per member); rb_out: output
  // row blocks of this wave's NRW sorted positions.  Scalar loads; member 0's activation scale
  // and code sums (vector loads) travel at the same time.
  static_assert(NRW == 4, "descriptor loads are 4 wide");
  const v4i tile_cnt = cload(reinterpret_cast<const v4i*>(p.ct_cnt), (size_t)ct);
  const v4i rb_out4 = cload(reinterpret_cast<const v4i*>(p.rb_out), (size_t)(ct * NRB_WG + wave * NRW) / 4);
  const int rb_out[NRW] = {rb_out4[0], rb_out4[1], rb_out4[2], rb_out4[3]};
  float sx = p.s_x[0];
  int rs[MTB];
  if constexpr (CONV) {
    // token code sum = the channel sums of the window's pixels that lie inside the image
#pragma unroll
    for (int b = 0; b < MTB; ++b) {
      int sum = 0;
      if (OFF) {
        const int t = t0 + b * 16 + (lane & 15);
        const int wo = t % p.cWo, ho = (t / p.cWo) % p.cHo, img = t / (p.cWo * p.cHo);
        const int h0 = ho * p.cstride - p.cpad, w0 = wo * p.cstride - p.cpad;
        if (t < p.T)
          for (int r = 0; r < p.ckh; ++r)
            for (int q = 0; q < p.ckw; ++q)
              if ((unsigned)(h0 + r) < (unsigned)p.cH && (unsigned)(w0 + q) < (unsigned)p.cW)
                sum += p.ccsum[(img * p.cH + h0 + r) * p.cW + w0 + q];
      }
      rs[b] = sum;
    }
  } else {
#pragma unroll
    for (int b = 0; b < MTB; ++b) rs[b] = OFF ? p.rowsum[t0 + b * 16 + (lane & 15)] : 0;
  }

  const bool fold_sx = p.reduce && p.M > 1;   // multi-member sum: fold s_x into the row scale
  const unsigned scl_lane = (unsigned)(uintptr_t)(__attribute__((address_space(3))) float*)&Scl[wave][0] + (lane >> 4) * 16;
  float yacc[NRW][MTB][4];
#pragma unroll
  for (int r = 0; r < NRW; ++r)
#pragma unroll
    for (int b = 0; b < MTB; ++b)
#pragma unroll
      for (int i = 0; i < 4; ++i) yacc[r][b][i] = 0.f;

  bool x0_requested = true;    // stage 0 of the next order to run is already on its way to LDS buffer 0
  for (int m = 0; m < p.M; ++m) {
    const uint8_t* qx = p.qx + (size_t)m * p.qx_mstride;
    const int32_t* rowsum = p.rowsum + (size_t)m * p.rowsum_mstride;
    if (m > 0) {
      sx = p.s_x[m * p.sx_mstride];
      if constexpr (!CONV) {   // the members of a convolution layer share its input: their code sums stay
#pragma unroll
        for (int b = 0; b < MTB; ++b) rs[b] = OFF ? rowsum[t0 + b * 16 + (lane & 15)] : 0;
      }
    }

    // In pass j every row block of the tile contributes its j-th stored order of this member (all
    // of a member's orders multiply the same Q(x)); the tile runs as many passes as its fullest
    // row block has orders.  Uniform over the workgroup.
    const int cnt_word = m < 4 ? tile_cnt[0] : (m < 8 ? tile_cnt[1] : (m < 12 ? tile_cnt[2] : tile_cnt[3]));
    const int n_pass = (cnt_word >> (8 * (m & 3))) & 255;
    for (int k = 0; k < n_pass; ++k) {
      const uint8_t* pk = p.codes;
      const float* sck = p.scales;
      const v4i src4 = cload(reinterpret_cast<const v4i*>(p.rb_src), ((size_t)(m * p.p_max + k) * p.n_sorted + ct * NRB_WG + wave * NRW) / 4);
      const int src[NRW] = {src4[0], src4[1], src4[2], src4[3]};
      const uint8_t* wb[NRW];
      bool active = false;
#pragma unroll
      for (int r = 0; r < NRW; ++r) {
        active |= src[r] >= 0;
        // a pruned row block among live ones reads row block 0; its result is dropped
        wb[r] = pk + (size_t)(src[r] < 0 ? 0 : src[r]) * nksup * 1024;
      }

      v4i acc[NRW][MTB];
#pragma unroll
      for (int r = 0; r < NRW; ++r)
#pragma unroll
        for (int b = 0; b < MTB; ++b) acc[r][b] = v4i{0, 0, 0, 0};

      WRegs<BITS> w0[NRW], w1[NRW];
      auto gload_w = [&](int s, WRegs<BITS>(&w)[NRW]) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < NRW; ++r)
#pragma unroll
          for (int q = 0; q < WN; ++q) w[r].v[q] = gload16(wb[r] + (size_t)(s * WN + q) * 1024 + lane * 16);
      };
      // One stage: wait for this stage's tiles, prefetch the next stage, multiply this one.
      // The LDS reads are issued by hand (the compiler cannot tell the two LDS buffers apart and
      // would otherwise wait for the just-issued prefetch before every read); each 64-k step
      // reads the next step's fragments while the MFMAs of the current one run.
      auto stage = [&](int s, auto bufc, WRegs<BITS>(&cur)[NRW], WRegs<BITS>(&nxt)[NRW]) __attribute__((always_inline)) {
        constexpr int buf = decltype(bufc)::value;
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's LDS-direct loads have landed
        __syncthreads();                      // everyone's have, and buffer buf^1 is free again
        if (s + 1 < n_stage) {
          xload(qx, s + 1, buf ^ 1);
          if (active) gload_w(s + 1, nxt);
        }
        if (s == 0 && active) {
          // row scales of this order -> LDS (one 4-byte LDS-direct load per lane), read at the fold
#pragma unroll
          for (int g = 0; g < (16 * NRW + 63) / 64; ++g) {
            const int e = g * 64 + lane, r = e >> 4;
            // src[r] for a lane-dependent r, written so that it stays a handful of selects on
            // scalar registers (an indexed array would be placed in scratch memory)
            int sr = 0;
#pragma unroll
            for (int q = 0; q < NRW; ++q) sr |= (r == q) ? (src[q] < 0 ? 0 : src[q]) : 0;
            const float* gp = sck + (size_t)sr * 16 + (e & 15);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gp,
                                             (__attribute__((address_space(3))) void*)&Scl[wave][g * 64], 4, 0, 0);
          }
        }
        if (active) {
          // Software pipeline of the S 64-k steps.  A wave issues in order, so everything that is
          // not an MFMA has to sit in the shadow of one: the fragments of step j+1 are requested
          // before step j's MFMAs start (two register sets), and the codes of row block r+1 are
          // widened between the MFMAs of row block r (two register sets).
          constexpr int XB = (BITS == 4 && MTB == 4) ? 1 : 2;   // the widest 4-bit variant has no registers for a second set
          v4i xf[XB][MTB];
          v4i wf[2];
          lds_read_frags<MTB, (buf * MTB * S) * 1024, S * 1024>(xs_lane, xf[0]);
          wf[0] = widen<BITS>(cur[0], 0);
#pragma unroll
          for (int j = 0; j < S; ++j) {
            if (XB == 2 && j + 1 < S) {
              lds_read_frags<MTB, (buf * MTB * S) * 1024, S * 1024>(xs_lane + (j + 1) * 1024, xf[(j + 1) % XB]);
              lds_wait<MTB, MTB>(xf[j % XB]);
            } else {
              lds_wait<MTB, 0>(xf[j % XB]);
            }
#pragma unroll
            for (int r = 0; r < NRW; ++r) {
              if (r + 1 < NRW) wf[(r + 1) & 1] = widen<BITS>(cur[r + 1], j);
              else if (j + 1 < S) wf[(r + 1) & 1] = widen<BITS>(cur[0], j + 1);
#pragma unroll
              for (int b = 0; b < MTB; ++b)
                acc[r][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf[r & 1], xf[j % XB][b], acc[r][b], 0, 0, 0);
              if (BITS != 8) {
                // one MFMA, then two of the unpack instructions, and so on
#pragma unroll
                for (int b = 0; b < MTB; ++b) {
                  __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                  __builtin_amdgcn_sched_group_barrier(0x002, 8 / MTB, 0);
                }
              }
              __builtin_amdgcn_sched_barrier(0);   // keep the row blocks apart: bounds live registers
            }
            // single set: the next step's fragments follow the last MFMAs that read this one's
            if (XB == 1 && j + 1 < S) lds_read_frags<MTB, (buf * MTB * S) * 1024, S * 1024>(xs_lane + (j + 1) * 1024, xf[0]);
          }
        }
      };

      if (!x0_requested) xload(qx, 0, 0);
      x0_requested = false;
      if (active) gload_w(0, w0);
      int s = 0;
      for (; s + 1 < n_stage; s += 2) {
        stage(s, std::integral_constant<int, 0>{}, w0, w1);
        stage(s + 1, std::integral_constant<int, 1>{}, w1, w0);
      }
      if (s < n_stage) stage(s, std::integral_constant<int, 0>{}, w0, w1);
      if (n_stage == 1) __builtin_amdgcn_s_waitcnt(0x0F70);   // the scales were requested in this very stage
      __syncthreads();

      // fold this order: yacc += s_k[o] * float(acc - OFF * rowsum)
#pragma unroll
      for (int r = 0; r < NRW; ++r) {
        if (src[r] < 0) continue;
        float4 sc;
        asm volatile("ds_read_b128 %0, %1 offset:%2\n\ts_waitcnt lgkmcnt(0)" : "=v"(sc) : "v"(scl_lane), "n"(r * 64) : "memory");
        float scv[4] = {sc.x, sc.y, sc.z, sc.w};
        if (fold_sx) {
#pragma unroll
          for (int i = 0; i < 4; ++i) scv[i] *= sx;
        }
#pragma unroll
        for (int b = 0; b < MTB; ++b) {
          const int t = t0 + b * 16 + (lane & 15);
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
    if (fold_sx && m + 1 < p.M) continue;   // keep accumulating into the same running sum
    // member (or final) epilogue.  The MFMA result layout gives a lane 4 channels of one token, so
    // a direct store would touch 16 tokens x 64 B per instruction.  Each 16-token block is instead
    // turned through this wave's 4 KiB of the idle LDS buffer 1 (XOR-swizzled, conflict free) so
    // that one store instruction writes 4 tokens x 256 contiguous bytes: whole cache lines.
    // The LDS accesses are issued by hand: left to the compiler, every read would first wait
    // for the previous global store to complete (it orders LDS accesses against all outstanding
    // vector-memory operations of a kernel that uses LDS-direct loads), serializing the stores.
    float mx = 0.f, mn = 0.f;
    const bool two_sided = p.amax_neg != nullptr;
    {
      int lane_e = lane;
      asm volatile("" : "+v"(lane_e));   // keeps the epilogue's address arithmetic out of the main loop's live range
      const int tl = lane_e & 15, g = lane_e >> 4;
      auto stg_of = [&](int w) __attribute__((always_inline)) {
        return (unsigned)(uintptr_t)(__attribute__((address_space(3))) uint4*)(MTB == 4 ? &Xs[1][w * 256] : &Stg[(MTB == 4 ? 0 : w) * 256]);
      };
      const unsigned stg = stg_of(wave);
      const unsigned wr_row = stg + tl * 256;                    // this lane's token row when writing
      int rb_l = rb_out[0];                                      // row block of the channels this lane stores
#pragma unroll
      for (int q = 1; q < NRW; ++q) rb_l = (tl >> 2) == q ? rb_out[q] : rb_l;
      const int ch = rb_l * 16 + 4 * (tl & 3);
      // gate||up layer: waves 0,1 hold gate blocks, waves 2,3 the matching up blocks (rb_l is the
      // block of the hidden channel for both); the up waves finish h = SiLU(gate) * up
      const bool is_up = MODE == MODE_GATED && wave >= 2;
      float4 bv = make_float4(0.f, 0.f, 0.f, 0.f), bg = make_float4(0.f, 0.f, 0.f, 0.f);
      if (rb_l >= 0 && (m == 0 || fold_sx || p.bias_mstride != 0) && p.bias != nullptr) {
        const float* bm = p.bias + (size_t)m * p.bias_mstride;
        bv = *reinterpret_cast<const float4*>(bm + ch + (is_up ? p.hidden : 0));
        if (is_up) bg = *reinterpret_cast<const float4*>(bm + ch);
      }
      const float bb[4] = {bv.x, bv.y, bv.z, bv.w};
      const float bgate[4] = {bg.x, bg.y, bg.z, bg.w};
      // the bias has to have arrived before the first (conditional) store block: a wait placed
      // inside those blocks would be repeated in each and then also wait for the stores before it
      __builtin_amdgcn_s_waitcnt(0x0F70);
      float* ycol = p.y + (size_t)(p.reduce ? 0 : m) * p.T * p.out + ch;
      // skip tensor: the members summed into this output each add their own (members kept
      // apart: member m adds its own if it has one)
      const int n_res = (MODE == MODE_CHAIN && p.res != nullptr) ? (fold_sx || p.reduce ? p.res_members : (m < p.res_members ? 1 : 0)) : 0;
      const float* rcol = MODE == MODE_CHAIN ? p.res + (size_t)(p.reduce ? 0 : m) * p.res_mstride + max(ch, 0) : nullptr;
#pragma unroll
      for (int b = 0; b < MTB; ++b) {
        float4 rq[4];
        if (MODE == MODE_CHAIN) {
#pragma unroll
          for (int q = 0; q < 4; ++q) rq[q] = make_float4(0.f, 0.f, 0.f, 0.f);
          for (int mm = 0; mm < n_res; ++mm) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const int tc = min(t0 + b * 16 + 4 * q + g, p.T - 1);   // clamped: loaded unconditionally
              const float4 r = *reinterpret_cast<const float4*>(rcol + (size_t)mm * p.res_mstride + (size_t)tc * p.out);
              rq[q].x += r.x; rq[q].y += r.y; rq[q].z += r.z; rq[q].w += r.w;
            }
          }
        }
#pragma unroll
        for (int r = 0; r < NRW; ++r) {
          const v4f val = v4f{yacc[r][b][0], yacc[r][b][1], yacc[r][b][2], yacc[r][b][3]};
          asm volatile("ds_write_b128 %0, %1" ::"v"(wr_row + (((r * 4 + g) ^ tl) << 4)), "v"(val) : "memory");
#pragma unroll
          for (int i = 0; i < 4; ++i) yacc[r][b][i] = 0.f;
        }
        if (MODE == MODE_GATED) {
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wave's block is in LDS ...
          __syncthreads();                                     // ... and so is its partner's
        }
        v4f a[4];
        if (MODE != MODE_GATED) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int tq = 4 * q + g;
            asm volatile("ds_read_b128 %0, %1" : "=v"(a[q]) : "v"(stg + tq * 256 + ((tl ^ tq) << 4)) : "memory");
          }
          asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3])::"memory");
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if (MODE == MODE_GATED && !is_up) break;
          const int t = t0 + b * 16 + 4 * q + g;
          v4f ga;
          if (MODE == MODE_GATED) {
            // one token row at a time: the up block from this wave's space, the gate block from its partner's
            const int tq = 4 * q + g;
            asm volatile("ds_read_b128 %0, %1" : "=v"(a[q]) : "v"(stg + tq * 256 + ((tl ^ tq) << 4)) : "memory");
            asm volatile("ds_read_b128 %0, %1" : "=v"(ga) : "v"(stg_of(wave ^ 2) + tq * 256 + ((tl ^ tq) << 4)) : "memory");
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a[q]), "+v"(ga)::"memory");
          }
          float v[4] = {a[q][0], a[q][1], a[q][2], a[q][3]};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            v[i] = fold_sx ? v[i] + bb[i] : fmaf(sx, v[i], bb[i]);   // same rounding as the streaming kernel
            if (MODE == MODE_GELU) v[i] = gelu_erf(v[i]);
            if (MODE == MODE_CHAIN) {
              const float r = i == 0 ? rq[q].x : i == 1 ? rq[q].y : i == 2 ? rq[q].z : rq[q].w;
              if (p.res_pre_act) v[i] += r;
              if (p.act == PIPE_ACT_RELU) v[i] = fmaxf(v[i], 0.f);
              else if (p.act == PIPE_ACT_GELU) v[i] = gelu_erf(v[i]);
              if (!p.res_pre_act) v[i] += r;
            }
            if (MODE == MODE_GATED) {
              const float gte = fmaf(sx, ga[i], bgate[i]);
              v[i] = gte / (1.f + expf(-gte)) * v[i];
            }
          }
          if (t < p.T && rb_l >= 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              mx = fmaxf(mx, two_sided ? v[i] : fabsf(v[i]));
              if (two_sided) mn = fmaxf(mn, -v[i]);
            }
            *reinterpret_cast<float4*>(ycol + (size_t)t * p.out) = make_float4(v[0], v[1], v[2], v[3]);
          }
        }
        if (MODE == MODE_GATED) __syncthreads();   // both blocks have been read: the staging space is free again
      }
    }
    if (p.amax_out != nullptr) {
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
      if (lane == 0) amax_raise(&p.amax_out[m], mx);
      if (two_sided) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) mn = fmaxf(mn, __shfl_xor(mn, o, 64));
        if (lane == 0) amax_raise(&p.amax_neg[m], mn);
      }
    }
  }  // members
}

template <int BITS, int MTB, int NRW, int MINW>
int launch_cfg(TiledParams& p, bool acc_out, hipEvent_t ev0, hipEvent_t ev1, hipStream_t st) {
  p.n_tt = ceil_div(p.T, 16 * MTB);
  p.n_ct = ceil_div(p.n_ct * NRB_TILE, 4 * NRW);   // column tiles of this variant's width
  // Super-tiles are dealt to the 8 XCDs in turn, column-tile rows (heaviest first) outermost.  With
  // 8 token super-tiles per row every XCD gets a share of every row; with 4 (e.g. 2048 tokens)
  // the even rows would all land on XCDs 0-3 and the odd rows on 4-7, the heavier half finishing
  // last: then 16 x 4 super-tiles restore 8 per row.
  p.st_c_log2 = 3;
  if (ceil_div(p.n_tt, 8) % 8 != 0 && ceil_div(p.n_tt, 4) % 8 == 0) p.st_c_log2 = 4;
  p.n_st_t = ceil_div(p.n_tt, 64 >> p.st_c_log2);
  const int n_st_c = ceil_div(p.n_ct, 1 << p.st_c_log2);
  // super-tile sidx runs on XCD sidx % 8 as blocks xcd + 8*(64*(sidx/8) + local), local = 0..63
  const dim3 grid((unsigned)(ceil_div(p.n_st_t * n_st_c, 8) * 8 * 64));
  if (p.cq8 != nullptr) {
    // implicit-GEMM convolution: plain epilogue or the integer export
    if (p.res != nullptr || p.act != 0) return PIPE_EINVAL;
    if (acc_out)
      PIPE_LAUNCH((gemm_tiled_kernel<BITS, MTB, NRW, MINW, MODE_ACC_OUT, true>), grid, dim3(256), st, ev0, ev1, p);
    else
      PIPE_LAUNCH((gemm_tiled_kernel<BITS, MTB, NRW, MINW, MODE_PLAIN, true>), grid, dim3(256), st, ev0, ev1, p);
    PIPE_HIP(hipGetLastError());
    return PIPE_OK;
  }
  if (acc_out)
    PIPE_LAUNCH((gemm_tiled_kernel<BITS, MTB, NRW, MINW, MODE_ACC_OUT>), grid, dim3(256), st, ev0, ev1, p);
  else if (p.res != nullptr || p.act == PIPE_ACT_RELU)
    PIPE_LAUNCH((gemm_tiled_kernel<BITS, MTB, NRW, MINW, MODE_CHAIN>), grid, dim3(256), st, ev0, ev1, p);
  else if (p.act == PIPE_ACT_GELU)
    PIPE_LAUNCH((gemm_tiled_kernel<BITS, MTB, NRW, MINW, MODE_GELU>), grid, dim3(256), st, ev0, ev1, p);
  else if (p.act == PIPE_ACT_SILU_GATED)
    PIPE_LAUNCH((gemm_tiled_kernel<BITS, MTB, NRW, MINW, MODE_GATED>), grid, dim3(256), st, ev0, ev1, p);
  else
    PIPE_LAUNCH((gemm_tiled_kernel<BITS, MTB, NRW, MINW, MODE_PLAIN>), grid, dim3(256), st, ev0, ev1, p);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

}  // namespace

int launch_gemm_tiled(const GemmArgs& a, hipStream_t st) {
  const pipe_expansion* e = a.e;
  if (a.T <= 0) return PIPE_OK;
  if (a.T_pad % TOK_TILE != 0 || a.T_pad < a.T) return PIPE_ESHAPE;
  TiledParams p;
  p.qx = a.qx; p.qx_mstride = a.qx_mstride;
  p.rowsum = a.rowsum; p.rowsum_mstride = a.rowsum_mstride;
  p.s_x = a.s_x; p.sx_mstride = a.sx_mstride;
  p.codes = e->codes_dev; p.scales = e->scales_all_dev;
  p.bias = a.bias; p.bias_mstride = a.bias_mstride; p.y = a.y; p.acc_out = a.acc_out; p.amax_out = a.amax_out; p.amax_neg = a.amax_neg; p.zero_after = a.zero_after; p.zero_n = a.zero_n; p.zero_big = a.zero_big; p.zero_big_n = a.zero_big_n;
  p.T = a.T; p.out = e->out; p.K = e->K; p.nks = e->nks;
  p.M = a.M; p.reduce = a.reduce; p.act = a.act;
  p.hidden = 0;
  p.cq8 = a.conv_q8; p.ccsum = a.conv_csum; p.czero = a.conv_zero;
  p.cC = a.conv_C; p.cH = a.conv_H; p.cW = a.conv_W; p.ckh = a.conv_kh; p.ckw = a.conv_kw; p.cstride = a.conv_stride; p.cpad = a.conv_pad;
  p.cHo = a.conv_Ho; p.cWo = a.conv_Wo;
  if (a.conv_q8 != nullptr && (a.conv_C % 64 != 0 || (a.M > 1 && a.qx_mstride != 0))) return PIPE_ESHAPE;
  p.res = a.res; p.res_mstride = a.res_mstride; p.res_members = a.res_members; p.res_pre_act = a.res_pre_act;
  if (a.res != nullptr && (a.acc_out != nullptr || a.act == PIPE_ACT_SILU_GATED || a.res_members < 1 || a.res_members > a.M))
    return PIPE_EINVAL;
  if (a.act == PIPE_ACT_SILU_GATED) {
    // gate||up layer: the pair schedule; the output is the hidden activation, H wide, members apart
    if (a.reduce || a.acc_out != nullptr) return PIPE_EINVAL;
    p.hidden = e->out / 2;
    p.out = e->out / 2;
  }
  const bool acc_out = a.acc_out != nullptr;
  if (acc_out && a.M != 1) return PIPE_EINVAL;   // the integer export writes pass j as order j
  int rc = PIPE_OK;
  const PassTables* tb = pipe_get_tables(e, a, acc_out ? 2 : (a.act == PIPE_ACT_SILU_GATED ? 1 : 0), &rc);
  if (tb == nullptr) return rc;
  p.rb_out = tb->rb_out_dev; p.rb_src = tb->src_dev; p.ct_cnt = tb->cnt_dev; p.n_sorted = tb->n_sorted;
  p.p_max = tb->p_max; p.n_ct = tb->n_ct;
  // Token-tile height: the tallest of 64, 32, 16 tokens that still gives at least 1024 tiles (two
  // rounds of the 512 workgroups the chip holds), or whose tiles fill whole rounds (the last one
  // at least 7/8 full): taller tiles re-read the packed codes from L2 less often, but a round
  // that leaves compute units idle costs more than that (measured on the 11008 x 4096 ternary
  // layer, 192 to 3072 tokens, and on 2048 x 2048 layers at 4096 tokens).
  const int n_ct = p.n_ct;
  int mtb = g_tiled_mtb;
  if (mtb != 1 && mtb != 2 && mtb != 4) {
    auto fits = [&](int tokens) {
      const int64_t tiles = (int64_t)n_ct * ceil_div(a.T, tokens);
      const int64_t last = tiles % 512;
      return tiles >= 1024 || (tiles >= 448 && (last == 0 || last >= 448));
    };
    mtb = fits(64) ? 4 : (fits(32) ? 2 : 1);
  }
  switch (e->bits * 8 + mtb) {
    case 8 * 8 + 4: return launch_cfg<8, 4, 4, 1>(p, acc_out, a.ev_start, a.ev_stop, st);
    case 8 * 8 + 2: return launch_cfg<8, 2, 4, 2>(p, acc_out, a.ev_start, a.ev_stop, st);
    case 8 * 8 + 1: return launch_cfg<8, 1, 4, 2>(p, acc_out, a.ev_start, a.ev_stop, st);
    case 4 * 8 + 4: return launch_cfg<4, 4, 4, 2>(p, acc_out, a.ev_start, a.ev_stop, st);
    case 4 * 8 + 2: return launch_cfg<4, 2, 4, 2>(p, acc_out, a.ev_start, a.ev_stop, st);
    case 4 * 8 + 1: return launch_cfg<4, 1, 4, 2>(p, acc_out, a.ev_start, a.ev_stop, st);
    case 2 * 8 + 4: return launch_cfg<2, 4, 4, 2>(p, acc_out, a.ev_start, a.ev_stop, st);
    case 2 * 8 + 2: return launch_cfg<2, 2, 4, 2>(p, acc_out, a.ev_start, a.ev_stop, st);
    case 2 * 8 + 1: return launch_cfg<2, 1, 4, 2>(p, acc_out, a.ev_start, a.ev_stop, st);
    default: return PIPE_EINVAL;
  }
}
