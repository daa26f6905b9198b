// Weight-streaming kernel of the expanded layer for decode-sized batches (T <= 128), where the
// path is bound by reading the packed codes from HBM once (App. B, Eq. (define_dre), same
// arithmetic as the tiled kernel).
//
// Work item = one stored row block (16 rows of one order, all of in_features).  A workgroup
// owns a bin of items that together hold every order of a few output row blocks; its waves
// split the k dimension (wave w takes packed tiles w, w+NW, ...), so each wave streams its
// own 1-KiB tiles straight from HBM into registers with fully coalesced 16-byte loads, widens
// them with a shift and a mask and feeds v_mfma_i32_16x16x64_i8 against the 16-token
// activation fragments (also read straight from L2: waves use disjoint k, nothing is shared,
// so the k loop has no LDS traffic and no barrier).  The waves' partial int32 tiles meet in
// LDS and are summed exactly; the epilogue then applies offsets, row scales, activation scale,
// bias and the member sum in a fixed order, so results are bit-reproducible.  A workgroup
// handles one 16-token block; larger batches (up to 128 tokens) run one workgroup per bin and
// token block, on the same XCD, so that the bin still comes from HBM once.  Expansions with more
// than 4 orders have bins of 8, 12 or 16 items: gemm_stream_multi_kernel streams them four at a
// time and keeps the integer tiles of the whole bin in LDS for one epilogue.
#include "pipe_internal.h"

#include <algorithm>

int g_stream_ksplit = 0;   // 0: automatic

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
  const uint8_t* codes;    // stored row blocks in schedule order: bin b owns positions [b*cap, (b+1)*cap), cap = 4, 8, 12 or 16
  const float* scales;     // 16 row scales per position
  const StreamBin* bins;
  const float* bias;
  long long bias_mstride;  // 0: the first member's (or the sum's) vector; else one vector per member
  float* y;
  int32_t* acc_out;
  uint32_t* amax_out;
  uint32_t* amax_neg;      // if set: positive and negative parts of the range apart
  const float* res;        // skip tensor [res_members, T, out] or nullptr
  long long res_mstride;
  int res_members, res_pre_act;
  uint32_t* zero_after;
  int zero_n;
  uint32_t* zero_big;
  int zero_big_n;
  int T, out, K, nks, M, reduce, act;
  int ksplit;              // workgroups per bin: each takes a contiguous share of the k tiles
  int n_tb;                // 16-token blocks: one workgroup per (bin, k share, token block)
  int n_bins;
  int thr0, thr1, thr2;    // bins of 4, fullest first: how many hold 4, at least 3, at least 2 items
  int zero_pos;            // an all-zero position (codes and scales): read for the items a bin does not have
  const float* x_f32;      // QFUSE: the fp32 input [T, in] (T <= 4), quantized by every workgroup itself
  float s_static;          // QFUSE: given activation scale, or <= 0 for max|x| / act_qmax
  float act_qmax;          // QFUSE: largest activation code
  int in;                  // QFUSE: in_features (multiple of 4)
  int32_t* ws_sum;         // [n_bins][ksplit][cap][256] partial tiles of split bins
  uint32_t* ws_cnt;        // [n_bins] arrival counters, zero between launches
  int member_lo[PIPE_MAX_K];
  int member_hi[PIPE_MAX_K];
  int member_of[PIPE_MAX_K];
};

// uniform dynamic index into a kernel-argument array without forcing it into scratch memory
template <class T>
__device__ __forceinline__ T pick(const T (&a)[PIPE_MAX_K], int k) {
  T v = a[0];
#pragma unroll
  for (int i = 1; i < PIPE_MAX_K; ++i) v = (i == k) ? a[i] : v;
  return v;
}

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

// XM = number of distinct activation tensors the items of a bin can read: 1 (one input for all
// orders), or 2 / 4 (one input per ensemble member, at most XM members).
// XMASK: the batch does not fill its last 16-token block; the activation loads of that block are
// issued for the lanes of real tokens only.
// QFUSE (a single token, one activation tensor): there is no quantizer launch; every
// workgroup reduces max|x| over the few-KiB input itself, quantizes it into LDS with the same
// arithmetic as the quantizer kernels (IEEE division, round half to even) while its first codes are
// on their way, and builds its activation fragments from there.
constexpr int QF_T = 1, QF_IN = 8192;
template <int BITS, int NW, int XM, bool ACC_OUT, bool XMASK, bool QFUSE = false>
__global__ __launch_bounds__(NW * 64, (XM * (BITS == 2 ? 4 : (BITS == 4 ? 2 : 1)) <= 4) ? 4 : 2) void gemm_stream_kernel(const StreamParams p) {
  static_assert(!QFUSE || (XM == 1 && !ACC_OUT), "the fused quantizer serves one shared input");
  __shared__ __attribute__((aligned(16))) uint8_t s_qx[QFUSE ? QF_T * QF_IN : 16];
  __shared__ float s_red[NW];
  __shared__ int s_rs[QF_T];
  constexpr int OFF = BITS == 8 ? 0 : (BITS == 4 ? 8 : 1);
  constexpr int KSUP = 512 / BITS;
  constexpr int STEPS = KSUP / 64;      // 64-k steps per packed tile
  constexpr int NX = XM * STEPS;
  constexpr int BIN_WORDS = sizeof(StreamBin) / 4;
  static_assert(BIN_WORDS <= 64, "bin descriptor is fetched with one load per lane");
  __shared__ int part[NW][R][256];   // each wave's partial tiles
  __shared__ int s_last;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n_tiles = (p.nks * 64) / KSUP;
  if (blockIdx.x == 0 && (int)threadIdx.x < p.zero_n && p.zero_after != nullptr) p.zero_after[threadIdx.x] = 0u;
  if (p.zero_big != nullptr)
    for (int i = blockIdx.x * (NW * 64) + threadIdx.x; i < p.zero_big_n; i += gridDim.x * (NW * 64)) p.zero_big[i] = 0u;

  // Block index -> (bin, k share, token block).  Blocks are handed to the XCDs round robin, so the
  // workgroups that stream the same bin (for different token blocks or k shares) get indices that
  // are equal modulo 8: they run on one XCD and the bin comes from HBM once, then from that L2.
  const int subs = p.ksplit * p.n_tb;
  const int grp = (int)blockIdx.x / (8 * subs), within = (int)blockIdx.x - grp * (8 * subs);
  const int bin = grp * 8 + (within & 7), sub = within >> 3;
  const int ksp = sub % p.ksplit, tb = sub / p.ksplit;
  if (bin >= p.n_bins) return;   // padding of the last group of eight bins

  // epilogue role of this thread: 256 threads per output row block, thread = (token t, channel ch)
  const int e = threadIdx.x & 255;
  const int t = e >> 4, ch = e & 15;   // token inside this workgroup's 16-token block
  const int tg = tb * 16 + t;          // token of the call
  const int fidx = ((ch >> 2) * 16 + t) * 4 + (ch & 3);   // lane*4 + i of the MFMA result layout
  const int o_first = __builtin_amdgcn_readfirstlane(threadIdx.x >> 8);
  constexpr int O_STEP = (NW * 64) / 256;
  const bool fold_sx = p.reduce && p.M > 1;

  // ---- everything that does not depend on the bin descriptor is requested first: where the bin's
  // stored row blocks sit in the schedule-ordered buffers follows from the bin's index (below), so
  // the code stream (the HBM traffic that bounds this kernel) starts at once.  Wave w streams
  // tiles w, w+NW, ...; two tiles per item are in flight.
  // this workgroup's share of the k tiles
  const int tile_lo = (int)((long long)n_tiles * ksp / p.ksplit), tile_hi = (int)((long long)n_tiles * (ksp + 1) / p.ksplit);
  // the bin's first position and item count, from its index: the bins lie without gaps, fullest first
  const int b3 = max(bin - p.thr0, 0), b2 = max(bin - p.thr1, 0), b1 = max(bin - p.thr2, 0);
  const int n_here = bin < p.thr0 ? 4 : (bin < p.thr1 ? 3 : (bin < p.thr2 ? 2 : 1));
  const int pos0 = 4 * bin - b3 - b2 - b1;
  size_t posr[R];
#pragma unroll
  for (int r = 0; r < R; ++r) posr[r] = (size_t)(r < n_here ? pos0 + r : p.zero_pos);
  const uint8_t* wb[R];
#pragma unroll
  for (int r = 0; r < R; ++r) wb[r] = p.codes + posr[r] * (size_t)n_tiles * 1024;
  const int d0 = lane < BIN_WORDS ? reinterpret_cast<const int32_t*>(p.bins + bin)[lane] : 0;
  uint4 w0[R], w1[R], x0[NX], x1[NX];
  auto load_w = [&](int tl, uint4 (&w)[R]) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < R; ++r) w[r] = reinterpret_cast<const uint4*>(wb[r] + (size_t)tl * 1024)[lane];
  };
  // member m's activations (members beyond M repeat the last one; never used)
  const uint8_t* xb[XM];
#pragma unroll
  for (int m = 0; m < XM; ++m) xb[m] = p.qx + (size_t)(m < p.M ? m : p.M - 1) * p.qx_mstride + (size_t)tb * p.nks * 1024;
  // lanes of tokens beyond the batch keep the zeros they start with: their codes are zero anyway, and
  // a load instruction costs the memory pipeline only its active lanes (one token in sixteen at T = 1)
  const bool xlive = tb * 16 + (lane & 15) < p.T;
  const bool xfull = !XMASK || tb * 16 + 16 <= p.T;   // uniform: a whole block needs no lane mask
  const int in_pad_q = p.nks * 64;
  auto load_x = [&](int tl, uint4 (&x)[NX]) __attribute__((always_inline)) {
    if constexpr (QFUSE) {
      // the fragment of a 64-k step: lane (kc, n) holds codes 16 kc .. 16 kc + 15 of token n
      if ((lane & 15) < p.T) {
#pragma unroll
        for (int j = 0; j < STEPS; ++j)
          x[j] = *reinterpret_cast<const uint4*>(&s_qx[(size_t)(lane & 15) * in_pad_q + (size_t)(tl * STEPS + j) * 64 + (lane >> 4) * 16]);
      }
    } else if (xfull) {
#pragma unroll
      for (int m = 0; m < XM; ++m)
#pragma unroll
        for (int j = 0; j < STEPS; ++j) x[m * STEPS + j] = reinterpret_cast<const uint4*>(xb[m] + (size_t)(tl * STEPS + j) * 1024)[lane];
    } else if (xlive) {
#pragma unroll
      for (int m = 0; m < XM; ++m)
#pragma unroll
        for (int j = 0; j < STEPS; ++j) x[m * STEPS + j] = reinterpret_cast<const uint4*>(xb[m] + (size_t)(tl * STEPS + j) * 1024)[lane];
    }
  };
#pragma unroll
  for (int j = 0; j < NX; ++j) { x0[j] = make_uint4(0, 0, 0, 0); x1[j] = make_uint4(0, 0, 0, 0); }
  int tl = tile_lo + wave;
  if (tl < tile_hi) { load_w(tl, w0); if (!QFUSE) load_x(tl, x0); }
  if (tl + NW < tile_hi) { load_w(tl + NW, w1); if (!QFUSE) load_x(tl + NW, x1); }
  // epilogue operands that need no descriptor: row scales (same positions), and per member the
  // activation scale and this thread's token code sum
  float scv[R];
#pragma unroll
  for (int r = 0; r < R; ++r) scv[r] = p.scales[posr[r] * 16 + ch];
  float sxm[R];
  int rsm[R];
  if constexpr (!QFUSE) {
#pragma unroll
    for (int m = 0; m < R; ++m) {       // at most R members (K <= R)
      const int mm = m < p.M ? m : p.M - 1;
      sxm[m] = p.s_x[mm * p.sx_mstride];
      rsm[m] = OFF ? p.rowsum[(size_t)mm * p.rowsum_mstride + tg] : 0;
    }
  } else {
    // ---- quantize the input here (the codes already requested are on their way meanwhile)
    const int in = p.in;
    const float4* x4 = reinterpret_cast<const float4*>(p.x_f32);
    const int n4 = (p.T * in) >> 2;
    if ((int)threadIdx.x < QF_T) s_rs[threadIdx.x] = 0;
    float s_act = p.s_static;
    if (!(s_act > 0.f)) {
      float mx = 0.f;
      for (int i = threadIdx.x; i < n4; i += NW * 64) {
        const float4 v = x4[i];
        mx = fmaxf(mx, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
      if (lane == 0) s_red[wave] = mx;
      __syncthreads();
      mx = s_red[0];
#pragma unroll
      for (int w = 1; w < NW; ++w) mx = fmaxf(mx, s_red[w]);
      s_act = __fdiv_rn(mx, p.act_qmax);
    } else {
      __syncthreads();   // the cleared code sums
    }
    const bool live_q = s_act > 0.f;
    auto q1 = [&](float v) __attribute__((always_inline)) {
      const float q = fminf(fmaxf(rintf(__fdiv_rn(v, s_act)), -p.act_qmax), p.act_qmax);
      return live_q ? (int)q : 0;
    };
    for (int i = threadIdx.x; i < n4; i += NW * 64) {
      const float4 v = x4[i];
      const int tq = (i * 4) / in, k = i * 4 - tq * in;   // in is a multiple of 4: one token per float4
      const int a = q1(v.x), b = q1(v.y), c = q1(v.z), d = q1(v.w);
      *reinterpret_cast<uint32_t*>(&s_qx[(size_t)tq * in_pad_q + k]) =
          (uint32_t)(uint8_t)a | ((uint32_t)(uint8_t)b << 8) | ((uint32_t)(uint8_t)c << 16) | ((uint32_t)(uint8_t)d << 24);
      const int sum4 = a + b + c + d;
      if (sum4 != 0) atomicAdd(&s_rs[tq], sum4);
    }
    // codes beyond in_features are zero
    const int pad4 = (in_pad_q - in) >> 2;
    for (int i = threadIdx.x; i < p.T * pad4; i += NW * 64) {
      const int tq = i / pad4, k = in + (i - tq * pad4) * 4;
      *reinterpret_cast<uint32_t*>(&s_qx[(size_t)tq * in_pad_q + k]) = 0u;
    }
    __syncthreads();
    const int rs_q = (OFF && tg < p.T) ? s_rs[min(tg, QF_T - 1)] : 0;
#pragma unroll
    for (int m = 0; m < R; ++m) { sxm[m] = s_act; rsm[m] = rs_q; }
    if (tl < tile_hi) load_x(tl, x0);
    if (tl + NW < tile_hi) load_x(tl + NW, x1);
  }

  // ---- the descriptor: scalar reads out of one vector register
  auto word = [&](int i) __attribute__((always_inline)) { return __builtin_amdgcn_readlane(d0, i); };
  const int n_items = word(0), n_out = word(1);
  int itk[R], its[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const bool on = r < n_items;
    itk[r] = word(2 + (on ? r : 0));
    its[r] = on ? word(2 + STREAM_BIN_CAP + r) : -1;
  }
  auto out_rb = [&](int o) __attribute__((always_inline)) { return word(2 + 2 * STREAM_BIN_CAP + o); };
  int itm[R];   // which activation tensor item r reads
#pragma unroll
  for (int r = 0; r < R; ++r) itm[r] = XM == 1 ? 0 : pick(p.member_of, itk[r]);

  v4i acc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = v4i{0, 0, 0, 0};
  auto mul_tile = [&](uint4 (&w)[R], uint4 (&x)[NX]) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < STEPS; ++j) {
#pragma unroll
      for (int r = 0; r < R; ++r) {
        v4i xf = v4i{(int)x[j].x, (int)x[j].y, (int)x[j].z, (int)x[j].w};
#pragma unroll
        for (int m = 1; m < XM; ++m) {   // uniform select, component by component
          const bool pickm = itm[r] == m;
          xf[0] = pickm ? (int)x[m * STEPS + j].x : xf[0];
          xf[1] = pickm ? (int)x[m * STEPS + j].y : xf[1];
          xf[2] = pickm ? (int)x[m * STEPS + j].z : xf[2];
          xf[3] = pickm ? (int)x[m * STEPS + j].w : xf[3];
        }
        v4i wf;
        unpack_step<BITS>(w[r], j, wf);
        acc[r] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf, xf, acc[r], 0, 0, 0);
      }
    }
  };
  for (; tl < tile_hi; tl += 2 * NW) {
    mul_tile(w0, x0);
    if (tl + 2 * NW < tile_hi) { load_w(tl + 2 * NW, w0); load_x(tl + 2 * NW, x0); }
    if (tl + NW < tile_hi) {
      mul_tile(w1, x1);
      if (tl + 3 * NW < tile_hi) { load_w(tl + 3 * NW, w1); load_x(tl + 3 * NW, x1); }
    }
  }
#pragma unroll
  for (int r = 0; r < R; ++r)
    *reinterpret_cast<v4i*>(&part[wave][r][lane * 4]) = acc[r];
  __syncthreads();

  // A split bin: every workgroup writes its integer partial tiles to its own slice of the bin's
  // workspace with device-scope stores (written through to memory, no cache maintenance), waits
  // for them to complete (vmcnt counts stores) and then counts its arrival; the one that arrives
  // last reads all slices with device-scope loads, sums them (exact, order independent), resets
  // the counter and runs the epilogue.  Nobody waits for anybody.
  // What this relies on is the hardware's behaviour, not the language's memory model (all accesses
  // are relaxed): a device-scope store is written through to the memory-side cache all compute
  // units share, s_waitcnt vmcnt(0) returns only once every such store of the wave has been
  // acknowledged from there, the barrier extends that to the workgroup, and only then is the
  // counter raised; the reader's device-scope loads bypass its own caches.  A release/acquire pair
  // on the counter would express the same order in the model; its cache write-back and invalidate
  // measured 11 to 34 us per exchange on this chip, more than the kernel.
  if (p.ksplit > 1) {
    int32_t* ws = p.ws_sum + ((size_t)bin * p.ksplit + ksp) * (R * 256);
    for (int i = threadIdx.x; i < R * 256; i += NW * 64) {
      int a = 0;
#pragma unroll
      for (int w = 0; w < NW; ++w) a += (&part[w][0][0])[i];
      __hip_atomic_store(&ws[i], a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    if (threadIdx.x == 0) s_last = atomicAdd(&p.ws_cnt[bin], 1u) == (unsigned)(p.ksplit - 1);
    __syncthreads();
    if (!s_last) return;
    const int32_t* wsb = p.ws_sum + (size_t)bin * p.ksplit * (R * 256);
    for (int i = threadIdx.x; i < R * 256; i += NW * 64) {
      int a = 0;
      for (int q = 0; q < p.ksplit; ++q) a += __hip_atomic_load(&wsb[(size_t)q * (R * 256) + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      (&part[0][0][0])[i] = a;
#pragma unroll
      for (int w = 1; w < NW; ++w) (&part[w][0][0])[i] = 0;
    }
    if (threadIdx.x == 0) __hip_atomic_store(&p.ws_cnt[bin], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
  }

  // epilogue: exact integer sum over the waves, then the fixed-order fp32 sum (same evaluation
  // order as the tiled kernel): one member, or members kept apart:
  //   y_m = s_x,m * (sum_k s_k * a_k) + b;  members summed: y = sum_m sum_k (s_k * s_x,m) * a_k + b.
  for (int o = o_first; o < n_out; o += O_STEP) {
    // a row block's items are adjacent, in ascending order k
    const int col = out_rb(o) * 16 + ch;
    const float bias = p.bias != nullptr ? p.bias[col] : 0.f;
    float yacc = 0.f;
#pragma unroll
    for (int m = 0; m < R; ++m) {
      if (m >= p.M) break;
      const int rs = rsm[m];
      const float sx = sxm[m];
      const int k_lo = pick(p.member_lo, m), k_hi = pick(p.member_hi, m);
#pragma unroll
      for (int r = 0; r < R; ++r) {
        if (its[r] != o || itk[r] < k_lo || itk[r] > k_hi) continue;
        int a = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) a += part[w][r][fidx];
        a -= OFF * rs;
        const float sc = fold_sx ? scv[r] * sx : scv[r];
        yacc = fmaf(sc, (float)a, yacc);
        if (ACC_OUT) {
          if (tg < p.T) p.acc_out[((size_t)itk[r] * p.T + tg) * p.out + col] = a;
        }
      }
      if (ACC_OUT) continue;
      if (fold_sx && m + 1 < p.M) continue;
      const float bm = (m == 0 || fold_sx) ? bias : (p.bias_mstride != 0 && p.bias != nullptr ? p.bias[(size_t)m * p.bias_mstride + col] : 0.f);
      float v = fold_sx ? yacc + bm : fmaf(sx, yacc, bm);   // same rounding as the tiled kernel
      yacc = 0.f;
      float rsum = 0.f;
      if (p.res != nullptr) {
        // the members summed into this output each add their own skip tensor
        const int n_res = p.reduce ? p.res_members : (m < p.res_members ? 1 : 0);
        const float* rp = p.res + (size_t)(p.reduce ? 0 : m) * p.res_mstride + (size_t)min(tg, p.T - 1) * p.out + col;
        for (int mm = 0; mm < n_res; ++mm) rsum += rp[(size_t)mm * p.res_mstride];
      }
      if (p.res_pre_act) v += rsum;
      if (p.act == PIPE_ACT_GELU) v = gelu_erf(v);
      else if (p.act == PIPE_ACT_RELU) v = fmaxf(v, 0.f);
      if (!p.res_pre_act) v += rsum;
      if (p.amax_out != nullptr) {
        const bool two_sided = p.amax_neg != nullptr;
        float mx = tg < p.T ? (two_sided ? fmaxf(v, 0.f) : fabsf(v)) : 0.f;
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) mx = fmaxf(mx, __shfl_xor(mx, s, 64));
        if (lane == 0) amax_raise(&p.amax_out[m], mx);
        if (two_sided) {
          float mn = tg < p.T ? fmaxf(-v, 0.f) : 0.f;
#pragma unroll
          for (int s = 32; s > 0; s >>= 1) mn = fmaxf(mn, __shfl_xor(mn, s, 64));
          if (lane == 0) amax_raise(&p.amax_neg[m], mn);
        }
      }
      if (tg < p.T) p.y[((size_t)(p.reduce ? 0 : m) * p.T + tg) * p.out + col] = v;
    }
  }
}

// Bins of CAP = 4 * NCH items (expansions with 5 to 16 orders).  The workgroup streams the bin in
// chunks of R = 4 items exactly as above (waves split k, two tiles per item in flight), reduces
// each chunk's per-wave tiles into isum and runs one epilogue over all items: per output row
// block and member the items are summed in ascending order k, the same fp32 order as everywhere.
// XM = 1: all items read one activation tensor; XM = 4: one stream per item of the chunk (its
// member's tensor; the streams need the bin descriptor, so it is fetched first).
template <int BITS, int NW, int XM, int NCH>
__global__ __launch_bounds__(NW * 64, 2) void gemm_stream_multi_kernel(const StreamParams p) {
  static_assert(XM == 1 || XM == R, "one stream, or one per item of a chunk");
  constexpr int CAP = R * NCH;
  constexpr int OFF = BITS == 8 ? 0 : (BITS == 4 ? 8 : 1);
  constexpr int KSUP = 512 / BITS;
  constexpr int STEPS = KSUP / 64;
  constexpr int NX = XM * STEPS;
  constexpr int BIN_WORDS = sizeof(StreamBin) / 4;
  static_assert(BIN_WORDS <= 64, "bin descriptor is fetched with one load per lane");
  __shared__ int part[NW][R][256];   // each wave's partial tiles of the current chunk
  __shared__ int isum[CAP][256];     // the bin's integer tiles, summed over the waves
  __shared__ int s_last;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n_tiles = (p.nks * 64) / KSUP;
  if (blockIdx.x == 0 && (int)threadIdx.x < p.zero_n && p.zero_after != nullptr) p.zero_after[threadIdx.x] = 0u;
  if (p.zero_big != nullptr)
    for (int i = blockIdx.x * (NW * 64) + threadIdx.x; i < p.zero_big_n; i += gridDim.x * (NW * 64)) p.zero_big[i] = 0u;

  const int subs = p.ksplit * p.n_tb;
  const int grp = (int)blockIdx.x / (8 * subs), within = (int)blockIdx.x - grp * (8 * subs);
  const int bin = grp * 8 + (within & 7), sub = within >> 3;
  const int ksp = sub % p.ksplit, tb = sub / p.ksplit;
  if (bin >= p.n_bins) return;

  const int e = threadIdx.x & 255;
  const int t = e >> 4, ch = e & 15;
  const int tg = tb * 16 + t;
  const int fidx = ((ch >> 2) * 16 + t) * 4 + (ch & 3);
  const int o_first = __builtin_amdgcn_readfirstlane(threadIdx.x >> 8);
  constexpr int O_STEP = (NW * 64) / 256;
  const bool fold_sx = p.reduce && p.M > 1;
  const int tile_lo = (int)((long long)n_tiles * ksp / p.ksplit), tile_hi = (int)((long long)n_tiles * (ksp + 1) / p.ksplit);

  const int d0 = lane < BIN_WORDS ? reinterpret_cast<const int32_t*>(p.bins + bin)[lane] : 0;
  auto word = [&](int i) __attribute__((always_inline)) { return __builtin_amdgcn_readlane(d0, i); };
  auto out_rb = [&](int o) __attribute__((always_inline)) { return word(2 + 2 * STREAM_BIN_CAP + o); };
  // epilogue operands, requested now and used (or staged in LDS) only after the code stream has
  // started: this thread's row scale of every item, and per member the activation scale and
  // the token's code sum
  float scv[CAP];
#pragma unroll
  for (int r = 0; r < CAP; ++r) scv[r] = p.scales[((size_t)bin * CAP + r) * 16 + ch];
  __shared__ float s_sx[PIPE_MAX_K];
  __shared__ int s_rs[PIPE_MAX_K][16];
  const float my_sx = (int)threadIdx.x < p.M ? p.s_x[threadIdx.x * p.sx_mstride] : 0.f;
  const int my_rs = (OFF && (int)threadIdx.x < p.M * 16)
                        ? p.rowsum[(size_t)(threadIdx.x >> 4) * p.rowsum_mstride + tb * 16 + (threadIdx.x & 15)] : 0;
  auto stage_member_operands = [&]() __attribute__((always_inline)) {
    if ((int)threadIdx.x < p.M) s_sx[threadIdx.x] = my_sx;
    if (OFF && (int)threadIdx.x < p.M * 16) s_rs[threadIdx.x >> 4][threadIdx.x & 15] = my_rs;
  };

  // One chunk of R items streamed by WPC waves (wave slot wk of WPC takes tiles wk, wk+WPC, ...);
  // leaves the wave's partial tiles in part[wave].
  auto run_chunk = [&](int c, int wk, int wpc) __attribute__((always_inline)) {
    v4i acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = v4i{0, 0, 0, 0};
    {
      // The codes are requested before anything that needs the bin descriptor (their positions
      // follow from the block index; unused positions of a bin hold zeros and are streamed too).
      const size_t pos0 = (size_t)bin * CAP + (size_t)c * R;
      const uint8_t* wb[R];
#pragma unroll
      for (int r = 0; r < R; ++r) wb[r] = p.codes + (pos0 + r) * (size_t)n_tiles * 1024;
      uint4 w0[R], w1[R], x0[NX], x1[NX];
      auto load_w = [&](int tl, uint4 (&w)[R]) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < R; ++r) w[r] = reinterpret_cast<const uint4*>(wb[r] + (size_t)tl * 1024)[lane];
      };
#pragma unroll
      for (int r = 0; r < R; ++r) { w0[r] = make_uint4(0, 0, 0, 0); w1[r] = make_uint4(0, 0, 0, 0); }
      int tl = tile_lo + wk;
      if (tl < tile_hi) load_w(tl, w0);
      if (tl + wpc < tile_hi) load_w(tl + wpc, w1);
      const int n_items = word(0);
      const uint8_t* xb[XM];
#pragma unroll
      for (int s = 0; s < XM; ++s) {
        // stream s feeds item s of the chunk: its member's tensor (items beyond the bin's last repeat it)
        const int it = min(c * R + s, n_items - 1);
        const int mem = XM == 1 ? 0 : pick(p.member_of, word(2 + it));
        xb[s] = p.qx + (size_t)mem * p.qx_mstride + (size_t)tb * p.nks * 1024;
      }
      auto load_x = [&](int tl, uint4 (&x)[NX]) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < XM; ++s)
#pragma unroll
          for (int j = 0; j < STEPS; ++j) x[s * STEPS + j] = reinterpret_cast<const uint4*>(xb[s] + (size_t)(tl * STEPS + j) * 1024)[lane];
      };
#pragma unroll
      for (int j = 0; j < NX; ++j) { x0[j] = make_uint4(0, 0, 0, 0); x1[j] = make_uint4(0, 0, 0, 0); }
      if (tl < tile_hi) load_x(tl, x0);
      if (tl + wpc < tile_hi) load_x(tl + wpc, x1);
      auto mul_tile = [&](uint4 (&w)[R], uint4 (&x)[NX]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < STEPS; ++j) {
#pragma unroll
          for (int r = 0; r < R; ++r) {
            const uint4& xs = x[(XM == 1 ? 0 : r) * STEPS + j];
            const v4i xf = v4i{(int)xs.x, (int)xs.y, (int)xs.z, (int)xs.w};
            v4i wf;
            unpack_step<BITS>(w[r], j, wf);
            acc[r] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf, xf, acc[r], 0, 0, 0);
          }
        }
      };
      for (; tl < tile_hi; tl += 2 * wpc) {
        mul_tile(w0, x0);
        if (tl + 2 * wpc < tile_hi) { load_w(tl + 2 * wpc, w0); load_x(tl + 2 * wpc, x0); }
        if (tl + wpc < tile_hi) {
          mul_tile(w1, x1);
          if (tl + 3 * wpc < tile_hi) { load_w(tl + 3 * wpc, w1); load_x(tl + 3 * wpc, x1); }
        }
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r)
      *reinterpret_cast<v4i*>(&part[wave][r][lane * 4]) = acc[r];
  };
  if constexpr (NW % NCH == 0) {
    // the waves share out the chunks: NW / NCH waves per chunk, all chunks in flight at once
    constexpr int WPC = NW / NCH;
    run_chunk(wave / WPC, wave % WPC, WPC);
    stage_member_operands();
    __syncthreads();
    for (int i = threadIdx.x; i < CAP * 256; i += NW * 64) {
      const int c = i / (R * 256), j = i - c * (R * 256);
      int a = 0;
#pragma unroll
      for (int w = 0; w < WPC; ++w) a += (&part[c * WPC + w][0][0])[j];
      (&isum[0][0])[i] = a;
    }
    __syncthreads();
  } else {
    for (int c = 0; c < NCH; ++c) {
      if (c > 0 && c * R >= word(0)) continue;   // uniform; chunk 0 always holds items
      run_chunk(c, wave, NW);
      if (c == 0) stage_member_operands();
      __syncthreads();
      for (int i = threadIdx.x; i < R * 256; i += NW * 64) {
        int a = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) a += (&part[w][0][0])[i];
        (&isum[c * R][0])[i] = a;
      }
      __syncthreads();   // part is free for the next chunk, isum of this one complete
    }
  }

  const int n_items = word(0), n_out = word(1);
  // a split bin: as in the 4-item kernel, over the tiles of the bin's n_items items
  if (p.ksplit > 1) {
    const int n_words = n_items * 256;
    int32_t* ws = p.ws_sum + ((size_t)bin * p.ksplit + ksp) * (CAP * 256);
    for (int i = threadIdx.x; i < n_words; i += NW * 64)
      __hip_atomic_store(&ws[i], (&isum[0][0])[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    if (threadIdx.x == 0) s_last = atomicAdd(&p.ws_cnt[bin], 1u) == (unsigned)(p.ksplit - 1);
    __syncthreads();
    if (!s_last) return;
    const int32_t* wsb = p.ws_sum + (size_t)bin * p.ksplit * (CAP * 256);
    for (int i = threadIdx.x; i < n_words; i += NW * 64) {
      int a = 0;
      for (int q = 0; q < p.ksplit; ++q) a += __hip_atomic_load(&wsb[(size_t)q * (CAP * 256) + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      (&isum[0][0])[i] = a;
    }
    if (threadIdx.x == 0) __hip_atomic_store(&p.ws_cnt[bin], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
  }

  // epilogue over all items of the bin (same arithmetic and order as the 4-item kernel)
  for (int o = o_first; o < n_out; o += O_STEP) {
    const int col = out_rb(o) * 16 + ch;
    const float bias = p.bias != nullptr ? p.bias[col] : 0.f;
    float yacc = 0.f;
    for (int m = 0; m < p.M; ++m) {
      const float sx = s_sx[m];
      const int rs = OFF ? s_rs[m][t] : 0;
      const int k_lo = pick(p.member_lo, m), k_hi = pick(p.member_hi, m);
#pragma unroll
      for (int r = 0; r < CAP; ++r) {
        const int kk = word(2 + r);
        if (r >= n_items || word(2 + STREAM_BIN_CAP + r) != o || kk < k_lo || kk > k_hi) continue;   // uniform
        const int a = isum[r][fidx] - OFF * rs;
        const float sc = fold_sx ? scv[r] * sx : scv[r];
        yacc = fmaf(sc, (float)a, yacc);
      }
      if (fold_sx && m + 1 < p.M) continue;
      const float bm = (m == 0 || fold_sx) ? bias : (p.bias_mstride != 0 && p.bias != nullptr ? p.bias[(size_t)m * p.bias_mstride + col] : 0.f);
      float v = fold_sx ? yacc + bm : fmaf(sx, yacc, bm);
      yacc = 0.f;
      float rsum = 0.f;
      if (p.res != nullptr) {
        const int n_res = p.reduce ? p.res_members : (m < p.res_members ? 1 : 0);
        const float* rp = p.res + (size_t)(p.reduce ? 0 : m) * p.res_mstride + (size_t)min(tg, p.T - 1) * p.out + col;
        for (int mm = 0; mm < n_res; ++mm) rsum += rp[(size_t)mm * p.res_mstride];
      }
      if (p.res_pre_act) v += rsum;
      if (p.act == PIPE_ACT_GELU) v = gelu_erf(v);
      else if (p.act == PIPE_ACT_RELU) v = fmaxf(v, 0.f);
      if (!p.res_pre_act) v += rsum;
      if (p.amax_out != nullptr) {
        const bool two_sided = p.amax_neg != nullptr;
        float mx = tg < p.T ? (two_sided ? fmaxf(v, 0.f) : fabsf(v)) : 0.f;
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) mx = fmaxf(mx, __shfl_xor(mx, s, 64));
        if (lane == 0) amax_raise(&p.amax_out[m], mx);
        if (two_sided) {
          float mn = tg < p.T ? fmaxf(-v, 0.f) : 0.f;
#pragma unroll
          for (int s = 32; s > 0; s >>= 1) mn = fmaxf(mn, __shfl_xor(mn, s, 64));
          if (lane == 0) amax_raise(&p.amax_neg[m], mn);
        }
      }
      if (tg < p.T) p.y[((size_t)(p.reduce ? 0 : m) * p.T + tg) * p.out + col] = v;
    }
  }
}

template <int BITS, int NW, int NCH>
int launch_multi(const StreamParams& p, int n_bins, int xm, const GemmArgs& a, hipStream_t st) {
  const dim3 grid((unsigned)((n_bins + 7) / 8 * 8 * p.ksplit * p.n_tb)), blk(NW * 64);
  if (xm == 1) PIPE_LAUNCH((gemm_stream_multi_kernel<BITS, NW, 1, NCH>), grid, blk, st, a.ev_start, a.ev_stop, p);
  else PIPE_LAUNCH((gemm_stream_multi_kernel<BITS, NW, R, NCH>), grid, blk, st, a.ev_start, a.ev_stop, p);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

template <int BITS>
int launch_multi_cap(const StreamParams& p, int n_bins, int cap, int xm, const GemmArgs& a, hipStream_t st) {
  switch (cap) {
    case 8: return launch_multi<BITS, 8, 2>(p, n_bins, xm, a, st);
    case 12: return launch_multi<BITS, 8, 3>(p, n_bins, xm, a, st);
    case 16: return launch_multi<BITS, 8, 4>(p, n_bins, xm, a, st);
    default: return PIPE_ESHAPE;
  }
}

template <int BITS, int NW>
int launch_nw(const StreamParams& p, int n_bins, int xm, bool acc_out, const GemmArgs& a, hipStream_t st) {
  const dim3 grid((unsigned)((n_bins + 7) / 8 * 8 * p.ksplit * p.n_tb)), blk(NW * 64);
  if (p.x_f32 != nullptr) {
    // no quantizer launch: the contraction quantizes its few tokens itself
    if (xm != 1 || acc_out || p.T > QF_T || p.nks * 64 > QF_IN || p.in % 4 != 0 || p.n_tb != 1) return PIPE_EINVAL;
    PIPE_LAUNCH((gemm_stream_kernel<BITS, NW, 1, false, true, true>), grid, blk, st, a.ev_start, a.ev_stop, p);
    PIPE_HIP(hipGetLastError());
    return PIPE_OK;
  }
  const bool xmask = p.T % 16 != 0;
#define PIPE_STREAM_LAUNCH(XMV, ACC, MASK) PIPE_LAUNCH((gemm_stream_kernel<BITS, NW, XMV, ACC, MASK>), grid, blk, st, a.ev_start, a.ev_stop, p)
#define PIPE_STREAM_PICK(XMV)                                                     \
  do {                                                                            \
    if (acc_out) { if (xmask) PIPE_STREAM_LAUNCH(XMV, true, true); else PIPE_STREAM_LAUNCH(XMV, true, false); }   \
    else { if (xmask) PIPE_STREAM_LAUNCH(XMV, false, true); else PIPE_STREAM_LAUNCH(XMV, false, false); }         \
  } while (0)
  if (xm == 1) PIPE_STREAM_PICK(1);
  else if (xm == 2) PIPE_STREAM_PICK(2);
  else PIPE_STREAM_PICK(4);
#undef PIPE_STREAM_PICK
#undef PIPE_STREAM_LAUNCH
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

}  // namespace

int launch_gemm_stream(const GemmArgs& a, hipStream_t st) {
  const pipe_expansion* e = a.e;
  if (a.T <= 0) return PIPE_OK;
  if (a.T > PIPE_STREAM_MAX_T || a.T_pad != (int)round_up64(a.T, 16) || e->K > e->bin_cap || e->bin_cap % R != 0) return PIPE_ESHAPE;
  if (e->bin_cap != R && a.acc_out != nullptr) return PIPE_EINVAL;   // the integer export of wide bins goes through the tiled kernel
  StreamParams p;
  p.qx = a.qx; p.qx_mstride = a.qx_mstride;
  p.rowsum = a.rowsum; p.rowsum_mstride = a.rowsum_mstride;
  p.s_x = a.s_x; p.sx_mstride = a.sx_mstride;
  p.codes = e->codes_dev; p.scales = e->scales_all_dev;
  p.bins = e->bins_dev;
  p.bias = a.bias; p.bias_mstride = a.bias_mstride; p.y = a.y; p.acc_out = a.acc_out; p.amax_out = a.amax_out; p.amax_neg = a.amax_neg; p.res = a.res; p.res_mstride = a.res_mstride; p.res_members = a.res_members; p.res_pre_act = a.res_pre_act; p.zero_after = a.zero_after; p.zero_n = a.zero_n; p.zero_big = a.zero_big; p.zero_big_n = a.zero_big_n;
  p.T = a.T; p.out = e->out; p.K = e->K; p.nks = e->nks; p.M = a.M; p.reduce = a.reduce; p.act = a.act;
  p.x_f32 = a.x_f32; p.s_static = a.s_static; p.act_qmax = g_act_qmax_host; p.in = e->in;
  if (a.x_f32 != nullptr && e->bin_cap != R) return PIPE_EINVAL;
  // Fewer bins than half the CUs and a long k: split each bin over several workgroups (each still
  // with at least two tiles per wave).  With more bins a split only adds the exchange through
  // the workspace (measured on the 4096 x 11008 4-bit layer: 160 bins, 21.7 us unsplit, 23.5 us
  // split in three).
  {
    const int n_tiles = e->in_pad / (512 / e->bits);
    int ks;
    if (g_stream_ksplit > 0) ks = std::min(std::min(g_stream_ksplit, PIPE_MAX_SPLIT), n_tiles);   // forced (tests, tuning)
    else ks = std::min(256 / (e->n_bins > 0 ? e->n_bins : 1), std::min(PIPE_MAX_SPLIT, n_tiles / 16));
    p.n_tb = a.T_pad / 16;
    p.n_bins = e->n_bins;
    p.thr0 = e->bin_thr[0]; p.thr1 = e->bin_thr[1]; p.thr2 = e->bin_thr[2]; p.zero_pos = e->zero_pos;
    if (p.n_tb > 1) ks = 1;   // several token blocks already multiply the workgroups
    p.ksplit = std::max(ks, 1);
    p.ws_sum = e->split_sum_dev; p.ws_cnt = e->split_cnt_dev;
  }
  for (int m = 0; m < PIPE_MAX_K; ++m) { p.member_lo[m] = a.member_lo[m]; p.member_hi[m] = a.member_hi[m]; p.member_of[m] = 0; }
  for (int m = 0; m < a.M; ++m)
    for (int k = a.member_lo[m]; k <= a.member_hi[m]; ++k) p.member_of[k] = m;
  // distinct activation tensors: one, or one per member
  const int xm = (a.qx_mstride == 0 || a.M <= 1) ? 1 : (a.M <= 2 ? 2 : 4);
  const bool acc_out = a.acc_out != nullptr;
  if (e->bin_cap != R) {
    const int xmm = (a.qx_mstride == 0 || a.M <= 1) ? 1 : R;
    switch (e->bits) {
      case 8: return launch_multi_cap<8>(p, e->n_bins, e->bin_cap, xmm, a, st);
      case 4: return launch_multi_cap<4>(p, e->n_bins, e->bin_cap, xmm, a, st);
      default: return launch_multi_cap<2>(p, e->n_bins, e->bin_cap, xmm, a, st);
    }
  }
  switch (e->bits) {
    case 8: return launch_nw<8, 8>(p, e->n_bins, xm, acc_out, a, st);
    case 4: return launch_nw<4, 8>(p, e->n_bins, xm, acc_out, a, st);
    default: return launch_nw<2, 8>(p, e->n_bins, xm, acc_out, a, st);
  }
}
