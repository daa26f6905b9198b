// Resident kernel for decode-sized batches (T <= 16): ONE launch walks a whole chain of expanded
// layers (App. B "Ensemble of more Layers", Sec. 3.2: a member is the whole network; App. B,
// Eq. (define_dre) per layer), so the packed codes of layer l+1 stream from HBM while layer l's
// results are still being exchanged, and no launch boundary separates the layers.
//
// One workgroup per compute unit, 12 waves:
//   waves 0-7  ("workers") stream packed codes and multiply.  A wave owns the 1-KiB code tiles
//              w, w+8, ... of every item (stored row block) of its workgroup's units and keeps RD
//              rounds of 4 tiles in flight in registers, across unit and LAYER boundaries: the
//              codes do not depend on the activations, so the first rounds of the next layer are
//              requested before the grid-wide exchange that makes its input codes available.
//              Exact int32 partial tiles are added up in LDS; token code sums (for the offset-binary
//              codes) come from one more MFMA per 64-k step against a row of ones.
//   waves 8-11 ("epilogue") turn the integer tiles into fp32 outputs with the arithmetic and order of
//              the per-layer kernels (bit-identical results), and run the exchange between layers:
//              every workgroup quantizes the outputs it produced itself (network input: a slice of x).
// Exchange between layers, two grid-wide steps, no read-modify-write atomics and no cache-wide
// fences (a release or acquire fence at device scope costs 10-30 us on this chip, measured):
//   A  max|.|: each workgroup publishes {epoch, max} as one 64-bit device-scope store per tensor and
//      reads everybody's, so all derive the same scale max/q_max (skipped for a given static scale);
//   B  codes:  each workgroup writes its own outputs' codes with device-scope (write-through) stores,
//      waits for their completion, publishes its epoch in its flag word and polls the others' flags.
//   Everything one workgroup writes for another goes through device-scope stores; the consumers'
//   bulk reads of the codes are ordinary loads from a buffer that no cache can hold stale (each
//   layer has its own, first read in this launch after the flags were seen).
// Every wait is bounded: after `spin_limit` polls a workgroup records the failure in a status word,
// stops waiting for the rest of the launch and runs to its end, so the grid always drains.
#include "pipe_internal.h"

#include <algorithm>
#include <cstring>

int g_decode_resident = 1;
int g_resident_spin_limit = 1 << 19;
unsigned long long* g_resident_trace = nullptr;

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int RES_WORKERS = 8;
constexpr int RES_EPI = 4;
constexpr int RES_THREADS = (RES_WORKERS + RES_EPI) * 64;
constexpr int RES_STASH = 48;            // 1-KiB slots of fp32 outputs a workgroup keeps in LDS between a layer and the next exchange
constexpr int RES_PAD_LDS = 88 * 1024;   // dynamic LDS: the stash, the rest untouched (it keeps a compute unit to one workgroup)

struct ResLayer {
  const uint8_t* codes;     // stored row blocks of the layer, schedule order
  const float* scales;      // 16 row scales per position
  const int32_t* subs;      // [n_units * nsub] ResSub
  const int32_t* epi;       // [n_units] ResUnitEpi
  const float* bias;        // or nullptr
  float* out;               // hidden layer: [M, T, out_w]; last layer: [T, out_w] (members summed)
  const float* res;         // skip tensor or nullptr
  long long res_mstride;
  uint8_t* qin;             // codes entering the layer: [xm][nks][1 KiB] (fragment layout, one 16-token block)
  int n_units, nsub, n_tiles, nks;
  int out_w;                // width of a row of `out` (gated layer: hidden width)
  int in, in_pad;
  int xm;                   // distinct activation tensors entering the layer: 1 (first layer) or M
  int act, res_members, res_pre_act, gated, reduce, res_device;
  float s_in[2];            // > 0: given scales of the tensors entering the layer (no exchange of maxima then)
};

struct ResParams {
  ResLayer layer[PIPE_RES_MAX_LAYERS];
  int L, T, M, G;
  int member_lo[PIPE_RES_MAX_M], member_hi[PIPE_RES_MAX_M];
  int member_of[4];
  const float* x;           // network input [T, in0]
  float s_static;           // > 0: given scale of the network input
  float act_qmax;
  uint32_t* flags;          // [G] epoch each workgroup reached
  unsigned long long* amax_tag;   // [G][2] {epoch, bit pattern of the local max}
  uint32_t* gen;            // epoch the previous launch on this scratch ended with
  uint32_t* status;         // != 0: a wait ran into the spin limit
  int spin_limit;
  unsigned long long* trace;   // profiling: [G][L][8] timestamps (100 MHz) of the phases of every layer, or nullptr
};

static_assert(sizeof(ResParams) <= 3584, "kernel arguments are limited to 4 KiB");

__device__ __forceinline__ float gelu_erf_r(float a) {
  return 0.5f * a * (1.f + erff(a * 0.70710678118654752440f));
}

template <int BITS>
__device__ __forceinline__ void unpack_step_r(const uint4& w, int j, v4i& o) {
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

// wave-uniform loads of the schedule tables (written once by the host): scalar loads
template <class T>
__device__ __forceinline__ T cload_r(const void* base, size_t idx) {
  typedef const __attribute__((address_space(4))) T* cptr;
  return ((cptr)(unsigned long long)base)[idx];
}

__device__ __forceinline__ void st_dev_u32(uint32_t* p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t ld_dev_u32(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// XM: activation tensors a unit's items can read (1, or one per member: 2).  RD: rounds of four code
// tiles a worker wave keeps in flight.
template <int BITS, int XM, int RD>
__global__ __launch_bounds__(RES_THREADS, 1) void chain_resident_kernel(const ResParams p) {
  static_assert(RD % 2 == 0, "the activation fragments alternate between two register sets");
  constexpr int OFF = BITS == 8 ? 0 : (BITS == 4 ? 8 : 1);
  constexpr int KSUP = 512 / BITS;
  constexpr int STEPS = KSUP / 64;
  __shared__ int tile[2][PIPE_RES_MAX_ITEMS + 2][256];
  __shared__ float s_wmax[RES_EPI][2];
  __shared__ float s_scale[2];   // scales of the codes entering the current layer
  __shared__ int s_fail;
  __shared__ unsigned long long s_ts[PIPE_RES_MAX_LAYERS][8];
  __shared__ uint32_t s_seen;   // the last epoch one of the polling waves has seen every workgroup reach
  // this workgroup's unit descriptors of all layers, copied once (a cold scalar load per unit on the
  // workers' path costs more than the unit's arithmetic): per layer, per local unit, its sub-units
  // (16 ints each) and then its epilogue descriptor (32 ints)
  __shared__ int s_desc[PIPE_RES_DESC_INTS];
  extern __shared__ int pad_lds[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wg = blockIdx.x, G = p.G;
  for (int i = threadIdx.x; i < 2 * (PIPE_RES_MAX_ITEMS + 2) * 256; i += RES_THREADS) (&tile[0][0][0])[i] = 0;
  if (threadIdx.x == 0) { s_fail = 0; s_scale[0] = 0.f; s_scale[1] = 0.f; }
  if (threadIdx.x < PIPE_RES_MAX_LAYERS * 8) (&s_ts[0][0])[threadIdx.x] = 0ull;
  auto units_of = [&](int n_units) { return n_units > wg ? (n_units - wg + G - 1) / G : 0; };
  auto dstride_of = [&](int l) { return p.layer[l].nsub * 16 + 32; };
  {
    int off = 0;
    for (int l = 0; l < p.L; ++l) {
      const ResLayer& ly = p.layer[l];
      const int stride = ly.nsub * 16 + 32, cnt = units_of(ly.n_units) * stride;
      for (int i = threadIdx.x; i < cnt; i += RES_THREADS) {
        const int u = i / stride, w = i - u * stride;
        const size_t unit = (size_t)(wg + u * G);
        s_desc[off + i] = w < ly.nsub * 16 ? ly.subs[unit * ly.nsub * 16 + w] : ly.epi[unit * 32 + (w - ly.nsub * 16)];
      }
      off += cnt;   // the host has checked that all layers fit
    }
  }
  __syncthreads();
  auto dword = [&](int i) __attribute__((always_inline)) { return __builtin_amdgcn_readfirstlane(s_desc[i]); };
  // profiling: slot 0 exchange begins, 1 maxima known, 2 codes stored, 3 all flags seen, 4 last unit's epilogue done
  // (first epilogue wave); 7 worker wave 0 has multiplied its last round and passed the unit's barrier
  // (kept in LDS and written out when the kernel ends: a store in the middle would be waited for by the next load)
  auto stamp = [&](int l, int slot) __attribute__((always_inline)) {
    if (p.trace != nullptr && lane == 0) s_ts[l][slot] = wall_clock64();
  };

  if (wave < RES_WORKERS) {
    // ============================================================== workers
    // The loads of a step are unconditional and their number fixed (a step without real work loads
    // a valid address and drops the result), so the waits for them are exact counts: RD - 1 rounds of
    // codes (across layer boundaries) and a round of fragments stay in flight while a round is multiplied.
    constexpr int NXL = XM * STEPS;        // fragment loads of a round
    const bool xlive = (lane & 15) < p.T;
    // lanes of tokens beyond the batch re-read token 0's bytes of their k chunk (no further cache lines) and are zeroed
    const int xl = xlive ? lane : (lane & 48);
    v4i acc[4], acc1[XM];
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[r] = v4i{0, 0, 0, 0};
#pragma unroll
    for (int m = 0; m < XM; ++m) acc1[m] = v4i{0, 0, 0, 0};
    // a ring of RD rounds of codes (round q of a layer lives in slot q % RD; every layer's rounds are
    // padded to a multiple of RD, so the mapping is static) and two rounds of activation fragments
    uint4 wreg[RD][4], xreg[2][NXL];
#pragma unroll
    for (int s = 0; s < RD; ++s)
#pragma unroll
      for (int r = 0; r < 4; ++r) wreg[s][r] = make_uint4(0, 0, 0, 0);

    // rounds of this wave in layer l: units x sub-units x tiles; a wave beyond the layer's tiles
    // still walks one empty round per sub-unit (it takes part in the unit's barrier)
    auto ru_of = [&](int l) { const int nt = p.layer[l].n_tiles; return nt > wave ? (nt - wave + RES_WORKERS - 1) / RES_WORKERS : 0; };
    auto rounds_of = [&](int l) { return units_of(p.layer[l].n_units) * p.layer[l].nsub * max(ru_of(l), 1); };

    // ---- issue cursor: the next round whose codes have not been requested (runs ahead, across layers)
    int il = 0, iq = 0, iu = 0, ig = 0, ij = 0;       // layer, round in layer, local unit, sub-unit, tile step
    int ioff = 0;                                     // where layer il's descriptors begin in s_desc
    int ipos[4] = {0, 0, 0, 0};
    // the cursor's layer, read from the kernel arguments once per layer (a scalar load per use sits on the issue path)
    const uint8_t* i_codes = p.layer[0].codes;
    int i_ntiles = 1, i_ru = 0, i_nsub = 1, i_nu = 0, i_stride = 48;
    auto issue_desc = [&]() __attribute__((always_inline)) {
      const int at = ioff + iu * i_stride + ig * 16;
#pragma unroll
      for (int r = 0; r < 4; ++r) ipos[r] = dword(at + r);
    };
    auto issue_seek = [&]() __attribute__((always_inline)) {   // skip layers without rounds, fetch the descriptor
      while (il < p.L && rounds_of(il) == 0) { ioff += units_of(p.layer[il].n_units) * dstride_of(il); ++il; }
      const int li = il < p.L ? il : p.L - 1;
      i_codes = p.layer[li].codes; i_ntiles = p.layer[li].n_tiles; i_ru = ru_of(li); i_nsub = p.layer[li].nsub;
      i_nu = units_of(p.layer[li].n_units); i_stride = dstride_of(li);
      if (il < p.L) issue_desc();
    };
    issue_seek();
    // Four code loads: the cursor's round if `real`, else a valid address whose data nobody uses.
    auto issue_codes = [&](uint4 (&w)[4], bool real) __attribute__((always_inline)) {
      const bool has = real && i_ru > 0;
      const int tl = has ? wave + RES_WORKERS * ij : 0;
      // items a sub-unit does not have repeat its first one (a cache hit; the product is dropped)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        w[r] = reinterpret_cast<const uint4*>(i_codes + ((size_t)(has ? ipos[r] : 0) * i_ntiles + tl) * 1024)[lane];
      if (real) {
        ++iq;
        if (++ij >= max(i_ru, 1)) {
          ij = 0;
          if (++ig >= i_nsub) { ig = 0; ++iu; }
          if (iu >= i_nu) { ioff += i_nu * i_stride; ++il; iq = 0; iu = 0; issue_seek(); }
          else issue_desc();
        }
      }
    };

    int buf = 0;
    const int mof0 = p.member_of[0], mof1 = p.member_of[1], mof2 = p.member_of[2], mof3 = p.member_of[3];
    int coff = 0;   // where layer l's descriptors begin in s_desc
    for (int l = 0; l < p.L; coff += units_of(p.layer[l].n_units) * dstride_of(l), ++l) {
      const ResLayer& ly = p.layer[l];
      const int ru = ru_of(l), ru_eff = max(ru, 1);
      const int rounds = rounds_of(l);
      const int rounds_pad = (rounds + RD - 1) / RD * RD;
      // codes of the first rounds, unless the previous layer's last steps requested them already
      if (il == l && iq == 0) {
#pragma unroll
        for (int s = 0; s < RD; ++s)
          if (il == l && iq == s) issue_codes(wreg[s], true);
      }
      // the codes entering this layer are being produced: four workgroup barriers of the exchange
      __syncthreads();
      __syncthreads();
      __syncthreads();
      __syncthreads();
      int xj = 0;   // tile step of the next round whose fragments have not been requested
      const uint8_t* l_qin = ly.qin;
      const int l_nks = ly.nks, l_xm = ly.xm, l_nsub = ly.nsub, l_stride = dstride_of(l);
      auto issue_x = [&](uint4 (&x)[NXL], bool real) __attribute__((always_inline)) {
        const bool has = real && ru > 0;
        const int tl = has ? wave + RES_WORKERS * xj : 0;
#pragma unroll
        for (int m = 0; m < XM; ++m)
#pragma unroll
          for (int j = 0; j < STEPS; ++j)
            x[m * STEPS + j] = reinterpret_cast<const uint4*>(l_qin + ((size_t)(m < l_xm ? m : 0) * l_nks + (size_t)tl * STEPS + j) * 1024)[xl];
        if (real && ++xj >= ru_eff) xj = 0;
      };
      if (rounds_pad > 0) {
        issue_x(xreg[0], 0 < rounds);
        issue_x(xreg[1], 1 < rounds);
      }
      // ---- consume cursor
      int cu = 0, cg = 0, cj = 0, cn = 0, cslot0 = 0, clast = 0, citm[4] = {0, 0, 0, 0};
      auto cons_desc = [&]() __attribute__((always_inline)) {
        const int at = coff + cu * l_stride + cg * 16;
        cn = dword(at + 8); cslot0 = dword(at + 9); clast = dword(at + 10);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int k = (XM == 1) ? 0 : dword(at + 4 + r);
          citm[r] = (XM == 1 || l_xm == 1) ? 0 : (k == 0 ? mof0 : (k == 1 ? mof1 : (k == 2 ? mof2 : mof3)));
        }
      };
      if (rounds > 0) cons_desc();

      for (int q0 = 0; q0 < rounds_pad; q0 += RD) {
#pragma unroll
        for (int s = 0; s < RD; ++s) {
          const int q = q0 + s;
          // 1. multiply round q
          if (q < rounds) {
            if (ru > 0) {
              uint4 (&w)[4] = wreg[s];
#pragma unroll
              for (int j = 0; j < STEPS; ++j) {
                // the fragments of this 64-k step, lanes of tokens beyond the batch zeroed (at use, not at
                // load: nothing waits for a load before the step that needs it)
                v4i x[XM];
#pragma unroll
                for (int m = 0; m < XM; ++m) {
                  const uint4& xr = xreg[s & 1][m * STEPS + j];
                  x[m] = v4i{xlive ? (int)xr.x : 0, xlive ? (int)xr.y : 0, xlive ? (int)xr.z : 0, xlive ? (int)xr.w : 0};
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                  v4i xf = x[0];
                  if (XM == 2) {
                    const bool pick1 = citm[r] == 1;
                    xf[0] = pick1 ? x[1][0] : xf[0];
                    xf[1] = pick1 ? x[1][1] : xf[1];
                    xf[2] = pick1 ? x[1][2] : xf[2];
                    xf[3] = pick1 ? x[1][3] : xf[3];
                  }
                  v4i wf;
                  unpack_step_r<BITS>(w[r], j, wf);
                  acc[r] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf, xf, acc[r], 0, 0, 0);
                }
                if (OFF != 0 && cg == 0) {
                  // token code sums: a row block of ones against the same fragments
                  const v4i ones = v4i{0x01010101, 0x01010101, 0x01010101, 0x01010101};
#pragma unroll
                  for (int m = 0; m < XM; ++m) acc1[m] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ones, x[m], acc1[m], 0, 0, 0);
                }
              }
            }
          }
          // 2. fragments of round q + 2 into the set just read; codes of round q + RD into the slot just read
          //    (once this layer's are all requested: round s of the next layer).  Always NXL + 4 loads.
          issue_x(xreg[s & 1], q + 2 < rounds);
          issue_codes(wreg[s], il < p.L && (il == l ? iq == q + RD : iq == s));
          // 3. end of a sub-unit: this wave's share of its integer tiles joins the others' in LDS
          if (q < rounds) {
            if (cj + 1 >= ru_eff) {
              if (ru > 0) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                  if (r < cn) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) atomicAdd(&tile[buf][cslot0 + r][lane * 4 + c], acc[r][c]);
                  }
                  acc[r] = v4i{0, 0, 0, 0};
                }
              }
              if (clast) {
                if (OFF != 0 && ru > 0) {
#pragma unroll
                  for (int m = 0; m < XM; ++m) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) atomicAdd(&tile[buf][PIPE_RES_MAX_ITEMS + m][lane * 4 + c], acc1[m][c]);
                    acc1[m] = v4i{0, 0, 0, 0};
                  }
                }
                __syncthreads();   // the unit's tiles are complete: the epilogue waves take them
                buf ^= 1;
              }
              cj = 0;
              if (++cg >= l_nsub) { cg = 0; ++cu; }
              if (q + 1 < rounds) cons_desc();
              else if (wave == 0) stamp(l, 7);
            } else {
              ++cj;
            }
          }
        }
      }
    }
  } else {
    // ============================================================== epilogue waves
    const int e = threadIdx.x - RES_WORKERS * 64;   // 0..255
    const int ewave = e >> 6;
    const int t = e >> 4, ch = e & 15;
    const int fidx = ((ch >> 2) * 16 + t) * 4 + (ch & 3);
    const bool tok = t < p.T;
    // Every epilogue wave tracks the epoch; the first one polls and tells the others through LDS and
    // the workgroup barrier that follows.
    uint32_t epoch = ld_dev_u32(p.gen);
    const uint32_t epoch0 = epoch;
    if (e == 0) s_seen = epoch;
    int buf = 0;
    const float qmax = p.act_qmax;
    // what this thread produced in the current layer: its max|.| per member, and the values themselves
    // (LDS, as far as it reaches; the rest is read back from the layer's output)
    float* stash = reinterpret_cast<float*>(pad_lds);
    float mx_out[2] = {0.f, 0.f};
    auto seen = [&]() __attribute__((always_inline)) {
      return (int)(__hip_atomic_load(&s_seen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) - epoch) >= 0 || s_fail != 0;
    };

    // one grid-wide step: publish this workgroup's epoch, wait until every workgroup has reached it
    auto grid_wait = [&]() __attribute__((always_inline)) {
      if (ewave != 0) return;   // one polling wave per workgroup: more of them only crowd the flags' memory channel (measured)
      if (e == 0) st_dev_u32(&p.flags[wg], epoch);
      bool ok = seen();
      for (int it = 0; it < p.spin_limit && !ok; ++it) {
        bool mine = true;
        for (int i = lane; i < G; i += 64) mine &= (int)(ld_dev_u32(&p.flags[i]) - epoch) >= 0;
        ok = __all(mine);
        if (ok && lane == 0) __hip_atomic_store(&s_seen, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        ok = ok || seen();
      }
      if (!ok && lane == 0) { s_fail = 1; st_dev_u32(p.status, 1u); }
    };

    int eoff = 0, eoff_prev = 0;   // where the descriptors of layer l and of layer l-1 begin in s_desc
    for (int l = 0; l < p.L; eoff_prev = eoff, eoff += units_of(p.layer[l].n_units) * dstride_of(l), ++l) {
      const ResLayer& ly = p.layer[l];
      const int n_in = ly.xm;   // tensors to quantize for this layer
      const ResLayer& lp = p.layer[l > 0 ? l - 1 : 0];
      const int nu_prev = l > 0 ? units_of(lp.n_units) : 0;
      const float st0 = l == 0 ? p.s_static : ly.s_in[0], st1 = l == 0 ? p.s_static : ly.s_in[1];
      const bool dynamic = !(st0 > 0.f);
      // ---------------- exchange, step A: max|.| of the tensor(s) entering layer l
      if (wave == RES_WORKERS) stamp(l, 0);
      float mx[2] = {0.f, 0.f};
      if (dynamic) {
        if (l == 0) {
          const int n4 = (p.T * ly.in) >> 2;
          const float4* x4 = reinterpret_cast<const float4*>(p.x);
          for (int i = wg * 256 + e; i < n4; i += G * 256) {
            const float4 v = x4[i];
            mx[0] = fmaxf(mx[0], fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
          }
        } else {
          // the outputs this workgroup produced in layer l-1
          mx[0] = mx_out[0]; mx[1] = mx_out[1];
        }
#pragma unroll
        for (int m = 0; m < 2; ++m) {
#pragma unroll
          for (int o = 32; o > 0; o >>= 1) mx[m] = fmaxf(mx[m], __shfl_xor(mx[m], o, 64));
          if (lane == 0) s_wmax[ewave][m] = mx[m];
        }
      }
      __syncthreads();   // P1
      if (dynamic) {
        ++epoch;
        if (ewave == 0) {
          if (lane < n_in) {
            float v = s_wmax[0][lane];
#pragma unroll
            for (int w = 1; w < RES_EPI; ++w) v = fmaxf(v, s_wmax[w][lane]);
            __hip_atomic_store(&p.amax_tag[wg * 2 + lane], ((unsigned long long)epoch << 32) | __float_as_uint(v), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
          }
          if (lane == 0) st_dev_u32(&p.flags[wg], epoch);   // keeps the flag word in step with the epoch
        }
        bool ok = ewave != 0 || seen();   // one polling wave per workgroup
        for (int it = 0; it < p.spin_limit && !ok; ++it) {
          bool mine = true;
          float g0 = 0.f, g1 = 0.f;
          for (int i = lane; i < G * n_in; i += 64) {
            const int w = i / n_in, m = i - w * n_in;
            const unsigned long long tv = __hip_atomic_load(&p.amax_tag[w * 2 + m], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            mine &= (uint32_t)(tv >> 32) == epoch;
            const float v = __uint_as_float((uint32_t)tv);
            if (m == 0) g0 = fmaxf(g0, v); else g1 = fmaxf(g1, v);
          }
          ok = __all(mine);
          if (ok) {
            // every workgroup's maximum of this epoch: the scales (any wave that gets here writes the same values)
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) { g0 = fmaxf(g0, __shfl_xor(g0, o, 64)); g1 = fmaxf(g1, __shfl_xor(g1, o, 64)); }
            if (lane == 0) {
              s_scale[0] = __fdiv_rn(g0, qmax); s_scale[1] = __fdiv_rn(g1, qmax);
              __hip_atomic_store(&s_seen, epoch, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
          }
          ok = ok || seen();
        }
        if (!ok && lane == 0) { s_fail = 1; s_scale[0] = 0.f; s_scale[1] = 0.f; st_dev_u32(p.status, 2u); }
      } else if (e == 0) {
        s_scale[0] = st0; s_scale[1] = st1;
      }
      __syncthreads();   // P2
      if (wave == RES_WORKERS) stamp(l, 1);
      // ---------------- exchange, step B: every workgroup writes the codes of what it produced
      {
        const float s0 = s_scale[0], s1 = s_scale[1];
        auto q1 = [&](float v, float s) __attribute__((always_inline)) {
          const float q = fminf(fmaxf(rintf(__fdiv_rn(v, s)), -qmax), qmax);
          return s > 0.f ? (int)q : 0;
        };
        uint32_t* qw = reinterpret_cast<uint32_t*>(ly.qin);
        if (l == 0) {
          const int in = ly.in, q4 = in >> 2, n4 = p.T * q4;
          const float4* x4 = reinterpret_cast<const float4*>(p.x);
          for (int i = wg * 256 + e; i < n4; i += G * 256) {
            const float4 v = x4[i];
            const int tq = i / q4, k = (i - tq * q4) * 4;
            const uint32_t c = (uint32_t)(uint8_t)q1(v.x, s0) | ((uint32_t)(uint8_t)q1(v.y, s0) << 8) | ((uint32_t)(uint8_t)q1(v.z, s0) << 16) |
                               ((uint32_t)(uint8_t)q1(v.w, s0) << 24);
            st_dev_u32(&qw[(((k >> 6) * 64 + ((k >> 4) & 3) * 16 + tq) * 16 + (k & 15)) >> 2], c);
          }
        } else {
          for (int u = 0; u < nu_prev; ++u) {
            const int ep = eoff_prev + u * dstride_of(l - 1) + lp.nsub * 16;
            const int n_out = lp.gated ? 1 : dword(ep + 1);
            for (int o = 0; o < n_out; ++o) {
              const int col = dword(ep + 26 + o) * 16 + ch;
#pragma unroll
              for (int m = 0; m < 2; ++m)
                if (m < n_in) {
                  int c = 0;
                  if (tok) {
                    const int si = (u * 4 + o) * 2 + m;
                    float v;
                    if (si < RES_STASH) {
                      v = stash[si * 256 + e];
                    } else {
                      __builtin_amdgcn_s_waitcnt(0x0F70);   // this thread's own store of the value has completed
                      v = __uint_as_float(ld_dev_u32(reinterpret_cast<const uint32_t*>(lp.out + ((size_t)m * p.T + t) * lp.out_w + col)));
                    }
                    c = q1(v, m == 0 ? s0 : s1);
                  }
                  // four neighbouring channels of a token are four neighbouring bytes of a fragment
                  uint32_t w = (uint32_t)(uint8_t)c;
                  w |= (uint32_t)(uint8_t)__shfl_down(c, 1, 64) << 8;
                  w |= (uint32_t)(uint8_t)__shfl_down(c, 2, 64) << 16;
                  w |= (uint32_t)(uint8_t)__shfl_down(c, 3, 64) << 24;
                  if ((ch & 3) == 0 && tok)
                    st_dev_u32(&qw[((size_t)m * ly.nks * 1024 + (size_t)(((col >> 6) * 64 + ((col >> 4) & 3) * 16 + t) * 16 + (col & 15))) >> 2], w);
                }
            }
          }
        }
        // codes beyond in_features are zero: the first workgroup writes them
        if (wg == 0) {
          const int pad4 = (ly.in_pad - ly.in) >> 2;
          for (int i = e; i < p.T * pad4 * n_in; i += 256) {
            const int m = i / (p.T * pad4), r = i - m * (p.T * pad4);
            const int tq = r / pad4, k = ly.in + (r - tq * pad4) * 4;
            st_dev_u32(&qw[((size_t)m * ly.nks * 1024 + (size_t)(((k >> 6) * 64 + ((k >> 4) & 3) * 16 + tq) * 16 + (k & 15))) >> 2], 0u);
          }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's device-scope stores have completed
      }
      __syncthreads();   // P3
      if (wave == RES_WORKERS) stamp(l, 2);
      ++epoch;
      grid_wait();
      if (wave == RES_WORKERS) stamp(l, 3);
      __syncthreads();   // P4: the workers may read the codes entering layer l

      // ---------------- the layer's units
      const float sx0 = s_scale[0], sx1 = s_scale[1];
      const int nu = units_of(ly.n_units);
      const bool last = l == p.L - 1;
      // the layer's description, read from the kernel arguments once (not once per use inside the units' epilogues)
      const int e_reduce = ly.reduce, e_xm = ly.xm, e_act = ly.act, e_pre = ly.res_pre_act, e_gated = ly.gated, e_outw = ly.out_w;
      const int e_resm = ly.res_members, e_resdev = ly.res_device, e_nsub = ly.nsub, e_stride = dstride_of(l), e_M = p.M, e_T = p.T;
      const long long e_resms = ly.res_mstride;
      const float* e_bias = ly.bias;
      const float* e_res = ly.res;
      const float* e_scales = ly.scales;
      float* e_out = ly.out;
      const int e_klo0 = p.member_lo[0], e_khi0 = p.member_hi[0], e_klo1 = p.member_lo[1], e_khi1 = p.member_hi[1];
      const bool fold_sx = e_reduce && e_M > 1;
      mx_out[0] = 0.f; mx_out[1] = 0.f;
      for (int u = 0; u < nu; ++u) {
        int d[32];   // the unit's descriptor: scalar registers
#pragma unroll
        for (int i = 0; i < 32; ++i) d[i] = dword(eoff + u * e_stride + e_nsub * 16 + i);
        const int n_items = d[0], n_out = e_gated ? 1 : d[1];
        // Every global load of the unit's epilogue is issued here, before the unit's barrier, and every
        // result is computed before the first store: a wait for a load also waits for the stores
        // before it, and a device-scope (write-through) store takes more than a microsecond to complete.
        float scv[PIPE_RES_MAX_ITEMS];
#pragma unroll
        for (int i = 0; i < PIPE_RES_MAX_ITEMS; ++i) scv[i] = i < n_items ? e_scales[(size_t)d[18 + i] * 16 + ch] : 0.f;
        float bsv[4] = {0.f, 0.f, 0.f, 0.f};   // plain: bias of output o; gated: bias of the gate and of the up channel
        float rsv[4][2];                         // skip tensor: what output o of member m (or the member sum) adds
#pragma unroll
        for (int o = 0; o < 4; ++o) { rsv[o][0] = 0.f; rsv[o][1] = 0.f; }
        if (e_gated) {
          if (e_bias != nullptr) { bsv[0] = e_bias[d[27] * 16 + ch]; bsv[1] = e_bias[d[28] * 16 + ch]; }
        } else {
#pragma unroll
          for (int o = 0; o < 4; ++o) {
            if (o >= n_out) continue;
            const int col = d[26 + o] * 16 + ch;
            if (e_bias != nullptr) bsv[o] = e_bias[col];
            if (e_res != nullptr) {
#pragma unroll
              for (int m = 0; m < 2; ++m) {
                if (m >= e_M || (e_reduce && m > 0)) continue;
                // the members summed into this output each add their own skip tensor (members kept apart:
                // member m adds its own if it has one)
                const int n_res = e_reduce ? e_resm : (m < e_resm ? 1 : 0);
                const float* rp = e_res + (size_t)(e_reduce ? 0 : m) * e_resms + (size_t)min(t, e_T - 1) * e_outw + col;
                float rsum = 0.f;
                for (int mm = 0; mm < n_res; ++mm) {
                  // a tensor an earlier layer of this launch produced is read with device scope
                  const float* rq = rp + (size_t)mm * e_resms;
                  rsum += e_resdev ? __uint_as_float(ld_dev_u32(reinterpret_cast<const uint32_t*>(rq))) : *rq;
                }
                rsv[o][m] = rsum;
              }
            }
          }
        }
        __syncthreads();   // the workers have added up this unit's tiles
        if (wave == RES_WORKERS && u == 0) stamp(l, 5);
        int a_it[PIPE_RES_MAX_ITEMS];
#pragma unroll
        for (int i = 0; i < PIPE_RES_MAX_ITEMS; ++i) {
          a_it[i] = i < n_items ? tile[buf][i][fidx] : 0;
          if (i < n_items) tile[buf][i][fidx] = 0;
        }
        int rs[2] = {0, 0};
        if (OFF != 0) {
#pragma unroll
          for (int m = 0; m < XM; ++m) { rs[m] = tile[buf][PIPE_RES_MAX_ITEMS + m][fidx]; tile[buf][PIPE_RES_MAX_ITEMS + m][fidx] = 0; }
        }
        buf ^= 1;
        float vout[4][2];   // output o of member m (the member sum in vout[o][0] when members are summed)
#pragma unroll
        for (int o = 0; o < 4; ++o) { vout[o][0] = 0.f; vout[o][1] = 0.f; }
        if (e_gated) {
          // items with slot 0 are the gate block's orders, slot 1 the up block's; h = SiLU(gate) * up per member
#pragma unroll
          for (int m = 0; m < 2; ++m) {
            if (m >= e_M) continue;
            const int k_lo = m == 0 ? e_klo0 : e_klo1, k_hi = m == 0 ? e_khi0 : e_khi1;
            float gs = 0.f, us = 0.f;
#pragma unroll
            for (int i = 0; i < PIPE_RES_MAX_ITEMS; ++i) {
              const int kk = d[2 + i], sl = d[10 + i];
              if (i >= n_items || kk < k_lo || kk > k_hi) continue;
              const int a = a_it[i] - OFF * rs[0];
              if (sl == 0) gs = fmaf(scv[i], (float)a, gs); else us = fmaf(scv[i], (float)a, us);
            }
            const float vg = fmaf(sx0, gs, m == 0 ? bsv[0] : 0.f), vu = fmaf(sx0, us, m == 0 ? bsv[1] : 0.f);
            vout[0][m] = vg / (1.f + expf(-vg)) * vu;
          }
        } else {
#pragma unroll
          for (int o = 0; o < 4; ++o) {
            if (o >= n_out) continue;
            float yacc = 0.f;
#pragma unroll
            for (int m = 0; m < 2; ++m) {
              if (m >= e_M) continue;
              const int st_m = e_xm == 1 ? 0 : m;
              const int rsm = st_m == 0 ? rs[0] : rs[1];
              const float sx = st_m == 0 ? sx0 : sx1;
              const int k_lo = m == 0 ? e_klo0 : e_klo1, k_hi = m == 0 ? e_khi0 : e_khi1;
#pragma unroll
              for (int i = 0; i < PIPE_RES_MAX_ITEMS; ++i) {
                const int kk = d[2 + i], sl = d[10 + i];
                if (i >= n_items || sl != o || kk < k_lo || kk > k_hi) continue;
                const int a = a_it[i] - OFF * rsm;
                const float sc = fold_sx ? scv[i] * sx : scv[i];
                yacc = fmaf(sc, (float)a, yacc);
              }
              if (fold_sx && m + 1 < e_M) continue;
              const float bm = (m == 0 || fold_sx) ? bsv[o] : 0.f;
              float v = fold_sx ? yacc + bm : fmaf(sx, yacc, bm);   // same rounding as the per-layer kernels
              yacc = 0.f;
              const float rsum = rsv[o][e_reduce ? 0 : m];
              if (e_pre) v += rsum;
              if (e_act == PIPE_ACT_GELU) v = gelu_erf_r(v);
              else if (e_act == PIPE_ACT_RELU) v = fmaxf(v, 0.f);
              if (!e_pre) v += rsum;
              vout[o][e_reduce ? 0 : m] = v;
            }
          }
        }
        if (wave == RES_WORKERS && u == 0) stamp(l, 6);
        // ---- stores: the last layer's result plainly, a hidden tensor with device scope (other workgroups'
        // skips read it), into the stash (this thread quantizes it in the next exchange), and its max
        if (tok) {
#pragma unroll
          for (int o = 0; o < 4; ++o) {
            if (o >= n_out) continue;
            const int col = d[26 + o] * 16 + ch;
#pragma unroll
            for (int m = 0; m < 2; ++m) {
              if (m >= (e_reduce ? 1 : e_M)) continue;
              const float v = vout[o][m];
              float* dst = e_out + ((size_t)m * e_T + t) * e_outw + col;
              if (last) {
                *dst = v;
              } else {
                st_dev_u32(reinterpret_cast<uint32_t*>(dst), __float_as_uint(v));
                const int si = (u * 4 + o) * 2 + m;
                if (si < RES_STASH) stash[si * 256 + e] = v;
                if (m == 0) mx_out[0] = fmaxf(mx_out[0], fabsf(v)); else mx_out[1] = fmaxf(mx_out[1], fabsf(v));
              }
            }
          }
        }
      }
      if (wave == RES_WORKERS) stamp(l, 4);
    }
    if (wg == 0 && e == 0 && epoch != epoch0) st_dev_u32(p.gen, epoch);
  }
  if (p.trace != nullptr) {
    __syncthreads();
    if ((int)threadIdx.x < p.L * 8) p.trace[(size_t)wg * p.L * 8 + threadIdx.x] = (&s_ts[0][0])[threadIdx.x];
  }
}

template <int BITS, int XM>
int launch_res(const ResParams& p, hipEvent_t ev0, hipEvent_t ev1, hipStream_t st) {
  constexpr int RD = (XM == 2 && BITS == 2) ? 2 : 4;   // rounds of code registers; two tensors of ternary fragments leave room for two
  static bool attr_set = false;
  if (!attr_set) {
    PIPE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&chain_resident_kernel<BITS, XM, RD>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, RES_PAD_LDS));
    attr_set = true;
  }
  if (pipe_dry_run()) return PIPE_OK;
  if (ev0 != nullptr)
    hipExtLaunchKernelGGL((chain_resident_kernel<BITS, XM, RD>), dim3((unsigned)p.G), dim3(RES_THREADS), RES_PAD_LDS, st, ev0, ev1, 0, p);
  else
    hipLaunchKernelGGL((chain_resident_kernel<BITS, XM, RD>), dim3((unsigned)p.G), dim3(RES_THREADS), RES_PAD_LDS, st, p);
  PIPE_HIP(hipGetLastError());
  return PIPE_OK;
}

}  // namespace

// ------------------------------------------------------------------ host side
// Work units of the resident kernel for one expansion.  kind 0: groups of output row blocks with all
// their orders, at most 4 items each, when there are at least as many groups as workgroups, else one unit per
// output row block; kind 1: a gate||up layer as (gate block, up block) pairs, two sub-units of at most 4 items.
int pipe_resident_tables(const pipe_expansion* ce, int kind, int G, ResidentTables* out) {
  pipe_expansion* e = const_cast<pipe_expansion*>(ce);
  ResidentTables& t = e->res_tables[kind];
  if (t.subs_dev != nullptr && t.G == G) { *out = t; return PIPE_OK; }
  if (pipe_capturing()) return PIPE_ENOTREADY;
  if (e->bin_cap != 4 || e->K > 4) return PIPE_ESHAPE;
  // kind 0: units of at most 4 items and 4 output row blocks, formed here from the row blocks' stored orders:
  // row blocks with the most orders first, those with equal sets of orders next to each other, each into the
  // most recent of the last 64 units that still has room.  (The bins of the weight-streaming kernel fix where
  // the codes lie in memory and are packed for the fewest unused positions; units need no neighbours in
  // memory, and this grouping measured 6 % faster on an 8-layer stack than units taken from those bins: its
  // units hold row blocks of like weight, so fewer units carry several outputs through the epilogue.)
  struct RbItems { uint32_t mask; int pop; int rb; };
  struct UnitBin { int n_items, n_out, k[4], slot[4], out_rb[4], pos[4]; };
  std::vector<UnitBin> bins;
  if (kind == 0) {
    std::vector<RbItems> rbs(e->n_rb);
    for (int rb = 0; rb < e->n_rb; ++rb) {
      uint32_t mask = 0;
      for (int kk = 0; kk < e->K; ++kk)
        if (e->pos_of[(size_t)kk * e->n_rb + rb] >= 0) mask |= 1u << kk;
      rbs[rb] = RbItems{mask, __builtin_popcount(mask), rb};
    }
    std::stable_sort(rbs.begin(), rbs.end(), [](const RbItems& a, const RbItems& b) {
      if (a.pop != b.pop) return a.pop > b.pop;
      if (a.mask != b.mask) return a.mask < b.mask;
      return a.rb < b.rb;
    });
    std::vector<int> room;
    for (const RbItems& it : rbs) {
      int which = -1;
      for (int j = (int)bins.size() - 1; j >= 0 && j >= (int)bins.size() - 64; --j)
        if (room[j] >= it.pop) { which = j; break; }
      if (which < 0) {
        bins.push_back(UnitBin{});
        room.push_back(4);
        which = (int)bins.size() - 1;
      }
      UnitBin& bn = bins[which];
      const int slot = bn.n_out++;
      bn.out_rb[slot] = it.rb;
      for (int kk = 0; kk < e->K; ++kk) {
        const int32_t q = e->pos_of[(size_t)kk * e->n_rb + it.rb];
        if (q < 0) continue;
        const int i = bn.n_items++;
        bn.k[i] = kk; bn.slot[i] = slot;
        bn.pos[i] = q;
      }
      room[which] -= it.pop;
    }
  }
  const int n_bins = (int)bins.size();
  std::vector<int32_t> subs, epi;
  int n_units = 0, nsub = 1;
  auto push_sub = [&](const int* pos, const int* k, int n, int slot0, int last) {
    int32_t s[16] = {0};
    for (int r = 0; r < 4; ++r) { s[r] = pos[r < n ? r : 0]; s[4 + r] = r < n ? k[r] : 0; }
    s[8] = n; s[9] = slot0; s[10] = last;
    subs.insert(subs.end(), s, s + 16);
  };
  auto push_epi = [&](int n_items, int n_out, const int* k, const int* slot, const int* pos, const int* orb) {
    int32_t s[32] = {0};
    s[0] = n_items; s[1] = n_out;
    for (int i = 0; i < n_items; ++i) { s[2 + i] = k[i]; s[10 + i] = slot[i]; s[18 + i] = pos[i]; }
    for (int o = 0; o < 4; ++o) s[26 + o] = orb[o];
    epi.insert(epi.end(), s, s + 32);
  };
  if (kind == 0) {
    const bool by_bin = n_bins >= G;   // (one unit per output row block whenever bins deal unevenly measured slower: the per-unit barrier and epilogue cost more than the imbalance)
    struct U { int n; int pos[4], k[4], slot[4], orb[4], n_out; };
    std::vector<U> us;
    for (int b = 0; b < n_bins; ++b) {
      const UnitBin& bn = bins[b];
      if (by_bin) {
        U u{};
        u.n = bn.n_items; u.n_out = bn.n_out;
        for (int i = 0; i < bn.n_items; ++i) { u.pos[i] = bn.pos[i]; u.k[i] = bn.k[i]; u.slot[i] = bn.slot[i]; }
        for (int o = 0; o < bn.n_out; ++o) u.orb[o] = bn.out_rb[o];
        us.push_back(u);
      } else {
        for (int o = 0; o < bn.n_out; ++o) {
          U u{};
          u.n_out = 1; u.orb[0] = bn.out_rb[o];
          for (int i = 0; i < bn.n_items; ++i)
            if (bn.slot[i] == o) { u.pos[u.n] = bn.pos[i]; u.k[u.n] = bn.k[i]; u.slot[u.n] = 0; ++u.n; }
          us.push_back(u);
        }
      }
    }
    std::stable_sort(us.begin(), us.end(), [](const U& a, const U& b) { return a.n > b.n; });
    for (const U& u : us) {
      push_sub(u.pos, u.k, u.n, 0, 1);
      push_epi(u.n, u.n_out, u.k, u.slot, u.pos, u.orb);
    }
    n_units = (int)us.size();
  } else {
    if (e->n_rb % 2 != 0) return PIPE_ESHAPE;
    nsub = 2;
    const int half = e->n_rb / 2;
    struct P { int rb; int n; };
    std::vector<P> ps;
    auto items_of = [&](int rb, int* pos, int* k) {
      int n = 0;
      for (int kk = 0; kk < e->K; ++kk) {
        const int32_t q = e->pos_of[(size_t)kk * e->n_rb + rb];
        if (q >= 0) { pos[n] = q; k[n] = kk; ++n; }
      }
      return n;
    };
    for (int rb = 0; rb < half; ++rb) {
      int pos[4], k[4];
      ps.push_back(P{rb, items_of(rb, pos, k) + items_of(rb + half, pos, k)});
    }
    std::stable_sort(ps.begin(), ps.end(), [](const P& a, const P& b) { return a.n > b.n; });
    for (const P& pr : ps) {
      int pg[4], kg[4], pu[4], ku[4];
      const int ng = items_of(pr.rb, pg, kg), nu = items_of(pr.rb + half, pu, ku);
      push_sub(pg, kg, ng, 0, 0);
      push_sub(pu, ku, nu, 4, 1);
      int k8[8] = {0}, slot8[8] = {0}, pos8[8] = {0};
      // the epilogue indexes the LDS tiles: gate items at 0.., up items at 4..
      int kk[8] = {0}, ss[8] = {0}, pp[8] = {0};
      for (int i = 0; i < ng; ++i) { kk[i] = kg[i]; ss[i] = 0; pp[i] = pg[i]; }
      for (int i = 0; i < nu; ++i) { kk[4 + i] = ku[i]; ss[4 + i] = 1; pp[4 + i] = pu[i]; }
      // items the blocks do not have: order -1 matches no member
      for (int i = ng; i < 4; ++i) kk[i] = -1;
      for (int i = nu; i < 4; ++i) kk[4 + i] = -1;
      (void)k8; (void)slot8; (void)pos8;
      const int orb[4] = {pr.rb, pr.rb, pr.rb + half, 0};
      int32_t s[32] = {0};
      s[0] = 8; s[1] = 1;
      for (int i = 0; i < 8; ++i) { s[2 + i] = kk[i]; s[10 + i] = ss[i]; s[18 + i] = pp[i]; }
      for (int o = 0; o < 4; ++o) s[26 + o] = orb[o];
      epi.insert(epi.end(), s, s + 32);
    }
    n_units = (int)ps.size();
  }
  int32_t *sd = nullptr, *ed = nullptr;
  PIPE_HIP(hipMalloc(&sd, subs.size() * 4));
  if (hipMalloc(&ed, epi.size() * 4) != hipSuccess) { (void)hipFree(sd); return PIPE_ENOMEM; }
  if (hipMemcpy(sd, subs.data(), subs.size() * 4, hipMemcpyHostToDevice) != hipSuccess ||
      hipMemcpy(ed, epi.data(), epi.size() * 4, hipMemcpyHostToDevice) != hipSuccess) {
    (void)hipFree(sd); (void)hipFree(ed);
    return PIPE_EDEVICE;
  }
  if (t.subs_dev) (void)hipFree(t.subs_dev);
  if (t.epi_dev) (void)hipFree(t.epi_dev);
  t.subs_dev = sd; t.epi_dev = ed; t.n_units = n_units; t.nsub = nsub; t.G = G;
  *out = t;
  return PIPE_OK;
}

int pipe_resident_workgroups() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 64;
    cus = std::min(n, 1024);
  }
  return cus;
}

int launch_resident_chain(const ResidentArgs& a, hipStream_t st) {
  if (a.L < 1 || a.L > PIPE_RES_MAX_LAYERS || a.T < 1 || a.T > 16 || a.M < 1 || a.M > PIPE_RES_MAX_M) return PIPE_ESHAPE;
  ResParams p;
  std::memset(&p, 0, sizeof(p));
  p.L = a.L; p.T = a.T; p.M = a.M; p.G = a.G;
  for (int m = 0; m < a.M; ++m) {
    p.member_lo[m] = a.member_lo[m]; p.member_hi[m] = a.member_hi[m];
    for (int k = a.member_lo[m]; k <= a.member_hi[m] && k < 4; ++k) p.member_of[k] = m;
  }
  p.x = a.x; p.s_static = a.s_static; p.act_qmax = g_act_qmax_host;
  p.flags = a.flags; p.amax_tag = a.amax_tag; p.gen = a.gen; p.status = a.status;
  p.spin_limit = g_resident_spin_limit;
  p.trace = g_resident_trace;
  const int bits = a.layers[0].e->bits;
  for (int l = 0; l < a.L; ++l) {
    const ResidentLayerArgs& la = a.layers[l];
    const pipe_expansion* e = la.e;
    if (e->bits != bits || e->bin_cap != 4) return PIPE_ESHAPE;
    ResLayer& ly = p.layer[l];
    ly.codes = e->codes_dev; ly.scales = e->scales_all_dev;
    ly.subs = la.tables.subs_dev; ly.epi = la.tables.epi_dev;
    ly.n_units = la.tables.n_units; ly.nsub = la.tables.nsub;
    ly.bias = la.bias; ly.out = la.out; ly.res = la.res; ly.res_mstride = la.res_mstride;
    ly.qin = la.qin;
    ly.n_tiles = e->in_pad / (512 / e->bits); ly.nks = e->nks;
    ly.out_w = la.gated ? e->out / 2 : e->out;
    ly.in = e->in; ly.in_pad = e->in_pad;
    ly.xm = l == 0 ? 1 : a.M;
    ly.act = la.act; ly.res_members = la.res_members; ly.res_pre_act = la.res_pre_act; ly.gated = la.gated;
    ly.reduce = l == a.L - 1 ? 1 : 0;
    ly.res_device = la.res_device;
    ly.s_in[0] = la.s_in[0]; ly.s_in[1] = la.s_in[1];
  }
  // the descriptors of the busiest workgroup (the first) have to fit their LDS copy
  int desc_ints = 0;
  for (int l = 0; l < a.L; ++l) desc_ints += ceil_div(p.layer[l].n_units, p.G) * (p.layer[l].nsub * 16 + 32);
  if (desc_ints > PIPE_RES_DESC_INTS) return PIPE_ESHAPE;
  if (a.M == 1) {
    switch (bits) {
      case 8: return launch_res<8, 1>(p, a.ev_start, a.ev_stop, st);
      case 4: return launch_res<4, 1>(p, a.ev_start, a.ev_stop, st);
      default: return launch_res<2, 1>(p, a.ev_start, a.ev_stop, st);
    }
  }
  switch (bits) {
    case 8: return launch_res<8, 2>(p, a.ev_start, a.ev_stop, st);
    case 4: return launch_res<4, 2>(p, a.ev_start, a.ev_stop, st);
    default: return launch_res<2, 2>(p, a.ev_start, a.ev_stop, st);
  }
}
