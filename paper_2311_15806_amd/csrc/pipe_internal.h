// Internal declarations shared by the HIP sources of the PIPE library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <vector>

#include "../../include/pipe.h"

// ---------------------------------------------------------------------------------------
// Data layout in HBM
//
// Quantized activations ("fragment layout"): tokens are padded to a multiple of TOK_TILE (16 for the streaming kernel) and
// in_features to a multiple of IN_PAD (pad entries are 0).  A fragment holds 16 tokens x 64
// consecutive k as 64 lanes x 16 bytes: lane = kc*16 + n holds token n, k = 64*ks + 16*kc + e,
// e = 0..15.  Fragments are stored [token_block][ks], 1 KiB each, so that one wave reads a
// fragment with a single fully coalesced 16-byte-per-lane load, already in the register
// layout of the B operand of v_mfma_i32_16x16x64_i8.
//
// Packed codes of one order ("tile layout"): stored rows are grouped in row blocks of 16
// (compact index crb = kept_group_slot * (group/16) + block).  A tile holds 16 rows x KSUP
// k-values (KSUP = 512/bits) as 64 lanes x 16 bytes; lane = kc*16 + r holds, for row r and
// each 64-k step j inside the tile, the 16 codes k = KSUP*ksup + 64*j + 16*kc + e.  Tiles are
// stored [crb][ksup].  Codes are stored offset-binary (code + 2^(bits-1) for 4 bit, code + 1
// for ternary; int8 is stored as is) so that unpacking is a shift and a mask:
//   bits = 4: step j uses dwords 2j, 2j+1; code e = 4i + byte sits in dword 2j + (i >> 1) at
//             bit 8*byte + 4*(i & 1)      =>  out dword i = (w >> 4*(i&1)) & 0x0F0F0F0F
//   bits = 2: step j uses dword j; code e = 4i + byte sits at bit 8*byte + 2i
//                                          =>  out dword i = (w >> 2i) & 0x03030303
// The exact integer accumulator is recovered as acc - offset * rowsum(Qx[t,:]).
// ---------------------------------------------------------------------------------------
constexpr int PIPE_MAX_K = 16;
constexpr int IN_PAD = 256;    // in_features padded to this (largest KSUP)
constexpr int TOK_TILE = 64;   // tokens per tile of the tiled kernel; token padding of its buffers
constexpr int RB = 16;         // rows per row block
constexpr int NRB_TILE = 16;   // row blocks per column tile of the tiled kernel

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
static inline int64_t round_up64(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

// A bin of the weight-streaming kernel: up to STREAM_BIN_CAP stored row blocks that together
// hold every order of n_out output row blocks (items of one output row block are adjacent and
// in ascending order k).
constexpr int STREAM_BIN_CAP = 16;
constexpr int PIPE_STREAM_MAX_T = 128;   // the weight-streaming kernel serves up to this many tokens
constexpr int PIPE_FUSED_QUANT_MAX_T = 1;     // the streaming kernel quantizes a single token itself (no quantizer launch); every workgroup repeats the work, which costs more than the launch it saves from 2 tokens on
constexpr int PIPE_FUSED_QUANT_MAX_IN = 8192; // ... for layers of at most this many (padded) input features
constexpr int PIPE_QUANT1_MAX_T = 64;    // the one-launch quantizer (every token's workgroup scans the whole input for the maximum) up to this many
constexpr int PIPE_MAX_SPLIT = 8;   // workgroups per bin of the weight-streaming kernel, at most
struct StreamBin {
  int32_t n_items, n_out;
  int32_t k[STREAM_BIN_CAP];       // 0-based order of the item
  int32_t slot[STREAM_BIN_CAP];    // index into out_rb
  int32_t out_rb[STREAM_BIN_CAP];  // output row block (channel / 16)
};

struct PipeOrder {
  int n_kept = 0;               // groups stored at this order
  int32_t* gids_dev = nullptr;  // [n_kept] ascending
  float* scales_dev = nullptr;  // [n_kept*group]: while the expansion is built, then freed
  uint8_t* packed_dev = nullptr;  // tile layout in compact row order: while the expansion is built, then freed
  size_t packed_bytes = 0;
  std::vector<int32_t> gids;    // host copy
  int32_t* pos_dev = nullptr;   // [n_kept*group/16] position of compact row block c in codes_dev / scales_all_dev
  std::vector<int32_t> pos;     // host copy
};

// Tile schedule of the tiled kernel for one grouping of the orders into members.
//
// All orders of a member multiply the same Q(x), so within a member a wave may take its row
// blocks' stored orders in any grouping: in pass j each row block contributes its j-th stored
// order of the member (ascending, so every output row is still summed in order k = 1..K).  A
// column tile of 16 row blocks then runs max(count) passes per member instead of one pass per
// order present anywhere in the tile: tiles need row blocks with equal order COUNTS per member,
// not equal order sets, and sorting by count vector gets close to that even for few groups and
// many orders.
//   kind 0: row blocks sorted by count vector.
//   kind 1: a gate||up layer (out = 2H, rows [0,H) gate, [H,2H) up): a tile is 8 (gate block i,
//           up block i) pairs -- sorted positions 16t..16t+7 the gate blocks, 16t+8..16t+15
//           their up blocks -- so a workgroup holds both halves of SiLU(gate)*up; rb_out is the
//           gate block (= block of the hidden channel) for both.
//   kind 2: one pass per order, pruned or not (pass j = order j): the integer export.
struct PassTables {
  unsigned long long member_nib = 0;   // member of order k in bits [4k, 4k+4)
  int M = 0, kind = 0;
  int n_ct = 0;                        // column tiles
  int n_sorted = 0;                    // 16 * n_ct rounded up to a multiple of 64
  int p_max = 0;                       // most passes any (tile, member) runs
  int32_t* rb_out_dev = nullptr;       // [n_sorted] output row block of sorted position i, or -1
  int32_t* src_dev = nullptr;          // [M][p_max][n_sorted] position of the row block's j-th stored order, or -1
  uint8_t* cnt_dev = nullptr;          // [n_ct][16] passes of member m in tile t
};
// Work units of the resident decode kernel (pipe_resident.hip), built on first use per expansion.
//   sub-unit: 16 ints  {pos[4] (items a sub-unit does not have repeat pos[0]), k[4], n_items,
//             first LDS tile of its items, 1 = last sub-unit of its unit, 5 unused}
//   unit:     32 ints  {n_items, n_out, k[8], slot[8], pos[8], out_rb[4], 2 unused}; a gate||up pair:
//             items 0-3 the gate block's orders (slot 0), 4-7 the up block's (slot 1), order -1 = absent,
//             out_rb = {hidden block, gate row block, up row block}
constexpr int PIPE_RES_MAX_LAYERS = 16;
constexpr int PIPE_RES_MAX_M = 2;
constexpr int PIPE_RES_MAX_ITEMS = 8;
constexpr int PIPE_RES_DESC_INTS = 4096;   // LDS copy of one workgroup's unit descriptors, all layers
struct ResidentTables {
  int32_t* subs_dev = nullptr;
  int32_t* epi_dev = nullptr;
  int n_units = 0, nsub = 1, G = 0;
};
struct pipe_expansion;
struct GemmArgs;
// The tables for the members of `a` (built and uploaded on first use: allocates and copies
// synchronously); nullptr with *rc set on failure.  Not thread safe per expansion.
const PassTables* pipe_get_tables(const pipe_expansion* e, const GemmArgs& a, int kind, int* rc);

struct pipe_expansion {
  int out = 0, in = 0, bits = 0, K = 0, group = 0;   // bits: width of a stored code (8, 4 or 2)
  int qbits = 0;      // width the quantizer was asked for (2..8); codes lie in +-(2^(qbits-1)-1)
  float gamma = 1.f;
  bool unstructured = false;   // orders k >= 2 keep single entries (all rows stored) instead of groups
  int n_groups = 0;
  int rbpg = 0;       // row blocks per group = group/16
  int n_rb = 0;       // out/16
  int in_pad = 0;     // in rounded up to IN_PAD
  int nks = 0;        // in_pad/64
  int device = 0;
  std::vector<PipeOrder> orders;
  // Tile schedules of the tiled kernel (PassTables below): built on first use for each grouping
  // of the orders into members, kept until the expansion is freed.
  std::vector<int32_t> pos_of;       // [K][n_rb] position (in codes_dev) of output row block rb at order k, or -1
  std::vector<PassTables> tables;
  // dense per-order codes [K][in][out] (int8, tap-major, pruned rows zero) and scales [K][out] of a depthwise layer
  // (in = kh*kw), built on first use of pipe_forward_depthwise2d
  int8_t* dw_codes_dev = nullptr;
  float* dw_scales_dev = nullptr;
  // Stored row blocks of all orders in schedule order, bin after bin of the weight-streaming kernel, which
  // addresses its codes from its block index alone: bins of 4 lie without gaps, fullest first (a bin's first
  // position follows from bin_thr), wider bins own positions [b*bin_cap, (b+1)*bin_cap) with zeros in the unused
  // ones.  The tiled and resident kernels reach the row blocks through their tables (pos_of).
  uint8_t* codes_dev = nullptr;       // [n_pos + 1][in_pad/KSUP][1 KiB]
  float* scales_all_dev = nullptr;    // [n_pos + 1][16]
  int n_bins = 0, bin_cap = 0;
  int n_pos = 0, zero_pos = 0;        // stored positions; the all-zero position behind them
  int bin_thr[3] = {0, 0, 0};         // bins of 4 (fullest first): how many hold 4, at least 3, at least 2 items
  StreamBin* bins_dev = nullptr;
  // asymmetric activations (built on first use of pipe_forward_asymmetric): per order and output channel the sum of
  // the row's codes [K][out] (pruned rows 0), C[o] = sum_k s_k[o] * wsum_k[o], and the effective bias of the last call
  int32_t* asym_wsum_dev = nullptr;
  float* asym_C_dev = nullptr;
  float* asym_bias_dev = nullptr;
  float* asym_P_dev = nullptr;        // [K][out]: s_k[o] * wsum_k[o] (member chains sum their own orders' rows)
  // split bins of the weight-streaming kernel: partial tiles, and arrival counters (zero between launches)
  int32_t* split_sum_dev = nullptr;   // [n_bins][PIPE_MAX_SPLIT][bin_cap][256]
  uint32_t* split_cnt_dev = nullptr;  // [n_bins]
  int64_t stream_bytes = 0;  // packed codes + scales + indices
  ResidentTables res_tables[2];   // resident decode kernel: plain units, gate||up pairs
  // an expansion of a convolution weight with its k axis stored tap-major, channel-minor
  // (pipe_expand_conv2d): channels, kernel size; 0 = a plain [out, in] expansion
  int conv_C = 0, conv_kh = 0, conv_kw = 0;
  uint8_t* conv_zero_dev = nullptr;   // 256 zero bytes
};

// max|.| reduction slot (fp32 bit pattern of a non-negative value).  Atomics of many waves on
// one address are served one after another (about 10 ns each, measured: 4096 of them added 40 us
// to a 23-us kernel), so a wave first reads the slot -- a device-coherent load, not serialized --
// and sends the atomic only if it would raise the value: a handful per launch instead of one per wave.
#if defined(__HIPCC__)
__device__ __forceinline__ void amax_raise(uint32_t* slot, float mx) {
  const uint32_t bits = __float_as_uint(mx);
  if (bits == 0u) return;
  if (__hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= bits) return;
  atomicMax(slot, bits);
}
#endif

// ------------------------------------------------------------------ error plumbing
void pipe_note_hip_error(hipError_t e, const char* what);
#define PIPE_HIP(call)                                   \
  do {                                                   \
    hipError_t _e = (call);                              \
    if (_e != hipSuccess) {                              \
      pipe_note_hip_error(_e, #call);                    \
      return PIPE_EDEVICE;                               \
    }                                                    \
  } while (0)

// ------------------------------------------------------------------ workspace
struct PipeWorkspace {
  void* ptr = nullptr;
  size_t bytes = 0;
};
// Returns a device buffer of at least `bytes` from slot `slot` of the workspace of the calling
// entry point's (device, stream).  Grow-only: a larger block is allocated next to the old one,
// which stays allocated until the process ends (graphs captured earlier keep its address).
// nullptr on failure; pipe_ws_error() then tells why (PIPE_ENOMEM, or PIPE_ENOTREADY when the
// stream is being captured and the block would have to grow).
void* pipe_ws_get(int slot, size_t bytes);
int pipe_ws_error();
// true while a pipe_prepare* call walks a forward entry point: sizes and schedules are set up,
// nothing is launched or copied
bool pipe_dry_run();
// true while the calling entry point's stream is being captured into a graph
bool pipe_capturing();
// every kernel launch of the library goes through this (or PIPE_LAUNCH below)
#define PIPE_KLAUNCH(...)                                   \
  do {                                                      \
    if (!pipe_dry_run()) hipLaunchKernelGGL(__VA_ARGS__);   \
  } while (0)
enum { WS_QX = 0, WS_ROWSUM, WS_SCAL, WS_Y1, WS_H, WS_QH, WS_ROWSUM_H, WS_RESID, WS_ENERGY, WS_MISC, WS_Q8X, WS_CHAIN, WS_DIAG, WS_DIAG_CODES, WS_DIAG_DENSE, WS_RES, WS_RES_Q, WS_CSUM, WS_ABIAS, WS_SLOTS };

// ------------------------------------------------------------------ expand kernels (pipe_expand.hip)
int launch_row_energy(const float* E, int out, int in, double* row_energy, hipStream_t st);
int launch_group_select(const double* row_energy, int n_groups, int group, int n_keep,
                        int32_t* gids_out, hipStream_t st);
// W [out, C*kh*kw] with rows flattened [C, kh, kw] -> rows flattened [kh, kw, C] (tap-major)
int launch_permute_conv_weight(const float* W, int out, int C, int taps, float* W_out, hipStream_t st);
// channels-last int8 codes of a convolution input and the per-pixel sums of their channels (zero on entry)
int launch_quantize_nhwc_sums(const float* x, int N, int C, int HW, int nhwc, float s_static, const uint32_t* amax_bits,
                              int8_t* q8, int32_t* csum, float* scale_out, hipStream_t st);
int launch_fold_batchnorm(const float* W, const float* b, const float* gamma, const float* beta, const float* mean,
                          const float* var, float eps, int out, int in, float* W_out, float* b_out, hipStream_t st);
// An entry takes part if the bit pattern of its magnitude exceeds thr_key, or equals it with a
// flat index <= tie_cut; PIPE_NO_MASK_KEY / PIPE_NO_MASK_CUT: every entry.
constexpr uint32_t PIPE_NO_MASK_KEY = 0u;
constexpr long long PIPE_NO_MASK_CUT = 0x7fffffffffffffffll;
int launch_quantize_rows(float* E, int out, int in, int in_pad, int bits, int qbits, int group,
                         const int32_t* gids, int n_kept, float* scales, uint8_t* packed,
                         const int8_t* given, uint32_t thr_key, long long tie_cut, hipStream_t st);
// unstructured mask: bit pattern of the keep-th largest magnitude among the n entries of E and the
// flat index up to which entries of exactly that magnitude are kept; hist_dev: 2049 words of scratch
int select_entry_threshold(const float* E, long long n, long long keep, uint32_t* hist_dev, uint32_t* thr_key,
                           long long* tie_cut, hipStream_t st);
// the rows an order quantizes, compact [n_kept*group, in], and their scales max|row| / q_max
int launch_gather_rows(const float* E, int in, int qbits, int group, const int32_t* gids, int n_kept,
                       float* rows_out, float* scales_out, hipStream_t st);
int launch_unpack_codes(const uint8_t* packed, const int32_t* rb_map_dev, int bits, int rows, int in, int in_pad,
                        int8_t* codes, hipStream_t st);
int launch_gather_row_blocks(const uint8_t* codes_k, const float* scales_k, const int32_t* pos_of_dev, int n_crb,
                             int64_t rb_bytes, uint8_t* codes_all, float* scales_all, hipStream_t st);

// ------------------------------------------------------------------ activation kernels (pipe_quant.hip)
// amax_bits: device uint32 holding the bit pattern of max|x| (must be zeroed first).
int launch_zero_u32(uint32_t* p, int n, hipStream_t st);
// asymmetric activation codes: range slots {max(x,0), max(-x,0)}; unsigned a-bit codes stored minus 2^(a-1) in the
// fragment layout with their token sums, scale and 2^(a-1) - z to device memory; the token-free correction as a bias
int launch_minmax(const float* x, int64_t n, uint32_t* slots, hipStream_t st);
int launch_quantize_asym(const float* x, int T, int in, int in_pad, int T_pad, const uint32_t* hi_slot, const uint32_t* nlo_slot, int act_bits,
                         uint8_t* qx_frag, int32_t* rowsum, uint8_t* qx_rowmajor, float* scale_out, int32_t* dz_out,
                         hipStream_t st);
int launch_quantize_im2col_asym(const float* x, int N, int C, int H, int W, int kh, int kw, int stride, int pad, int nhwc,
                                int Ho, int Wo, int in_pad, int T_pad, const uint32_t* hi_slot, const uint32_t* nlo_slot,
                                int act_bits, int8_t* q8_scratch, uint8_t* qx_frag, int32_t* rowsum, float* scale_out,
                                int32_t* dz_out, hipStream_t st);
int launch_asym_bias(const float* bias, const float* C, const float* scale, const int32_t* dz, float* out, int n,
                     uint32_t* slots, hipStream_t st);
int launch_asym_acc_fix(int32_t* acc, const int32_t* wsum, const int32_t* dz, int K, int T, int out, hipStream_t st);
// member chains with asymmetric codes: per-member offset vectors [M][n] (reduce = 0; the bias joins member 0) or their
// sum plus the bias [n] (reduce = 1) from P[k][o] = s_k[o] * sum_i q_k[o,i]; clears n_clear words at `clear`
struct MemberRanges {
  int M;
  int lo[PIPE_MAX_K], hi[PIPE_MAX_K];
};
int launch_asym_bias_members(const float* bias, const float* P, const float* scale, int scale_stride, const int32_t* dz,
                             int dz_stride, int M, const int* lo, const int* hi, int reduce, float* outv, int n, uint32_t* clear,
                             int n_clear, hipStream_t st);
int launch_row_code_sums(const int8_t* codes, int rows, int in, int group, const int32_t* gids, int32_t* wsum, hipStream_t st);
// launch_absmax also zeroes n_zero ints at zero_me (the code sums of the quantizer that follows).
int launch_absmax(const float* x, int64_t n, uint32_t* amax_bits, int32_t* zero_me, int n_zero, hipStream_t st);
// Quantize x [T, in] into the fragment layout (padded region written as zero), row sums and
// optionally row-major int8.  scale: if s_static > 0 use it, else amax/127 from amax_bits.
// Writes the scale used to *scale_out (device).
int launch_quantize_act(const float* x, int T, int in, int in_pad, int T_pad, float s_static,
                        const uint32_t* amax_bits, uint8_t* qx_frag, int32_t* rowsum, bool rowsum_is_zero,
                        int8_t* qx_rowmajor, float* scale_out, hipStream_t st);
// Decode-sized batches (T <= 16, T_pad == 16): max|x|, scale, codes and code sums in ONE launch,
// one workgroup per member (x, qx_frag, rowsum [16 per member], scale_out [M] with member strides).
// One launch for all members: member m quantizes x + m*x_mstride ([T, in]) with its own dynamic
// scale (amax_bits[m]) into qx_frag + m*qx_mstride and rowsum + m*T_pad; scale_out[m].
int launch_quantize_members(const float* x, int64_t x_mstride, int M, int T, int in, int in_pad, int T_pad,
                            const uint32_t* amax_bits, uint8_t* qx_frag, int64_t qx_mstride, int32_t* rowsum,
                            bool rowsum_is_zero, float* scale_out, hipStream_t st);
int set_act_qmax(float qmax);   // largest activation code of all quantizers from now on (synchronous copy to the device)
// every element quantized once, in the input's own layout (scale from s_static or the max slot)
int launch_quantize_elem(const float* x, int64_t n, float s_static, const uint32_t* amax_bits, int8_t* q8,
                         float* scale_out, hipStream_t st);
int launch_quantize_small(const float* x, int64_t x_mstride, int M, int T, int in, int in_pad, float s_static,
                          const uint32_t* amax_bits, uint8_t* qx_frag, int64_t qx_mstride, int32_t* rowsum,
                          int8_t* qx_rowmajor, float* scale_out, hipStream_t st);
// Same for the virtual im2col matrix of a convolution.
int launch_quantize_im2col(const float* x, int N, int C, int H, int W, int kh, int kw, int stride,
                           int pad, int nhwc, int Ho, int Wo, int in_pad, int T_pad,
                           float s_static, const uint32_t* amax_bits, int8_t* q8_scratch, uint8_t* qx_frag,
                           int32_t* rowsum, float* scale_out, hipStream_t st);
// Hidden activation of the MLP call: h = act(y1) element-wise, plus per-member max|h| (or, with amax_neg, the
// positive and negative parts of its range apart).
int launch_mlp_act(const float* y1, int M, int T, int H, int act, float* h, uint32_t* amax_bits, uint32_t* amax_neg,
                   hipStream_t st);

// ------------------------------------------------------------------ contraction kernels
struct GemmArgs {
  const pipe_expansion* e;
  int T;                 // valid tokens
  int T_pad;             // padded tokens of the fragment buffers
  const uint8_t* qx;     // fragment layout, member stride below
  int64_t qx_mstride;    // bytes between members' activations (0 = shared input)
  const int32_t* rowsum; // [T_pad] per member
  int64_t rowsum_mstride;
  const float* s_x;      // device: activation scale per member
  int sx_mstride;        // 0 = shared
  int M;                 // members
  int member_lo[PIPE_MAX_K];  // 0-based first order of member m
  int member_hi[PIPE_MAX_K];  // 0-based last order (inclusive)
  const float* x_f32;    // streaming kernel, at most 4 tokens: the fp32 input [T, in] when the contraction quantizes it
                         // itself (then qx, rowsum and s_x are not read), else nullptr
  float s_static;        // with x_f32: the given activation scale, or <= 0 for the dynamic one
  const float* bias;     // or nullptr
  int64_t bias_mstride = 0;   // 0: one vector, added to the first member (or to the members' sum); else member m adds
                              // bias + m * bias_mstride (members kept apart: the asymmetric codes' per-member offsets)
  int reduce;            // 1: y[T,out]; 0: y[M,T,out]
  int act;               // 0 none; PIPE_ACT_GELU fused in the epilogue; PIPE_ACT_SILU_GATED: the layer is gate||up and
                         // the tiled kernel writes h = SiLU(gate)*up, [M,T,out/2] (members kept apart)
                         // PIPE_ACT_RELU; GELU and ReLU combine with `res`
  const float* res = nullptr;   // a tensor added to the output, [res_members, T, out], or nullptr
  int64_t res_mstride = 0;      // floats between its members
  int res_members = 0;          // members that add it: M, or 1 (the first member only)
  int res_pre_act = 1;          // 1: act(z + res); 0: act(z) + res
  float* y;
  int32_t* acc_out;      // debug: [K,T,out] or nullptr (then y may be nullptr)
  uint32_t* amax_out;    // per member max|output| bit pattern (or nullptr)
  uint32_t* amax_neg = nullptr;   // if set: amax_out[m] receives max(output, 0) and amax_neg[m] max(-output, 0), the
                                  // range the asymmetric quantizer of the next layer needs
  uint32_t* zero_after;  // words the kernel clears (the max|x| slots this call consumed), or nullptr
  int zero_n = 1;        // how many (at most 64)
  uint32_t* zero_big = nullptr;   // a buffer the kernel clears as well (the code sums the next layer's quantizer
  int zero_big_n = 0;             // adds into: nobody reads them while this kernel runs), any length
  hipEvent_t ev_start = nullptr, ev_stop = nullptr;   // if set: the dispatch's own begin/end timestamps
  // implicit-GEMM convolution (tiled kernel, an expansion built by pipe_expand_conv2d): the channels-last
  // codes of the input tensor, the per-pixel sums of their channels, 16 zero bytes, the geometry;
  // qx and rowsum are then not read
  const int8_t* conv_q8 = nullptr;
  const int32_t* conv_csum = nullptr;
  const uint8_t* conv_zero = nullptr;
  int conv_C = 0, conv_H = 0, conv_W = 0, conv_kh = 0, conv_kw = 0, conv_stride = 1, conv_pad = 0, conv_Ho = 0, conv_Wo = 0;
};
// Launches with the dispatch's begin/end timestamps recorded into the two events when they are set
// (the kernel alone: no event-record packets on the stream in between).
#define PIPE_LAUNCH(kernel, grid, block, st, ev0, ev1, ...)                                   \
  do {                                                                                       \
    if (pipe_dry_run()) break;                                                               \
    if ((ev0) != nullptr) hipExtLaunchKernelGGL(kernel, grid, block, 0, st, ev0, ev1, 0, __VA_ARGS__); \
    else hipLaunchKernelGGL(kernel, grid, block, 0, st, __VA_ARGS__);                         \
  } while (0)
int launch_gemm_tiled(const GemmArgs& a, hipStream_t st);
// depthwise layers: dense per-order codes and scales (built once), then the forward kernel
int pipe_depthwise_prepare(pipe_expansion* e, hipStream_t st);
int launch_quantize_to_nhwc(const float* x, int N, int C, int HW, float s_static, const uint32_t* amax_bits, float qmax,
                            int8_t* q8, float* scale_out, hipStream_t st);   // fp32 [N,C,H,W] -> int8 codes [N,H,W,C]
int launch_depthwise(const pipe_expansion* e, const int8_t* q8, const float* s_x, int N, int C, int H, int W, int kh, int kw,
                     int stride, int pad, int Ho, int Wo, int M, const int* lo, const int* hi,
                     const float* bias, int reduce, float* y, hipStream_t st);   // q8 channels last
extern float g_act_qmax_host;   // the activation quantizer's largest code (host copy of the device constant)
int launch_gemm_stream(const GemmArgs& a, hipStream_t st);
// ---- resident decode kernel (pipe_resident.hip)
struct ResidentLayerArgs {
  const pipe_expansion* e;
  ResidentTables tables;
  const float* bias;
  float* out;             // [M, T, width] (hidden layers) or [T, out] (last layer)
  const float* res;       // skip tensor or nullptr
  long long res_mstride;
  int res_members, res_pre_act, res_device;   // res_device: the skip tensor is produced inside the launch
  int act, gated;
  float s_in[PIPE_RES_MAX_M];   // > 0: given scale of member m's tensor entering the layer (layers after the first)
  uint8_t* qin;           // scratch for the codes entering the layer: M * 16 * in_pad bytes (first layer: 16 * in_pad)
};
struct ResidentArgs {
  ResidentLayerArgs layers[PIPE_RES_MAX_LAYERS];
  int L, T, M, G;
  int member_lo[PIPE_RES_MAX_M], member_hi[PIPE_RES_MAX_M];
  const float* x;
  float s_static;
  uint32_t* flags;                 // zero when allocated; the kernels keep them consistent from then on
  unsigned long long* amax_tag;
  uint32_t* gen;
  uint32_t* status;
  hipEvent_t ev_start, ev_stop;    // if set: the dispatch's own begin/end timestamps
};
int pipe_resident_workgroups();   // one per compute unit
int pipe_resident_tables(const pipe_expansion* e, int kind, int G, ResidentTables* out);
int launch_resident_chain(const ResidentArgs& a, hipStream_t st);
extern int g_decode_resident;        // 1: chains of decode-sized batches run as one resident launch
extern int g_resident_spin_limit;    // polls of a grid-wide wait before a workgroup gives up
extern unsigned long long* g_resident_trace;   // profiling buffer of the resident kernel, or nullptr
extern int g_tiled_mtb;       // token blocks per tile of the tiled kernel; 0 = automatic
extern int g_stream_ksplit;   // workgroups per bin of the streaming kernel; 0 = automatic
extern int g_decode_fusion;   // 1: batches of at most 4 tokens are quantized inside the streaming kernel
