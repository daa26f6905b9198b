/*
 * pipe.h -- C ABI of the residual-expanded quantized layer (PIPE, arXiv 2311.15806)
 *           for AMD MI355X (gfx950).
 *
 * The library computes, for one layer with weights W [out, in],
 *
 *      y = lambda_x * sum_{k=1..K} lambda_{R^k} (.) ( R^k Q(x) )  (+ b)
 *
 * where R^1 = Q(W), R^k = M^k Q(W - sum_{j<k} R^j) are low-bit integer residual
 * terms (Sec. 3.1, Eq. (2)-(3) and the masked form), Q is the symmetric
 * per-output-channel quantizer of Sec. 3 Eq. (1), M^k keeps a fraction gamma of
 * the groups of consecutive output channels at orders k >= 2 (structured mask,
 * Sec. 3.1), and the K terms may be clustered into M ensemble members
 * [K_1..K_M] whose outputs are summed after the last layer (Sec. 3.2, Fig. 2).
 * The forward formula is App. B, Eq. (define_dre).
 *
 * Conventions
 *   - Every pointer named *_dev is DEVICE memory on the current HIP device, owned
 *     by the caller; every other pointer is HOST memory owned by the caller.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All
 *     forward calls are asynchronous on that stream.  pipe_expand and the
 *     introspection calls synchronize the stream before they return.
 *   - Matrices are row-major and dense; no strides.
 *   - Every function returns PIPE_OK (0) or a negative error code and never
 *     throws or aborts.  On an error detected before launch (bad argument,
 *     shape or split) no output is written.
 *   - Scratch (quantized activations, code sums, scales, hidden activations) lives in a
 *     library-owned workspace per (device, stream): calls on different streams use disjoint
 *     scratch and may overlap in time, calls on one stream are ordered by the stream.  Two
 *     calls that use the SAME expansion must not overlap in time (its tile schedules are
 *     built on first use and the weight-streaming kernel's split bins exchange partial sums
 *     through a buffer the expansion owns).  A workspace grows on demand; a block that has
 *     been handed out is never freed before the process ends, so graphs captured earlier
 *     keep valid pointers.  Growing allocates: a forward call on a stream that is being
 *     captured never allocates or synchronizes; if it would have to (first use of that
 *     stream, a larger batch, a new grouping of the orders) it returns PIPE_ENOTREADY and
 *     launches nothing.  pipe_prepare / pipe_prepare_mlp / pipe_prepare_chain do that work
 *     ahead of time, so that the first forward call on a stream may already be captured.
 *   - The tuning switches (pipe_set_*) are process-wide and read on the host at call time;
 *     change them only while no other thread is inside a forward call.
 *   - bits: 2..8; codes lie in +-(2^(bits-1)-1): 8 int8, 4 int4 (codes in [-7,7]), 2 ternary
 *     (codes in {-1,0,1}).  Codes are stored 2, 4 or 8 bits wide: 3-bit codes occupy 4-bit fields
 *     and 5..7-bit codes bytes (the arithmetic is the same; only the packed size is not minimal).
 */
#ifndef PIPE_H_
#define PIPE_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pipe_expansion pipe_expansion; /* opaque, owned by the library */

enum {
  PIPE_OK = 0,
  PIPE_EINVAL = -1,  /* NULL pointer, bits/K/gamma/group out of range            */
  PIPE_ESHAPE = -2,  /* out % group != 0, group % 16 != 0, sizes <= 0, overflow   */
  PIPE_ENOMEM = -3,  /* device or host allocation failed                         */
  PIPE_EDEVICE = -4, /* a HIP call failed (see pipe_last_device_error)           */
  PIPE_ESPLIT = -5,  /* split entries not positive or not summing to K            */
  PIPE_ELIMIT = -7,  /* pipe_forward_noalloc: the input exceeds its fixed scratch         */
  PIPE_ENOTREADY = -6 /* the call would have to allocate or synchronize where it may not
                         (its stream is being captured into a graph): run the matching
                         pipe_prepare* call first.  Nothing was launched.                */
};

enum { PIPE_ACT_NONE = 0, PIPE_ACT_GELU = 1, PIPE_ACT_SILU_GATED = 2, PIPE_ACT_RELU = 3 };

/* Batch-normalization folding (Sec. 4.1: done before anything else): the layer
 * y = BN(W x + b), BN(z) = gamma (z - mean) / sqrt(var + eps) + beta per output channel,
 * as one affine layer W' x + b' with g = gamma / sqrt(var + eps), W'[o,:] = W[o,:] g[o],
 * b'[o] = (b[o] - mean[o]) g[o] + beta[o]; g in fp64 rounded once to fp32, the rest fp32
 * with one rounding per operation.  A conv
 * weight is passed as [out, C*kh*kw].  All pointers DEVICE; bias_dev NULL = no bias;
 * bias_out_dev NULL = not wanted; W_out_dev may equal W_dev.  eps >= 0.              */
int pipe_fold_batchnorm(const float* W_dev, const float* bias_dev, const float* gamma_dev,
                        const float* beta_dev, const float* mean_dev, const float* var_dev,
                        float eps, int out, int in, float* W_out_dev, float* bias_out_dev,
                        void* stream);

/* Build the expansion (R^1..R^K) of W (Sec. 3.1, Eq. (2)-(3); mask: masked Eq.).
 *   W_dev   [out, in] fp32, read only.
 *   bits    2..8.               K >= 1 (at most 16).
 *   gamma   in (0,1]: fraction of channel groups KEPT at every order k >= 2
 *           (n_keep = ceil(gamma * out/group)); R^1 is always dense.
 *   group   output channels per group; out % group == 0 and group % 16 == 0.
 * Arithmetic: per row s = max|e| / (2^(bits-1)-1) (fp32 division), code =
 * clamp(rint(e / s)), rint = round half to even; residual e - s*code with a
 * rounded product and a rounded difference (no FMA); group score = sum of
 * squares of the residual in fp64, highest kept, ties to the lower group.
 * The result owns device memory (packed codes, scales, group indices, tile
 * schedules) until pipe_expansion_free.  *exp_out is written only on success. */
int pipe_expand(const float* W_dev, int out, int in, int bits, int K, float gamma,
                int group, void* stream, pipe_expansion** exp_out);

/* The expansion with an unstructured mask (Sec. 3.1: the pruning mask M^k of the masked
 * equation as a sparse tensor instead of row-wise zeros).  R^1 is dense; every order
 * k >= 2 keeps the ceil(gamma * out * in) entries of the residual that are largest in
 * magnitude (re-selected at every order; entries of equal magnitude go to the lower
 * row-major index), quantizes each row over its kept entries (scale = largest kept
 * magnitude / q_max, a row without kept entries has scale 0) and leaves the pruned
 * entries' residual to the next order.  Every row of every order is stored (pruned
 * entries are zero codes), so the stored size and the integer work are those of the
 * dense expansion: the mask buys accuracy per non-zero code, not speed on this
 * device.  `group` only fixes the row-block layout (same constraints as pipe_expand).
 * Arguments, ownership, errors and the arithmetic of the quantizer as pipe_expand;
 * every forward entry point accepts the result.  pipe_expansion_error_bound does not
 * (PIPE_EINVAL): a pruned entry keeps an earlier order's residual.                    */
int pipe_expand_unstructured(const float* W_dev, int out, int in, int bits, int K, float gamma,
                             int group, void* stream, pipe_expansion** exp_out);

/* The same expansion with another rounding operator (Sec. 1 and Sec. 4.5: the method is
 * agnostic to the quantization operator and combines with operators that choose the
 * rounding direction themselves).  For every order k = 1..K the builder writes, on
 * `stream`, the rows this order quantizes to rows_dev [rows, in] (compact: the kept
 * groups in ascending order) and their scales max|row| / q_max to scales_dev [rows], then
 * calls fn on the host; fn enqueues, on the same stream, work that writes one integer code
 * per element to codes_dev [rows, in] and returns 0 (anything else aborts the build with
 * PIPE_EINVAL).  The builder clamps the codes to +-q_max, gives rows of scale 0 the code 0,
 * forms R^k = s * code and the residual exactly as pipe_expand does; masks, scales and
 * layout are unchanged, so every forward entry point accepts the result.
 *   rows_dev, codes_dev  caller-owned DEVICE scratch of out*in elements; scales_dev [out]
 *   user                 passed through to fn
 * Round-to-nearest-even as fn reproduces pipe_expand bit for bit.                     */
typedef int (*pipe_rounding_fn)(void* user, int k, int rows, int in, int q_max, void* stream);
int pipe_expand_with_operator(const float* W_dev, int out, int in, int bits, int K, float gamma,
                              int group, pipe_rounding_fn fn, void* user, float* rows_dev,
                              float* scales_dev, int8_t* codes_dev, void* stream,
                              pipe_expansion** exp_out);

/* The expansion of a convolution weight for the implicit-GEMM path of pipe_forward_conv2d
 * (App. H: a convolution is the same contraction with in = C*kh*kw; Sec. 3.1 for the expansion).
 *   W_dev [out, C*kh*kw] fp32, a row flattened [C, kh, kw], read only.  C a multiple of 64.
 * Same arithmetic, masks and result as pipe_expand on the same matrix (pipe_expansion_order returns the
 * codes flattened [C, kh, kw] again); only the stored order of the in_features axis differs -- tap-major,
 * channel-minor -- so that pipe_forward_conv2d and pipe_forward_conv2d_acc read every tap's channels
 * straight from the channels-last codes of the input tensor and build no patch matrix.  The group
 * scores are fp64 sums over the rows in the stored order: a decision closer than the rounding of such
 * a sum may differ from pipe_expand's.  Only those two entry points (with the same C, kh, kw) accept
 * the result; every other forward entry point and pipe_expansion_reconstruct return PIPE_EINVAL.
 * Errors: as pipe_expand; PIPE_ESHAPE if C is not a multiple of 64 (use pipe_expand: pipe_forward_conv2d
 * then gathers the patches explicitly).                                                                */
int pipe_expand_conv2d(const float* W_dev, int out, int C, int kh, int kw, int bits, int K, float gamma,
                       int group, void* stream, pipe_expansion** exp_out);

int pipe_expansion_free(pipe_expansion* e);

/* Shape query; any output pointer may be NULL.  packed_bytes = bytes of packed
 * codes + scales + group indices the forward pass streams from HBM. */
int pipe_expansion_info(const pipe_expansion* e, int* out, int* in, int* bits, int* K,
                        int* group, float* gamma, int64_t* packed_bytes);

/* Introspection of order k (1-based): copies to HOST buffers (each may be NULL).
 *   n_groups_kept  number of groups stored at this order
 *   group_ids      [n_groups_kept] ascending
 *   scales         [n_groups_kept*group]      lambda_{R^k}, row-wise (Eq. (1))
 *   codes_unpacked [n_groups_kept*group, in]  signed codes, one per byte        */
int pipe_expansion_order(const pipe_expansion* e, int k, int* n_groups_kept,
                         int32_t* group_ids, float* scales, int8_t* codes_unpacked);

/* Expanded layer forward (App. B, Eq. (define_dre); members: Sec. 3.2).
 *   x_dev  [T, in] fp32.        T >= 0 (T == 0 is a no-op).
 *   s_x    > 0: static per-tensor activation scale; <= 0: dynamic max|x|/127.
 *          Q(x) = clamp(rint(x / s_x), -127, 127).
 *   split  HOST [M], positive, sum == K; NULL (then M is ignored) = one member.
 *   bias_dev NULL or [out]; added to the first member only (Fig. 2 caption).
 *   reduce_members  1: y_dev [T, out] = sum over members (ascending);
 *                   0: y_dev [M, T, out], one slab per member.
 * Per member: y_m = s_x * sum_{k in member, ascending} s_k[o] * float(acc_k[t,o]) (+b),
 * acc_k the exact int32 contraction.                                           */
int pipe_forward(const pipe_expansion* e, const float* x_dev, int T, float s_x,
                 const int* split, int M, const float* bias_dev, int reduce_members,
                 float* y_dev, void* stream);

/* Preparation for stream capture and for first calls that must not block: does everything
 * pipe_forward(e, x, T <= T_max, ..., split, M, ..., stream) would otherwise do on first
 * use -- builds the tile schedule of this grouping of the orders and sizes the scratch of
 * `stream` for T_max tokens -- and launches nothing.  Allocates and may synchronize: call it
 * outside capture.  Afterwards pipe_forward with the same expansion, grouping and stream and
 * any T <= T_max neither allocates nor synchronizes.  pipe_prepare_mlp and pipe_prepare_chain
 * are the same for pipe_mlp_forward and for pipe_chain_forward / pipe_chain_forward_conv
 * (arguments as in those calls; a chain over T tokens is the grid T x 1 x 1).
 * Errors: those of the forward call for the same arguments.                               */
int pipe_prepare(const pipe_expansion* e, const int* split, int M, int T_max, void* stream);
int pipe_prepare_mlp(const pipe_expansion* l1, const pipe_expansion* l2, int act, const int* split, int M,
                     int T_max, void* stream);

/* pipe_forward for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, arithmetic and results
 * (bit for bit) as pipe_forward; it calls no allocating routine and does not synchronize.
 *   - Its scratch (max|x| slot, scale, token code sums, Q(x)) is a fixed array of 8 MiB + 36 KiB
 *     in device memory that every GPU the library runs on holds until the process ends.  Limits:
 *     T <= 8192 and (T rounded up to 16, or to 64 above 128 tokens) x (in rounded up to 256)
 *     <= 8 MiB, e.g. 2048 tokens of 4096 features; beyond them PIPE_ELIMIT, nothing launched.
 *   - Above 128 tokens the tile schedule of this grouping of the orders must exist already
 *     (pipe_prepare, or any earlier pipe_forward with the same grouping above 128 tokens);
 *     otherwise PIPE_ENOTREADY, nothing launched.
 *   - All calls on one GPU share the one array, whatever their stream: calls that overlap in
 *     time on a GPU race on it.  Order them (one stream, or events).  Kernel timing
 *     (pipe_timing_enable) does not see this entry point.                                   */
int pipe_forward_noalloc(const pipe_expansion* e, const float* x_dev, int T, float s_x,
                         const int* split, int M, const float* bias_dev, int reduce_members,
                         float* y_dev, void* stream);

/* Debug twin of pipe_forward: exports the integer state for bit-exact checks.
 *   acc_dev     [K, T, out] int32, rows pruned at order k are 0 (may be NULL)
 *   qx_dev      [T, in] int8 Q(x), row-major                   (may be NULL)
 *   s_x_out_dev one float: the activation scale used           (may be NULL)  */
int pipe_forward_acc(const pipe_expansion* e, const float* x_dev, int T, float s_x,
                     int32_t* acc_dev, int8_t* qx_dev, float* s_x_out_dev, void* stream);

/* The layer with asymmetric activation codes (Sec. 4.3 makes its comparison under
 * asymmetric quantization; the affine quantizer is the usual one):  with
 * hi = max(x, 0) and lo = min(x, 0) over the tensor, a = the activation width set by
 * pipe_set_activation_bits,
 *   s = (hi - lo) / (2^a - 1),  z = clamp(rint(-lo / s), 0, 2^a - 1),
 *   Q(x) = clamp(rint(x / s) + z, 0, 2^a - 1),
 *   y[t,o] = s * sum_k s_k[o] * sum_i (Q(x)[t,i] - z) q_k[o,i]  (+ b[o]),
 * fp32 sums and IEEE divisions, rint half to even, the scale always dynamic.  The
 * contraction kernels run unchanged on the codes Q(x) - 2^(a-1); the term that does
 * not depend on the token, s (2^(a-1) - z) sum_k s_k[o] sum_i q_k[o,i], is added
 * with the bias (the sums of the codes are built on the first call: it allocates and
 * synchronizes once per expansion).  Members given by split are summed.
 *   x_dev [T, in], bias_dev NULL or [out], y_dev [T, out]: DEVICE, caller-owned.
 * PIPE_ESHAPE if (2^a - 1) * q_max * in does not fit the 32-bit accumulator.      */
int pipe_forward_asymmetric(const pipe_expansion* e, const float* x_dev, int T, const int* split, int M,
                            const float* bias_dev, float* y_dev, void* stream);

/* The convolution layer with the same asymmetric codes (range over the whole input
 * tensor): taps outside the image hold the real value 0, i.e. the code z.  Geometry,
 * layouts and the [N*Ho*Wo, out] channels-last output as pipe_forward_conv2d; members
 * summed; errors as pipe_forward_conv2d and pipe_forward_asymmetric.                 */
int pipe_forward_conv2d_asymmetric(const pipe_expansion* e, const float* x_dev, int N, int C, int H, int W,
                                   int kh, int kw, int stride, int pad, int nhwc, const int* split, int M,
                                   const float* bias_dev, float* y_dev, void* stream);

/* Debug export of the same call: the exact accumulators acc_dev [K, T, out]
 * (sum_i (Q(x) - z) q_k; pruned rows 0), optionally the unsigned codes qx_dev [T, in],
 * the scale and the zero point (DEVICE; NULL to skip).  Synchronizes.               */
int pipe_forward_acc_asymmetric(const pipe_expansion* e, const float* x_dev, int T, int32_t* acc_dev,
                                uint8_t* qx_dev, float* s_x_out_dev, int32_t* z_out_dev, void* stream);

/* Expanded convolution as a GEMM over output pixels (App. H treats conv and FC
 * alike).  The expansion was built from W [out, C*kh*kw], a row flattened as
 * [C, kh, kw]: by pipe_expand (the patches of Q(x) are gathered into a matrix first) or by
 * pipe_expand_conv2d (implicit GEMM: no patch matrix, three launches).  x_dev is [N,C,H,W] (nhwc == 0) or [N,H,W,C] (nhwc != 0), zero
 * padded by `pad`.  Tokens are output pixels ordered (n, ho, wo):
 * y_dev is [N*Ho*Wo, out] (channels last), or [M, N*Ho*Wo, out].
 * Remaining arguments as pipe_forward.                                        */
int pipe_forward_conv2d(const pipe_expansion* e, const float* x_dev, int N, int C, int H,
                        int W, int kh, int kw, int stride, int pad, int nhwc, float s_x,
                        const int* split, int M, const float* bias_dev,
                        int reduce_members, float* y_dev, void* stream);

/* Debug twin of pipe_forward_conv2d (App. B, Eq. (define_dre) on the contraction of App. H):
 * exports the integer state of the convolution layer for bit-exact checks.
 *   acc_dev     [K, N*Ho*Wo, out] int32: acc_k[t,o] = sum over (c, r, s) of Q(x)[n, c, ho*stride+r-pad,
 *               wo*stride+s-pad] * q_k[o, (c, r, s)], taps outside the image contributing 0; rows pruned
 *               at order k are 0.  Required (PIPE_EINVAL if NULL).
 *   qx_dev      int8 Q(x) in the layout of x_dev ([N,C,H,W] or [N,H,W,C])        (may be NULL)
 *   s_x_out_dev one float: the activation scale used                           (may be NULL)
 * Geometry arguments, s_x and errors as pipe_forward_conv2d.  All pointers DEVICE, caller-owned. */
int pipe_forward_conv2d_acc(const pipe_expansion* e, const float* x_dev, int N, int C, int H, int W,
                            int kh, int kw, int stride, int pad, int nhwc, float s_x, int32_t* acc_dev,
                            int8_t* qx_dev, float* s_x_out_dev, void* stream);

/* Expanded depthwise convolution (App. H: a convolution whose filters see one input
 * channel each; the separable blocks of MobileNet / EfficientNet).  The expansion was
 * built from W [C, kh*kw] (row c = the filter of channel c, flattened [kh, kw]; kh*kw
 * <= 49).  x_dev and y_dev as in pipe_forward_conv2d: y_dev is [N*Ho*Wo, C] (channels
 * last) or [M, N*Ho*Wo, C].  Same quantizer, scales, member ranges and summation order as
 * the dense layers; runs on the vector ALUs (kh*kw multiply-adds per output and order is
 * no contraction for the matrix cores).  The first call on an expansion builds a dense
 * copy of its codes (allocates, synchronizes).                                       */
int pipe_forward_depthwise2d(const pipe_expansion* e, const float* x_dev, int N, int C, int H,
                             int W, int kh, int kw, int stride, int pad, int nhwc, float s_x,
                             const int* split, int M, const float* bias_dev,
                             int reduce_members, float* y_dev, void* stream);

/* Two expanded layers with an activation between, run as an ensemble of M
 * members (Sec. 3.2; App. B "Ensemble of more Layers"): member m uses only its
 * own orders in both layers, quantizes its own hidden activation with its own
 * dynamic scale, carries the biases only if it is the first member, and the
 * members' outputs are summed after the second layer.
 *   act = PIPE_ACT_GELU:       l1 [H, in],  h = GELU_erf(l1(x))
 *   act = PIPE_ACT_SILU_GATED: l1 [2H, in] (gate rows, then up rows),
 *                              h = SiLU(gate) * up
 *   l2 [out, H]; both layers have the same K.  y_dev [T, out].
 *   h_dev  NULL, or [M, T, H] fp32 to receive the hidden activations.          */
int pipe_mlp_forward(const pipe_expansion* l1, const pipe_expansion* l2, int act,
                     const float* x_dev, int T, float s_x, const int* split, int M,
                     const float* bias1_dev, const float* bias2_dev, float* h_dev,
                     float* y_dev, void* stream);

/* pipe_mlp_forward with static activation ranges throughout (Sec. 4: activations quantized with
 * ranges fixed ahead of time, as in DFQ): s_x > 0 is the given scale of the input and s_h_host
 * (HOST, [M], positive, read during the call) the given scales of the members' hidden
 * activations, used instead of max|h_m| / q_max.  No maximum is reduced or exchanged anywhere
 * in the call.  Everything else as pipe_mlp_forward; PIPE_EINVAL if a scale is missing or not
 * positive.                                                                               */
int pipe_mlp_forward_given_scales(const pipe_expansion* l1, const pipe_expansion* l2, int act,
                                  const float* x_dev, int T, float s_x, const float* s_h_host,
                                  const int* split, int M, const float* bias1_dev,
                                  const float* bias2_dev, float* h_dev, float* y_dev, void* stream);

/* pipe_mlp_forward with asymmetric activation codes (Sec. 4.3; the affine quantizer of
 * pipe_forward_asymmetric) in front of both layers: the input is quantized over its own range
 * [min(x,0), max(x,0)], every member's hidden activation over that tensor's own range with its
 * own scale and integer zero point (GELU and SiLU(gate)*up take both signs).  Ranges are always
 * dynamic.  Arguments, member semantics, h_dev and errors as pipe_mlp_forward; PIPE_ESHAPE when
 * (2^a - 1) * q_max * in_features does not fit 31 bits.  The first call on an expansion builds
 * the sums of its codes (allocates, synchronizes: PIPE_ENOTREADY under capture).            */
int pipe_mlp_forward_asymmetric(const pipe_expansion* l1, const pipe_expansion* l2, int act,
                                const float* x_dev, int T, const int* split, int M,
                                const float* bias1_dev, const float* bias2_dev, float* h_dev,
                                float* y_dev, void* stream);

/* One layer of a member chain (pipe_chain_forward, pipe_chain_forward_conv).     */
typedef struct pipe_chain_layer {
  const pipe_expansion* e; /* [out_l, in_l]; in_l = width of the tensor entering it,
                              or C_l*kh*kw (a row flattened as [C, kh, kw], as for
                              pipe_forward_conv2d) for a convolution                 */
  const float* bias_dev;   /* DEVICE, NULL or [out_l]; first member only              */
  int act;                 /* PIPE_ACT_NONE, PIPE_ACT_RELU or PIPE_ACT_GELU (erf)     */
  int skip_from;           /* -1: no skip; j in 0..l: add the tensor that ENTERED
                              layer j (0 = the network input), width out_l          */
  int skip_pre_act;        /* 1: a = act(z + r) (residual block); 0: a = act(z) + r   */
  int kh, kw;              /* 0, 0: fully connected, applied at every grid position;
                              else the kernel size of a convolution over the grid    */
  int stride, pad;         /* of the convolution (stride >= 1, pad >= 0); ignored when
                              kh = kw = 0                                            */
  const float* s_in;       /* HOST, NULL or [M] positive: given (static) scales of the
                              members' tensors that ENTER this layer (Sec. 4: activation
                              ranges fixed ahead of time, as in DFQ), read during the call;
                              NULL: each member's max|tensor| / q_max.  Ignored for layer 0,
                              whose shared input takes the call's s_x                    */
} pipe_chain_layer;

/* An L-layer feed-forward network run as M independent member chains that are
 * summed after the last layer (Sec. 3.2, Fig. 2; App. B "Ensemble of more Layers
 * DNNs", App. D "Ensembling with more Layers").  Member m is the whole
 * architecture with, in every layer, only the orders of its own cluster; it
 * quantizes each tensor entering a layer with its own dynamic per-tensor scale
 * (s_x applies to the network input, which all members share); biases belong to
 * the first member.  A skip is member-wise -- member m adds its own copy of the
 * earlier tensor -- except a skip from the network input, which is not split
 * over the members and enters the sum once, through the first member.
 *   layers   HOST [L], L >= 1, same K in every layer; the last layer's act must be
 *            PIPE_ACT_NONE (the members are summed behind it)
 *   acts_dev HOST [L-1] of DEVICE pointers, or NULL; entry l NULL or [M, T, out_l]
 *            fp32 to receive the tensor leaving layer l of every member
 *   y_dev    [T, out_{L-1}] = sum over members, ascending
 * All members of a layer run in one launch.  Errors: PIPE_EINVAL (NULL, act or
 * skip out of range), PIPE_ESHAPE (widths do not chain, skip width mismatch),
 * PIPE_ESPLIT (layers differ in K, bad split), PIPE_ENOMEM, PIPE_EDEVICE.       */
int pipe_chain_forward(const pipe_chain_layer* layers, int L, const float* x_dev, int T,
                       float s_x, const int* split, int M, float* const* acts_dev,
                       float* y_dev, void* stream);

/* pipe_chain_forward with asymmetric activation codes (Sec. 4.3 makes its comparison under
 * asymmetric quantization; the affine quantizer is the one of pipe_forward_asymmetric) in front
 * of EVERY layer: the network input is quantized over its range [min(x,0), max(x,0)], and
 * every member quantizes each of its own hidden tensors over that tensor's own range, with its
 * own scale and integer zero point (after a ReLU the whole code range covers [0, max]: half the
 * step of the symmetric codes).  Everything else -- members, biases, skips, the sum behind the
 * last layer, acts_dev, y_dev -- as pipe_chain_forward; ranges are always dynamic (no s_x).
 * Fully-connected layers only (kh = kw = 0, else PIPE_EINVAL).  The first call on an expansion
 * builds the sums of its codes (allocates, synchronizes: not under capture, PIPE_ENOTREADY).
 * Further errors: PIPE_ESHAPE when (2^a - 1) * q_max * in_features does not fit 31 bits.     */
int pipe_chain_forward_asymmetric(const pipe_chain_layer* layers, int L, const float* x_dev, int T,
                                  const int* split, int M, float* const* acts_dev, float* y_dev,
                                  void* stream);

/* pipe_chain_forward_conv (below) with the asymmetric codes of pipe_chain_forward_asymmetric in
 * front of every layer, convolutions included: a member quantizes every element of its
 * channels-last input once, over that tensor's range, and a tap outside the image holds the code
 * of the real value 0 (the zero point), so the padding contributes nothing, as in
 * pipe_forward_conv2d_asymmetric.  Arguments, layouts and errors as pipe_chain_forward_conv
 * (no s_x: ranges are dynamic) and pipe_chain_forward_asymmetric.                            */
int pipe_chain_forward_conv_asymmetric(const pipe_chain_layer* layers, int L, const float* x_dev,
                                       int N, int H, int W, const int* split, int M,
                                       float* const* acts_dev, float* y_dev, void* stream);

/* The same member chains over convolution layers (Fig. 2 draws the expansion of a
 * convolutional network; Sec. 4 evaluates ResNets and MobileNets).  Every tensor is
 * channels-last: tokens are the positions (n, h, w) of an N x H_l x W_l grid in that
 * order, x_dev is [N, H, W, C_0].  A layer with kh, kw > 0 is a convolution (the
 * contraction of pipe_forward_conv2d over the member's quantized tensor) and maps the
 * grid to H_{l+1} = (H_l + 2 pad - kh) / stride + 1, likewise W; a layer with
 * kh = kw = 0 keeps the grid (a 1x1 convolution, or a classifier when the grid is
 * N x 1 x 1).  A skip needs equal grids and channel counts at both ends.
 *   acts_dev entry l: NULL or [M, N*H_{l+1}*W_{l+1}, out_l];  y_dev [N*H_L*W_L, out_{L-1}]
 * pipe_chain_forward is this call on a T x 1 x 1 grid and rejects convolution layers
 * (PIPE_EINVAL).  Further errors: PIPE_ESHAPE (kernel larger than the padded grid,
 * in_l not a multiple of kh*kw, grids of a skip differ).                            */
int pipe_chain_forward_conv(const pipe_chain_layer* layers, int L, const float* x_dev,
                            int N, int H, int W, float s_x, const int* split, int M,
                            float* const* acts_dev, float* y_dev, void* stream);

int pipe_prepare_chain(const pipe_chain_layer* layers, int L, int N, int H, int W, const int* split, int M,
                       void* stream);

/* Bit-width a of the activation quantizer of every forward entry point from now on
 * (Sec. 4 compares W4/A4, W4/A6, W8/A8): Q(x) = clamp(rint(x / s_x), +-(2^(a-1)-1)),
 * dynamic s_x = max|x| / (2^(a-1)-1).  Default 8.  Process-wide; the codes still travel as
 * bytes and feed the int8 MFMA.  Synchronous (copies one word to the device); do not call
 * it while forward calls are in flight.  Returns PIPE_EINVAL outside 2..8.              */
int pipe_set_activation_bits(int bits);

/* ---- Data-free error diagnostics (App. C, Theorems 1 and 2; Lemmas of App. B) ----
 * None of these is on the forward path.
 *
 * pipe_spectral_norm: s = largest singular value of W (the theorems' s_l), by `iters`
 * steps of the power iteration on W^T W: v <- W^T (W v) / ||W^T (W v)||, from the fixed
 * unit vector v0[i] = +-1/sqrt(in) (sign = bit 15 of i * 2654435761 mod 2^32); returns
 * ||W v|| for the last v, a lower bound that converges to s.  fp64 accumulation.
 *   W_dev [out, in] fp32 row-major, DEVICE.  sigma_host: HOST.  Synchronizes the stream.
 *
 * pipe_expansion_reconstruct: W_out_dev [out, in] fp32 = sum over orders k <= upto of
 * R^k = s_k * codes_k (Eq. 3; pruned rows contribute nothing), 1 <= upto <= K.
 *
 * pipe_expansion_error_bound: element-wise bounds on |W - sum_k R^k| from the stored
 * scales alone.  u_lemma = (1/q_max)^(K-1) * max_rows(s_1) / 2 (Lemma "dre" with lambda
 * read as the first-order scale; valid for rows stored at every order).  u_stored =
 * max over rows of (scale of the row's LAST stored order) / 2: valid for sparse
 * expansions too (the provable counterpart of Lemma "slim", whose printed numerator the
 * paper does not define).  HOST outputs, either may be NULL.  Synchronizes the device.
 *
 * pipe_error_bound_U: U = prod_{l=1..L} ( sum_{i<=l} s_i u_i + 1 ) - 1 as printed in
 * Theorem 1 (U_res with u_lemma, U_sparse with u_stored).  HOST arrays; pure arithmetic.
 *
 * pipe_expansion_order_norms: norms_host[k-1] = ||R^(k)||, k = 1..K, the spectral norm of
 * each term s_k * codes_k of the expansion (Eq. 3) by the power iteration of
 * pipe_spectral_norm on the order's stored rows (pruned rows are zero rows and change no
 * singular value); 0 for an order with no stored row.  HOST [K] doubles.  Synchronizes.
 *
 * pipe_error_bound_U_ens (App. C, Theorem "ensemble"): for L layers, K orders and the
 * grouping split [K_1..K_M] (NULL = one predictor),
 *   U_ens = ( sum_{k in cluster 1} norms[L-1][k] / 2^(L-1) )
 *           * ( 1 + sum_{m=2..M} prod_{l=0..L-2} sum_{k in cluster m} norms[l][k] lam[l][k] ).
 * The printed inner sum runs over k = K_m..K_{m+1} and writes R_L inside the product over
 * l: read as "the orders of cluster m" and "layer l's weights".  norms HOST [L][K]
 * (pipe_expansion_order_norms of each layer); lam HOST [L-1][K] stands for the printed
 * lambda of the quantized tensor entering the next layer, NULL = all 1.  Pure arithmetic.
 * Errors: PIPE_EINVAL, PIPE_ESPLIT (split does not sum to K).
 *
 * pipe_first_predictor_size (App. A, the paragraph on K_1; App. C closing remark): the
 * smallest K_1 for which the two-predictor ensemble [K_1, K-K_1] has
 * U_ens <= ratio * logit_norm (logit_norm: the caller's estimate of E||f^(K)||, e.g. from
 * the last batch-norm's statistics); K when no split qualifies.  Pure arithmetic.      */
int pipe_spectral_norm(const float* W_dev, int out, int in, int iters, float* sigma_host,
                       void* stream);
int pipe_expansion_reconstruct(const pipe_expansion* e, int upto, float* W_out_dev,
                               void* stream);
int pipe_expansion_error_bound(const pipe_expansion* e, double* u_lemma, double* u_stored);
int pipe_error_bound_U(const double* s, const double* u, int L, double* U_out);
int pipe_expansion_order_norms(const pipe_expansion* e, int iters, double* norms_host,
                               void* stream);
int pipe_error_bound_U_ens(const double* norms, const double* lam, int L, int K,
                           const int* split, int M, double* U_out);
int pipe_first_predictor_size(const double* norms, const double* lam, int L, int K,
                              double logit_norm, double ratio, int* K1_out);

/* Kernel selection for pipe_forward / pipe_mlp_forward (tuning and tests):
 * 0 = automatic by token count, 1 = tiled MFMA kernel, 2 = weight-streaming
 * small-batch kernel.  Returns PIPE_EINVAL for other values.                    */
int pipe_set_kernel(int which);

/* Token-tile height of the tiled MFMA kernel (tuning and tests): 0 = automatic
 * (64 tokens per workgroup when that still gives every CU several tiles, else 32
 * or 16), or 16, 32, 64.  Results do not depend on the setting.  Returns
 * PIPE_EINVAL for other values.                                                   */
int pipe_set_token_tile(int tokens);

/* Split of the weight-streaming kernel's bins along in_features (tuning and tests).
 * A bin (up to 4 stored row blocks -- 8, 12 or 16 for more than 4 orders -- holding every order of a few output row blocks)
 * is normally streamed by one workgroup; layers with few output channels and a long
 * in_features are split over several workgroups per bin, whose exact integer
 * partial sums meet in a workspace owned by the expansion (so two forward calls on
 * the same expansion must not overlap in time).  0 = automatic (default), n >= 1 =
 * that many workgroups per bin (capped by the number of packed k tiles).  Results
 * do not depend on the setting.  Returns PIPE_EINVAL outside 0..8.                */
int pipe_set_stream_split(int workgroups_per_bin);

/* A single token (pipe_forward, and layer 1 of pipe_mlp_forward, on a layer of at
 * most 8192 input features, a multiple of 4, 16-byte aligned input): by default the weight-streaming kernel quantizes the
 * input itself -- every workgroup reduces max|x| and rounds the few KiB of activations
 * with the quantizer's own arithmetic -- so the step is one launch instead of two.
 * (From two tokens on the repeated work costs more than the launch it saves.)
 * An output buffer that overlaps the input keeps the two-launch path.  0 switches
 * this off (tuning and tests), 1 on (default).  Results do not depend on the
 * setting.  Returns PIPE_EINVAL for other values.                                    */
int pipe_set_decode_fusion(int on);

/* Decode-sized batches (at most 16 tokens) through pipe_chain_forward and pipe_mlp_forward: the
 * whole chain of layers can run as ONE resident launch (one workgroup per compute unit walks the
 * layers; the packed codes of the next layer stream from HBM while the current layer's results are
 * exchanged between the workgroups) instead of two launches per layer.  Conditions: fully-connected
 * layers only, at most 4 orders and at most 2 members, every layer stored at the same code width, at most
 * 16 layers, in_features of the first layer a multiple of 4 and a 16-byte aligned input; otherwise
 * the calls take the per-layer launches.  `on`: 0 never, 2 whenever the conditions hold, 1 (default)
 * where it measured faster: chains of three or more layers at any batch, shorter chains and the MLP
 * call above 8 tokens, or at any batch when every activation scale is given (the exchange between
 * workgroups costs about 8 us per layer, half of it for the maxima that given scales make
 * unnecessary; two launches per layer cost about 10-17 us).  Results do not depend on the setting (the fp32 arithmetic and its
 * order are those of the per-layer kernels).  Returns PIPE_EINVAL for other values.
 * The resident launch needs every workgroup of its grid on the chip at once; its waits for other
 * workgroups are bounded (pipe_set_resident_spin_limit polls, 0 = the default of 2^19, about a second):
 * a workgroup whose wait runs out records it and runs to its end without waiting again, so the launch
 * always ends, with wrong results.  pipe_resident_status synchronizes `stream` and writes to *status_out
 * (HOST) 0, or a non-zero value if a launch on that stream's scratch ran into the limit since the last
 * query (then clears it).  Two resident launches in flight at once on one GPU (two streams) can starve
 * each other into that limit: order them.                                                          */
int pipe_set_decode_resident(int on);
int pipe_set_resident_spin_limit(int polls);
int pipe_resident_status(void* stream, int* status_out);
/* Profiling of the resident launch: with trace_dev != NULL (DEVICE, [workgroups][layers][8] 64-bit
 * words, workgroups = compute units of the chip) every later resident launch records, per workgroup and
 * layer, the time (100 MHz counter) at which 0 the exchange before the layer begins, 1 the scales are
 * known, 2 its codes are stored, 3 all workgroups' codes are visible, 4 its last unit's outputs are
 * written, 5 the integer tiles of its first unit are complete, 6 that unit's outputs are computed, 7 its
 * first worker wave has multiplied its last round.  NULL switches it off (default).  Process-wide.  */
int pipe_resident_trace(unsigned long long* trace_dev);

/* Kernel timing for benchmarks.  While enabled, every forward call brackets its
 * contraction kernel (the dominant kernel of the path) with a pair of HIP events
 * recorded on the call's stream.  pipe_timing_read waits for the recorded events,
 * returns the summed elapsed time and the number of bracketed launches since the
 * last read, and resets both.  At most 4096 launches are kept between reads.   */
int pipe_timing_enable(int on);
int pipe_timing_read(double* total_ms, int* launches);

/* Diagnostics for reports: reference rates measured on the chip the library runs on.
 * pipe_mfma_probe runs an MFMA-only kernel (back-to-back independent
 * v_mfma_i32_16x16x64_i8 on registers, no memory traffic in the loop) for `iters`
 * rounds of 16 instructions per wave and writes the int8 rate it sustained, in TOP/s,
 * to *tops_out (HOST).  `operands`: 0 = constant bytes, 1 = ternary offset codes
 * against random int8 (what a ternary layer feeds the pipe), 2 = random int8 against
 * random int8; the chip's clock under load depends on it.  10, 11, 12 = the same
 * operand kinds on v_mfma_i32_32x32x32_i8 (eight instructions per round, the same
 * multiply-adds), the instruction with twice the work per operand byte.
 * pipe_hbm_probe reads `bytes` (>= 1 MiB, rounded down to 128 KiB) of freshly
 * allocated device memory with the access pattern of the weight-streaming kernel and
 * writes the bandwidth, in GB/s, to *gbps_out (HOST); it allocates and frees `bytes`.
 * Both synchronize the stream.                                                     */
int pipe_mfma_probe(int iters, int operands, double* tops_out, void* stream);
int pipe_hbm_probe(int64_t bytes, double* gbps_out, void* stream);

const char* pipe_strerror(int code);
/* Text of the last HIP error seen by this thread ("" if none). */
const char* pipe_last_device_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PIPE_H_ */
