"""CPU checker for the residual-expanded quantized layer (PIPE, arXiv 2311.15806).

TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, step-by-step statement
of what the HIP path must compute.  Only the tests, the smoke check and the
benchmark's CPU-baseline leg may import it; the product never does, and this
file imports nothing from the product.  It is written in numpy, in the paper's
order and notation, with no blocking, fusion or packing.

Arithmetic (fixed, because the method is an encoding whose integer codes depend
on it): weights, scales and residuals are IEEE fp32 with round-to-nearest-even
and no fused multiply-add; group scores are fp64; the contraction is exact
integer arithmetic; the de-quantising epilogue is fp32 with an fp64 twin.

Passages followed
  * quantizer Q and de-quantizer Q^-1 ............ Sec. 3, Eq. (1)
  * residual expansion R^1..R^K .................. Sec. 3.1, Eq. (2), (3)
  * structured mask M^k, sparsity ratio gamma .... Sec. 3.1, masked Eq. after (4)
  * unstructured mask M^k (a sparse tensor) ...... Sec. 3.1, same passage
  * asymmetric activation codes .................. Sec. 4.3 (the comparison of Table
                                                   compar_sota is made under asymmetric quantization)
  * expanded-layer forward ....................... App. B, Eq. (define_dre)
  * ensemble members, bias in predictor 1 ........ Sec. 3.2, Fig. 2 caption,
                                                   App. B "Ensemble of more Layers"
  * L-layer member chains with skips ............. App. B / App. D "more Layers", Fig. 2
  * error diagnostics (spectral norms, U) ........ App. C, Theorems 1-2; Lemmas of App. B
  * per-order norms, U_ens, predictor size ....... App. C, Theorem "ensemble"; App. A on K_1
  * operation head-count ......................... App. H

Readings taken where the paper is silent (each is listed in the design notes):
scale = row absmax / (2^(b-1)-1) and codes clamped to +-(2^(b-1)-1); ties round
to even; an all-zero row has scale 0 and codes 0; R^1 is dense and orders k>=2
keep the ceil(gamma*n_groups) groups of `group` consecutive output channels with
the largest residual energy (sum of squares, fp64), re-selected at every order,
ties to the lower group index; an unstructured mask keeps the ceil(gamma*O*I)
entries of the residual that are largest in magnitude, re-selected at every
order k>=2, ties to the lower flat index, and a row's scale is the largest kept
magnitude over q_max; activations are per-tensor symmetric a-bit codes
(a = 8 unless stated) with a static scale if given, else absmax/(2^(a-1)-1); asymmetric activation codes are
the unsigned a-bit grid over [min(x, 0), max(x, 0)] with an integer zero point; a member owns a contiguous range of
orders in every layer and its own activation scale; in a chain a skip connection
is member-wise, except one that reads the network input, which only the first
member adds.

Pins: every function here is checked in tests/test_oracle_pins.py against facts
that do not come from this file (hand-worked example, exhaustive nearest-code
search, the Lemma's bound, brute-force mask enumeration, torch integer matmul
and conv2d, closed forms).  Not pinned by the paper (this build's reading only):
the group-selection criterion, the entry-selection criterion of an unstructured
mask, the member-wise treatment of gated MLPs, the
first-member-only skip from the network input, and the reading of U_ens' index
ranges with the predictor-size procedure built on it (parity unpinned: only
hand-evaluated instances of this reading; the per-order norms are pinned by SVD).
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

f32 = np.float32


# ----------------------------------------------------------------------------
# Sec. 3, Eq. (1): Q(W) = round(W / s), Q^-1(q) = s * q   (per output channel)
# ----------------------------------------------------------------------------
def q_max(bits: int) -> int:
    """Largest code magnitude 2^(b-1)-1 (the Lemma's constant): 127, 31, 7, 3, 1 for
    b = 8, 6, 4, 3, 2 (ternary)."""
    if not 2 <= int(bits) <= 8:
        raise ValueError("bits must lie in 2..8")
    return 2 ** (int(bits) - 1) - 1


def quantize_rows(E: np.ndarray, bits: int, operator=None, k: int = 1):
    """Row-wise symmetric quantizer.  E fp32 [R, I] -> (codes int8 [R, I], s fp32 [R]).

    s[o] = max_i |E[o,i]| / q_max (fp32 division); q = clamp(rint(E / s), +-q_max),
    rint rounds half to even.  A row whose scale is 0 gets codes 0.

    The method does not depend on how a value is rounded onto the grid (Sec. 1 and Sec. 4.5:
    the expansion combines with any quantization operator): `operator`, if given, replaces the
    rint step.  It is called as operator(k, E, s, q_max) and returns integer codes [R, I]; they
    are clamped to +-q_max and rows of scale 0 get codes 0, as above."""
    E = np.asarray(E, dtype=f32)
    qm = f32(q_max(bits))
    amax = np.max(np.abs(E), axis=1) if E.shape[1] else np.zeros(E.shape[0], f32)
    s = (amax / qm).astype(f32)
    live = s > 0
    if operator is None:
        div = np.where(live, s, f32(1.0)).astype(f32)
        q = np.rint(E / div[:, None])
    else:
        q = np.asarray(operator(k, E, s, int(qm)), dtype=np.float64)
        if q.shape != E.shape:
            raise ValueError("the operator returns one code per element")
    q = np.clip(q, -qm, qm)
    q[~live, :] = 0
    return q.astype(np.int8), s


# ----------------------------------------------------------------------------
# Sec. 3.1: structured mask M^k over groups of consecutive output channels
# ----------------------------------------------------------------------------
def n_keep(gamma: float, n_groups: int) -> int:
    """Number of groups kept at an order k>=2: ceil(gamma * n_groups).

    gamma is first rounded to fp32 (the boundary passes a C float); the factor
    (1 - 1e-6) keeps an exactly integral product from being pushed up by that
    rounding."""
    g = float(f32(gamma))
    if not (0.0 < g <= 1.0):
        raise ValueError("gamma must lie in (0, 1]")
    return max(1, min(n_groups, math.ceil(g * n_groups * (1.0 - 1e-6))))


def group_scores(E: np.ndarray, group: int) -> np.ndarray:
    """Residual energy per group: sum over the group's rows and all columns of
    E^2, accumulated in fp64 (each square of an fp32 value is exact in fp64)."""
    E64 = np.asarray(E, dtype=np.float64)
    row = np.sum(E64 * E64, axis=1)
    return row.reshape(-1, group).sum(axis=1)


def select_groups(scores: np.ndarray, keep: int) -> np.ndarray:
    """Indices (ascending) of the `keep` highest scores; ties go to the lower index."""
    n = scores.shape[0]
    order = sorted(range(n), key=lambda g: (-float(scores[g]), g))
    return np.array(sorted(order[:keep]), dtype=np.int32)


def selection_gap(scores: np.ndarray, keep: int) -> float:
    """Relative gap between the last kept and the first dropped score (inf if none
    is dropped).  Input generators use it to reject near-ties, where the order of
    an fp64 summation could decide the mask."""
    n = scores.shape[0]
    if keep >= n:
        return math.inf
    srt = np.sort(scores)[::-1]
    a, b = float(srt[keep - 1]), float(srt[keep])
    return (a - b) / a if a > 0 else 0.0


def select_entries(E: np.ndarray, keep: int) -> np.ndarray:
    """Unstructured mask (Sec. 3.1: M^k a sparse tensor): boolean [O, I], True on the `keep`
    entries of E largest in magnitude; entries of equal magnitude go to the lower flat
    (row-major) index."""
    a = np.abs(np.asarray(E, dtype=f32)).ravel()
    n = a.shape[0]
    M = np.zeros(n, dtype=bool)
    if keep >= n:
        M[:] = True
        return M.reshape(E.shape)
    thr = np.partition(a, n - keep)[n - keep]          # the keep-th largest magnitude
    M[a > thr] = True
    ties = np.flatnonzero(a == thr)
    M[ties[:keep - int(M.sum())]] = True
    return M.reshape(E.shape)


def quantize_rows_masked(E: np.ndarray, M: np.ndarray, bits: int):
    """quantize_rows over the entries M keeps: s[o] = max_{i: M[o,i]} |E[o,i]| / q_max, codes
    clamp(rint(E / s)) on kept entries and 0 elsewhere; a row without a kept entry (or whose
    kept entries are all zero) has scale 0 and codes 0."""
    E = np.asarray(E, dtype=f32)
    qm = f32(q_max(bits))
    amax = np.max(np.where(M, np.abs(E), f32(0)), axis=1).astype(f32)
    s = (amax / qm).astype(f32)
    live = s > 0
    div = np.where(live, s, f32(1.0)).astype(f32)
    q = np.clip(np.rint(E / div[:, None]), -qm, qm)
    q[~live, :] = 0
    q[~M] = 0
    return q.astype(np.int8), s


# ----------------------------------------------------------------------------
# Sec. 3.1, Eq. (2)-(3) and the masked form: R^k = M^k Q^-1(Q(W - sum_{j<k} R^j))
# ----------------------------------------------------------------------------
@dataclass
class Order:
    """One term R^k of the expansion, stored compactly over its kept groups."""
    group_ids: np.ndarray    # int32 [n_kept], ascending
    scales: np.ndarray       # fp32  [n_kept*group]   (lambda_{R^k}, row-wise)
    codes: np.ndarray        # int8  [n_kept*group, I]


@dataclass
class Expansion:
    out_features: int
    in_features: int
    bits: int
    K: int
    gamma: float
    group: int
    orders: List[Order]

    def rows(self, k: int) -> np.ndarray:
        """Output-channel index of every stored row of order k (1-based k)."""
        o = self.orders[k - 1]
        return (o.group_ids[:, None].astype(np.int64) * self.group
                + np.arange(self.group)[None, :]).reshape(-1)

    def dense_codes(self, k: int) -> np.ndarray:
        """int8 [O, I]; pruned rows are 0."""
        q = np.zeros((self.out_features, self.in_features), dtype=np.int8)
        q[self.rows(k)] = self.orders[k - 1].codes
        return q

    def dense_scales(self, k: int) -> np.ndarray:
        """fp32 [O]; pruned rows are 0."""
        s = np.zeros(self.out_features, dtype=f32)
        s[self.rows(k)] = self.orders[k - 1].scales
        return s

    def reconstruct(self, upto: Optional[int] = None) -> np.ndarray:
        """sum_{k<=upto} R^k in fp64 (for error measurements only)."""
        upto = self.K if upto is None else upto
        R = np.zeros((self.out_features, self.in_features), dtype=np.float64)
        for k in range(1, upto + 1):
            R += self.dense_scales(k).astype(np.float64)[:, None] * self.dense_codes(k)
        return R


def expand(W: np.ndarray, bits: int, K: int, gamma: float, group: int,
           residuals: Optional[list] = None, gaps: Optional[list] = None, operator=None,
           mask: str = "structured", masks: Optional[list] = None) -> Expansion:
    """Residual expansion of W [O, I] to order K.

    E_1 = W.  For k = 1..K: (k>=2 and gamma<1: keep the top n_keep groups of E_k
    by energy, else all groups); on kept rows s_k, q_k = quantize_rows(E_k) and
    E_{k+1} = E_k - s_k*q_k (fp32 multiply, then fp32 subtract); pruned rows pass
    their residual on unchanged.  If `residuals` is a list, E_2..E_{K+1} are
    appended to it (copies); if `gaps` is a list, the selection_gap of every mask
    that was chosen is appended to it.  `operator` replaces round-to-nearest in every
    order (see quantize_rows).

    mask = "unstructured": orders k >= 2 keep the n_keep(gamma, O*I) entries of E_k largest in
    magnitude instead of whole groups (select_entries); every row is stored, pruned entries have
    code 0 and pass their residual on unchanged.  If `masks` is a list, the boolean mask of every
    order k >= 2 is appended to it."""
    W = np.asarray(W, dtype=f32)
    if W.ndim != 2:
        raise ValueError("W must be [out, in]")
    O, I = W.shape
    if K < 1 or group < 1 or O % group:
        raise ValueError("need K >= 1 and out % group == 0")
    q_max(bits)
    n_g = O // group
    if mask not in ("structured", "unstructured"):
        raise ValueError("mask is 'structured' or 'unstructured'")
    unstructured = mask == "unstructured"
    if unstructured and operator is not None:
        raise ValueError("the operator plug-in goes with structured masks")
    keep = n_g if unstructured else n_keep(gamma, n_g)
    keep_entries = n_keep(gamma, O * I)
    E = W.copy()
    orders: List[Order] = []
    for k in range(1, K + 1):
        if unstructured and k >= 2 and keep_entries < O * I:
            Mk = select_entries(E, keep_entries)
            if masks is not None:
                masks.append(Mk.copy())
            q, s = quantize_rows_masked(E, Mk, bits)
            Rk = (s[:, None] * q.astype(f32)).astype(f32)
            E = np.where(Mk, (E - Rk).astype(f32), E)          # pruned entries pass on unchanged
            orders.append(Order(np.arange(n_g, dtype=np.int32), s, q))
            if residuals is not None:
                residuals.append(E.copy())
            continue
        if k == 1 or keep == n_g:
            gids = np.arange(n_g, dtype=np.int32)
        else:
            scores = group_scores(E, group)
            gids = select_groups(scores, keep)
            if gaps is not None:
                gaps.append(selection_gap(scores, keep))
        rows = (gids[:, None].astype(np.int64) * group + np.arange(group)[None, :]).reshape(-1)
        q, s = quantize_rows(E[rows], bits, operator, k)
        Rk = (s[:, None] * q.astype(f32)).astype(f32)      # Q^-1(Q(.)), one rounding
        E[rows] = (E[rows] - Rk).astype(f32)               # second rounding, no FMA
        orders.append(Order(gids, s, q))
        if residuals is not None:
            residuals.append(E.copy())
    return Expansion(O, I, bits, K, float(f32(gamma)), group, orders)


# ----------------------------------------------------------------------------
# Sec. 4.1: batch-normalization layers are folded into the preceding layer before anything else
# ----------------------------------------------------------------------------
def fold_batchnorm(W: np.ndarray, b, gamma: np.ndarray, beta: np.ndarray, mean: np.ndarray,
                   var: np.ndarray, eps: float):
    """The layer y = BN(W x + b), BN(z) = gamma (z - mean) / sqrt(var + eps) + beta per output
    channel, as one affine layer: W'[o,:] = W[o,:] * g[o], b'[o] = (b[o] - mean[o]) * g[o] + beta[o]
    with g = gamma / sqrt(var + eps) evaluated in fp64 from the fp32 inputs (eps as fp32) and
    rounded once to fp32; the products and sums are fp32, one rounding per operation (the
    folded weight is what gets quantized, so its bits matter).  b may be None (taken as 0).
    Returns (W', b')."""
    W = np.asarray(W, dtype=f32)
    g = (np.asarray(gamma, f32).astype(np.float64)
         / np.sqrt(np.asarray(var, f32).astype(np.float64) + np.float64(f32(eps)))).astype(f32)
    Wf = (W * g[:, None]).astype(f32)
    b0 = np.zeros(W.shape[0], f32) if b is None else np.asarray(b, f32)
    bf = (((b0 - np.asarray(mean, f32)).astype(f32) * g).astype(f32) + np.asarray(beta, f32)).astype(f32)
    return Wf, bf


# ----------------------------------------------------------------------------
# App. B, Eq. (define_dre): f(x) = sigma( sum_k R^(k) Q(x) lambda_{R^(k)} lambda_x + b )
# ----------------------------------------------------------------------------
def quantize_activations(x: np.ndarray, s_x: Optional[float] = None, bits: int = 8):
    """Per-tensor symmetric a-bit codes (a = bits, 8 unless stated; Sec. 4 also uses A6 and
    A4), held in int8.  s_x > 0: static scale; None or <= 0: max|x| / (2^(a-1)-1).
    Returns (Qx int8 same shape, s_x fp32).  s_x == 0 (all-zero input) gives Qx = 0."""
    x = np.asarray(x, dtype=f32)
    qa = q_max(bits)
    if s_x is None or not (s_x > 0):
        amax = np.max(np.abs(x)) if x.size else f32(0)
        s = f32(f32(amax) / f32(qa))
    else:
        s = f32(s_x)
    if not (s > 0):
        return np.zeros(x.shape, np.int8), f32(0)
    q = np.clip(np.rint(x / s), -qa, qa)
    return q.astype(np.int8), s


def quantize_activations_asymmetric(x: np.ndarray, bits: int = 8):
    """Per-tensor asymmetric a-bit codes (Sec. 4.3 runs its comparison under asymmetric
    quantization; the paper gives no formula, this is the usual affine quantizer):
    with hi = max(x, 0) and lo = min(x, 0) over the tensor (so that 0 is a grid point),
      s = (hi - lo) / (2^a - 1),  z = clamp(rint(-lo / s), 0, 2^a - 1),
      Q(x) = clamp(rint(x / s) + z, 0, 2^a - 1),   x ~ s * (Q(x) - z),
    fp32 sums and divisions, rint half to even.  Returns (Q int16 in [0, 2^a - 1], s fp32, z int).
    An all-zero input gives Q = 0, s = 0, z = 0."""
    x = np.asarray(x, dtype=f32)
    if not 2 <= int(bits) <= 8:
        raise ValueError("bits must lie in 2..8")
    qa = 2 ** int(bits) - 1
    hi = f32(max(float(np.max(x)), 0.0)) if x.size else f32(0)
    nlo = f32(max(float(np.max(-x)), 0.0)) if x.size else f32(0)
    s = f32(f32(hi + nlo) / f32(qa))
    if not (s > 0):
        return np.zeros(x.shape, np.int16), f32(0), 0
    z = int(np.clip(np.rint(f32(nlo) / s), 0, qa))
    q = np.clip(np.rint(x / s) + f32(z), 0, qa)
    return q.astype(np.int16), s, z


def contract(Qx: np.ndarray, codes: np.ndarray) -> np.ndarray:
    """acc[t, r] = sum_i Qx[t,i] * codes[r,i], exact, returned as int32.

    The products are formed and summed by an fp64 matmul: every operand is an
    integer of magnitude <= 255 and every partial sum is an integer below
    255*127*I < 2^53, so each fp64 operation is exact whatever the order."""
    I = Qx.shape[1]
    bound = int(np.max(np.abs(Qx.astype(np.int64)))) if Qx.size else 0     # 127, or up to 255 for centred asymmetric codes
    if max(bound, 127) * 127 * max(I, 1) >= 2 ** 31:
        raise ValueError("accumulator would not fit int32")
    a = Qx.astype(np.float64) @ codes.astype(np.float64).T
    return a.astype(np.int64).astype(np.int32)


def forward_acc(exp: Expansion, Qx: np.ndarray) -> np.ndarray:
    """int32 [K, T, O]: acc_k[t,o] = sum_i Qx[t,i] q_k[o,i]; pruned rows are 0."""
    T = Qx.shape[0]
    acc = np.zeros((exp.K, T, exp.out_features), dtype=np.int32)
    for k in range(1, exp.K + 1):
        acc[k - 1][:, exp.rows(k)] = contract(Qx, exp.orders[k - 1].codes)
    return acc


def member_ranges(K: int, split: Optional[Sequence[int]]):
    """[K_1..K_M] -> list of 1-based inclusive order ranges; None means one member."""
    if split is None:
        split = [K]
    if len(split) < 1 or any(int(s) < 1 for s in split) or sum(int(s) for s in split) != K:
        raise ValueError("split must be positive and sum to K")
    out, lo = [], 1
    for s in split:
        out.append((lo, lo + int(s) - 1))
        lo += int(s)
    return out


def dequantize(exp: Expansion, acc: np.ndarray, s_x, split=None, bias=None, dtype=f32):
    """Members' outputs [M, T, O]: y_m = s_x * sum_{k in m, ascending} s_k[o]*acc_k[t,o]
    (+ b[o] for the first member only), evaluated in `dtype`."""
    rngs = member_ranges(exp.K, split)
    T = acc.shape[1]
    ys = np.zeros((len(rngs), T, exp.out_features), dtype=dtype)
    for m, (lo, hi) in enumerate(rngs):
        tot = np.zeros((T, exp.out_features), dtype=dtype)
        for k in range(lo, hi + 1):
            term = exp.dense_scales(k).astype(dtype)[None, :] * acc[k - 1].astype(dtype)
            tot = (tot + term).astype(dtype)
        ym = (dtype(s_x) * tot).astype(dtype)
        if m == 0 and bias is not None:
            ym = (ym + np.asarray(bias).astype(dtype)[None, :]).astype(dtype)
        ys[m] = ym
    return ys


def sum_members(ys: np.ndarray) -> np.ndarray:
    """Ensemble output: members added in ascending order, in the array's dtype."""
    y = ys[0].copy()
    for m in range(1, ys.shape[0]):
        y = (y + ys[m]).astype(ys.dtype)
    return y


def forward(exp: Expansion, x: np.ndarray, s_x: Optional[float] = None, split=None,
            bias=None, reduce_members: bool = True, act_bits: int = 8):
    """Expanded linear layer on x [T, I].  Returns a dict with Qx, s_x, acc (int32
    [K,T,O]), y (fp32; [T,O] if reduce_members else [M,T,O]) and y64 (fp64 twin)."""
    Qx, sx = quantize_activations(x, s_x, act_bits)
    acc = forward_acc(exp, Qx)
    ys = dequantize(exp, acc, sx, split, bias, f32)
    ys64 = dequantize(exp, acc, sx, split, bias, np.float64)
    if reduce_members:
        return dict(Qx=Qx, s_x=sx, acc=acc, y=sum_members(ys), y64=sum_members(ys64))
    return dict(Qx=Qx, s_x=sx, acc=acc, y=ys, y64=ys64)


def forward_asymmetric(exp: Expansion, x: np.ndarray, split=None, bias=None, act_bits: int = 8):
    """The expanded layer with asymmetric activation codes: acc_k[t,o] = sum_i (Q(x)[t,i] - z) q_k[o,i]
    (exact), y = s * sum_k s_k acc_k (+ b), members summed.  Returns a dict with Qx (unsigned codes),
    s_x, z, acc (int32 [K,T,O]), y (fp32 [T,O]) and y64."""
    Qx, sx, z = quantize_activations_asymmetric(x, act_bits)
    acc = forward_acc(exp, Qx.astype(np.int32) - z)
    ys = dequantize(exp, acc, sx, split, bias, f32)
    ys64 = dequantize(exp, acc, sx, split, bias, np.float64)
    return dict(Qx=Qx, s_x=sx, z=z, acc=acc, y=sum_members(ys), y64=sum_members(ys64))


# ----------------------------------------------------------------------------
# Convolution (App. H treats conv and fully-connected layers uniformly)
# ----------------------------------------------------------------------------
def conv_out_size(H, W, kh, kw, stride, pad):
    return (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1


def conv2d_acc_direct(Qx: np.ndarray, codes: np.ndarray, kh: int, kw: int,
                      stride: int, pad: int) -> np.ndarray:
    """Direct integer convolution.  Qx int8 [N,C,H,W] (zero padded), codes int8
    [R, C*kh*kw] with a row flattened as [C, kh, kw].  Returns int32 [N*Ho*Wo, R]
    with tokens ordered (n, ho, wo).  One accumulation per kernel tap (r, s)."""
    N, C, H, W = Qx.shape
    R = codes.shape[0]
    Ho, Wo = conv_out_size(H, W, kh, kw, stride, pad)
    xp = np.zeros((N, C, H + 2 * pad, W + 2 * pad), dtype=np.int64)
    xp[:, :, pad:pad + H, pad:pad + W] = Qx
    w = codes.astype(np.int64).reshape(R, C, kh, kw)
    acc = np.zeros((N, Ho, Wo, R), dtype=np.int64)
    for r in range(kh):
        for s in range(kw):
            patch = xp[:, :, r:r + stride * Ho:stride, s:s + stride * Wo:stride]   # [N,C,Ho,Wo]
            acc += np.einsum("nchw,oc->nhwo", patch, w[:, :, r, s])
    return acc.reshape(N * Ho * Wo, R).astype(np.int32)


def im2col(Q: np.ndarray, kh: int, kw: int, stride: int, pad: int) -> np.ndarray:
    """[N,C,H,W] -> [N*Ho*Wo, C*kh*kw], column index (c, r, s), zero padding."""
    N, C, H, W = Q.shape
    Ho, Wo = conv_out_size(H, W, kh, kw, stride, pad)
    xp = np.zeros((N, C, H + 2 * pad, W + 2 * pad), dtype=Q.dtype)
    xp[:, :, pad:pad + H, pad:pad + W] = Q
    cols = np.zeros((N, Ho, Wo, C, kh, kw), dtype=Q.dtype)
    for r in range(kh):
        for s in range(kw):
            cols[:, :, :, :, r, s] = xp[:, :, r:r + stride * Ho:stride,
                                        s:s + stride * Wo:stride].transpose(0, 2, 3, 1)
    return cols.reshape(N * Ho * Wo, C * kh * kw)


def forward_conv2d(exp: Expansion, x: np.ndarray, kh, kw, stride, pad,
                   s_x: Optional[float] = None, split=None, bias=None,
                   reduce_members: bool = True, act_bits: int = 8):
    """Expanded conv layer on x [N,C,H,W] fp32; output rows are tokens (n, ho, wo),
    i.e. y is [N*Ho*Wo, O] (channels last)."""
    Qx, sx = quantize_activations(x, s_x, act_bits)
    T = Qx.shape[0] * np.prod(conv_out_size(x.shape[2], x.shape[3], kh, kw, stride, pad))
    acc = np.zeros((exp.K, int(T), exp.out_features), dtype=np.int32)
    for k in range(1, exp.K + 1):
        acc[k - 1][:, exp.rows(k)] = conv2d_acc_direct(Qx, exp.orders[k - 1].codes,
                                                        kh, kw, stride, pad)
    ys = dequantize(exp, acc, sx, split, bias, f32)
    ys64 = dequantize(exp, acc, sx, split, bias, np.float64)
    if reduce_members:
        return dict(Qx=Qx, s_x=sx, acc=acc, y=sum_members(ys), y64=sum_members(ys64))
    return dict(Qx=Qx, s_x=sx, acc=acc, y=ys, y64=ys64)


def forward_conv2d_asymmetric(exp: Expansion, x: np.ndarray, kh, kw, stride, pad, split=None, bias=None,
                              act_bits: int = 8):
    """The expanded conv layer with asymmetric activation codes (quantize_activations_asymmetric over
    the whole input tensor): the direct integer convolution runs on Q(x) - z, so the zero padding
    of the input is the real value 0 (code z).  Members summed; y is [N*Ho*Wo, O]."""
    Qx, sx, z = quantize_activations_asymmetric(x, act_bits)
    Qc = Qx.astype(np.int32) - z
    T = Qx.shape[0] * np.prod(conv_out_size(x.shape[2], x.shape[3], kh, kw, stride, pad))
    acc = np.zeros((exp.K, int(T), exp.out_features), dtype=np.int32)
    for k in range(1, exp.K + 1):
        acc[k - 1][:, exp.rows(k)] = conv2d_acc_direct(Qc, exp.orders[k - 1].codes, kh, kw, stride, pad)
    ys = dequantize(exp, acc, sx, split, bias, f32)
    ys64 = dequantize(exp, acc, sx, split, bias, np.float64)
    return dict(Qx=Qx, s_x=sx, z=z, acc=acc, y=sum_members(ys), y64=sum_members(ys64))


def depthwise_acc_direct(Qx: np.ndarray, codes: np.ndarray, kh: int, kw: int, stride: int, pad: int) -> np.ndarray:
    """Depthwise integer convolution: one kh x kw filter per channel (App. H: a conv with
    n_i = 1).  Qx int8 [N,C,H,W], codes int8 [C, kh*kw] (row c = filter of channel c, flattened
    [kh, kw]).  Returns int32 [N*Ho*Wo, C]: acc[(n,ho,wo), c] = sum_{r,q} Qx[n,c,ho*s-p+r,wo*s-p+q]
    * codes[c, r*kw+q], zero outside the image.  Exact (int64 sums of |terms| <= 127*127)."""
    N, C, H, W = Qx.shape
    Ho, Wo = conv_out_size(H, W, kh, kw, stride, pad)
    xp = np.zeros((N, C, H + 2 * pad, W + 2 * pad), dtype=np.int64)
    xp[:, :, pad:pad + H, pad:pad + W] = Qx
    acc = np.zeros((N, Ho, Wo, C), dtype=np.int64)
    for r in range(kh):
        for q in range(kw):
            win = xp[:, :, r:r + stride * (Ho - 1) + 1:stride, q:q + stride * (Wo - 1) + 1:stride]   # [N,C,Ho,Wo]
            acc += win.transpose(0, 2, 3, 1) * codes[:, r * kw + q].astype(np.int64)[None, None, None, :]
    return acc.reshape(N * Ho * Wo, C).astype(np.int32)


def forward_depthwise2d(exp: Expansion, x: np.ndarray, kh, kw, stride, pad,
                        s_x: Optional[float] = None, split=None, bias=None,
                        reduce_members: bool = True, act_bits: int = 8):
    """Expanded depthwise conv layer: exp was built from W [C, kh*kw]; x [N,C,H,W] fp32.
    Output rows are pixels (n, ho, wo): y is [N*Ho*Wo, C] (channels last).  Same quantizer,
    per-channel scales, member ranges and evaluation order as the dense layers."""
    if exp.out_features != x.shape[1] or exp.in_features != kh * kw:
        raise ValueError("depthwise: expansion must be [C, kh*kw]")
    Qx, sx = quantize_activations(x, s_x, act_bits)
    T = Qx.shape[0] * int(np.prod(conv_out_size(x.shape[2], x.shape[3], kh, kw, stride, pad)))
    acc = np.zeros((exp.K, T, exp.out_features), dtype=np.int32)
    for k in range(1, exp.K + 1):
        rows = exp.rows(k)
        acc[k - 1][:, rows] = depthwise_acc_direct(Qx[:, rows], exp.orders[k - 1].codes, kh, kw, stride, pad)
    ys = dequantize(exp, acc, sx, split, bias, f32)
    ys64 = dequantize(exp, acc, sx, split, bias, np.float64)
    if reduce_members:
        return dict(Qx=Qx, s_x=sx, acc=acc, y=sum_members(ys), y64=sum_members(ys64))
    return dict(Qx=Qx, s_x=sx, acc=acc, y=ys, y64=ys64)


# ----------------------------------------------------------------------------
# Sec. 3.2 / App. B: ensemble of M predictors over a two-layer MLP
# ----------------------------------------------------------------------------
def gelu(v: np.ndarray) -> np.ndarray:
    """erf-form GELU of fp32 values, evaluated in fp64 and rounded once to fp32."""
    from scipy.special import erf
    v64 = np.asarray(v, dtype=np.float64)
    return (0.5 * v64 * (1.0 + erf(v64 / math.sqrt(2.0)))).astype(f32)


def silu_mul(gate: np.ndarray, up: np.ndarray) -> np.ndarray:
    """SiLU(gate) * up of fp32 values, evaluated in fp64 and rounded once to fp32."""
    g = np.asarray(gate, dtype=np.float64)
    return (g / (1.0 + np.exp(-g)) * np.asarray(up, dtype=np.float64)).astype(f32)


def mlp_forward(exp1: Expansion, exp2: Expansion, kind: str, x: np.ndarray, split=None,
                bias1=None, bias2=None, s_x: Optional[float] = None, act_bits: int = 8,
                asymmetric: bool = False, s_h: Optional[Sequence[float]] = None):
    """Two expanded layers with an activation between, run as an ensemble.

    Member m uses only its own orders in BOTH layers, quantizes its own hidden
    activation with its own dynamic scale, and carries the biases only if m is the
    first member; the members' outputs are summed after the last layer.
    kind = "gelu": h = GELU(layer1(x));  kind = "gated": layer1 has 2H outputs
    (gate rows first, then up rows) and h = SiLU(gate) * up.
    s_h: given (static) scales of the members' hidden activations instead of their dynamic ones.
    asymmetric: the input and every member's hidden activation get the affine codes of
    Sec. 4.3 (quantize_activations_asymmetric), each over its own range; the contractions run
    on the codes minus their zero point.
    Returns dict(y fp32 [T,O2], members [M,T,O2], h [M,T,H], s_h [M])."""
    if exp1.K != exp2.K:
        raise ValueError("both layers need the same expansion order")
    rngs = member_ranges(exp1.K, split)
    if asymmetric:
        if s_x is not None:
            raise ValueError("asymmetric codes take their range from the tensor")
        Qu, sx, zx = quantize_activations_asymmetric(x, act_bits)
        Qx = Qu.astype(np.int32) - int(zx)
    else:
        Qx, sx = quantize_activations(x, s_x, act_bits)
    acc1 = forward_acc(exp1, Qx)
    y1 = dequantize(exp1, acc1, sx, split, bias1, f32)          # [M, T, O1]
    hs = []
    for m in range(len(rngs)):
        if kind == "gelu":
            h = gelu(y1[m])
        elif kind == "gated":
            H = exp1.out_features // 2
            h = silu_mul(y1[m][:, :H], y1[m][:, H:])
        else:
            raise ValueError("kind must be 'gelu' or 'gated'")
        hs.append(h)
    hs = np.stack(hs)
    second = mlp_second_layer(exp2, hs, split, bias2, act_bits, asymmetric, s_h)
    second.update(h=hs, y1=y1, s_x=sx, Qx=Qx)
    return second


def mlp_second_layer(exp2: Expansion, hs: np.ndarray, split=None, bias2=None, act_bits: int = 8,
                     asymmetric: bool = False, s_h: Optional[Sequence[float]] = None):
    """Last layer of the ensemble on given hidden activations hs [M, T, H]: member m
    quantizes hs[m] with its own dynamic scale, uses its own orders of exp2 (bias in
    the first member only), and the members are summed in ascending order.
    Returns dict(y [T,O2], members [M,T,O2], s_h [M], Qh [M,T,H])."""
    rngs = member_ranges(exp2.K, split)
    if hs.shape[0] != len(rngs):
        raise ValueError("one hidden activation per member")
    outs, shs, Qhs = [], [], []
    for m in range(len(rngs)):
        if asymmetric:
            Qu, sh, zh = quantize_activations_asymmetric(hs[m], act_bits)
            Qh = Qu.astype(np.int32) - int(zh)
        else:
            Qh, sh = quantize_activations(hs[m], None if s_h is None else float(s_h[m]), act_bits)
        acc2 = forward_acc(exp2, Qh)
        outs.append(dequantize(exp2, acc2, sh, split, bias2 if m == 0 else None, f32)[m])
        shs.append(sh)
        Qhs.append(Qh)
    members = np.stack(outs)
    return dict(y=sum_members(members), members=members, s_h=np.array(shs, dtype=f32),
                Qh=np.stack(Qhs))


# ----------------------------------------------------------------------------
# App. B "Ensemble of more Layers" / App. D "Ensembling with more Layers":
# an L-layer feed-forward network as M independent member chains
# ----------------------------------------------------------------------------
@dataclass
class ChainLayer:
    """One layer of the chain: z = expanded layer (+ bias), then activation and skip.

    act          "none" | "relu" | "gelu" (erf form)
    skip_from    -1: no skip; j >= 0: add the tensor that ENTERED layer j (0-based;
                 j = 0 is the network input, j <= this layer's index), as in the residual
                 network of Fig. 2
    skip_pre_act True: a = act(z + r) (ResNet block); False: a = act(z) + r
    kh, kw, stride, pad   kh = 0: a fully-connected layer applied to every token; kh > 0: a
                 convolution over the [N, H, W] grid the tokens form (tensors are channels
                 last, tokens ordered (n, h, w)), exp built from W [O, C*kh*kw]
    s_in         None, or one given (static) activation scale per member for the tensors that
                 enter this layer (Sec. 4: ranges fixed ahead of time); not used by the first
                 layer, whose shared input takes chain_forward's s_x"""
    exp: Expansion
    bias: Optional[np.ndarray] = None
    act: str = "none"
    skip_from: int = -1
    skip_pre_act: bool = True
    kh: int = 0
    kw: int = 0
    stride: int = 1
    pad: int = 0
    s_in: Optional[Sequence[float]] = None


def chain_layer_acc(layer: ChainLayer, Qa: np.ndarray, grid):
    """Integer accumulators [K, T', O] of one layer on codes Qa [T, C] whose tokens form the
    grid (N, H, W); returns them with the output grid.  A fully-connected layer keeps the grid."""
    exp = layer.exp
    if layer.kh == 0:
        return forward_acc(exp, Qa), grid
    N, H, W = grid
    C = Qa.shape[1]
    Qn = Qa.reshape(N, H, W, C).transpose(0, 3, 1, 2)
    Ho, Wo = conv_out_size(H, W, layer.kh, layer.kw, layer.stride, layer.pad)
    acc = np.zeros((exp.K, N * Ho * Wo, exp.out_features), dtype=np.int32)
    for k in range(1, exp.K + 1):
        acc[k - 1][:, exp.rows(k)] = conv2d_acc_direct(Qn, exp.orders[k - 1].codes, layer.kh, layer.kw,
                                                        layer.stride, layer.pad)
    return acc, (N, Ho, Wo)


def relu(v: np.ndarray) -> np.ndarray:
    return np.maximum(np.asarray(v, dtype=f32), f32(0))


def chain_layer_members(layer: ChainLayer, inputs: np.ndarray, shared_input: bool, skips,
                        split=None, s_x: Optional[float] = None, act_bits: int = 8, grid=None,
                        asymmetric: bool = False) -> np.ndarray:
    """One layer for all members.  inputs: [T, I] when every member reads the same tensor
    (the network input; s_x is its static scale if given), else [M, T, I] and member m
    quantizes inputs[m] with its own dynamic scale.  Member m contracts with its own orders
    only; the bias goes to the first member.  skips: None, or a list of M entries (an array
    [T, O] or None) added before or after the activation.  grid = (N, H, W) of the tokens
    (needed by convolution layers; default: T tokens, no spatial extent).
    asymmetric: every tensor entering the layer is quantized with the affine quantizer of
    Sec. 4.3 (quantize_activations_asymmetric) over its own range, and the contraction runs on
    the codes minus their zero point (a tap outside the image then contributes nothing).
    Returns [M, T', O] fp32."""
    exp = layer.exp
    rngs = member_ranges(exp.K, split)
    M = len(rngs)
    out = []
    for m in range(M):
        xin = inputs if shared_input else inputs[m]
        if asymmetric:
            if s_x is not None:
                raise ValueError("asymmetric codes take their range from the tensor")
            Qu, sa, zp = quantize_activations_asymmetric(xin, act_bits)
            Qa = Qu.astype(np.int32) - int(zp)
        else:
            given = s_x if shared_input else (None if layer.s_in is None else float(layer.s_in[m]))
            Qa, sa = quantize_activations(xin, given, act_bits)
        acc, _ = chain_layer_acc(layer, Qa, grid if grid is not None else (Qa.shape[0], 1, 1))
        z = dequantize(exp, acc, sa, split, layer.bias, f32)[m]
        r = None if skips is None else skips[m]
        if r is not None and layer.skip_pre_act:
            z = (z + np.asarray(r, dtype=f32)).astype(f32)
        if layer.act == "relu":
            a = relu(z)
        elif layer.act == "gelu":
            a = gelu(z)
        elif layer.act == "none":
            a = z
        else:
            raise ValueError("act must be 'none', 'relu' or 'gelu'")
        if r is not None and not layer.skip_pre_act:
            a = (a + np.asarray(r, dtype=f32)).astype(f32)
        out.append(a.astype(f32))
    return np.stack(out)


def chain_skips(layers: Sequence[ChainLayer], l: int, x: np.ndarray, acts: Sequence[np.ndarray], M: int):
    """The tensors layer l adds: member m's own copy of what entered layer skip_from.  The
    network input is not split over the members, so -- like the bias -- a skip that reads it
    enters the sum once, through the first member."""
    j = layers[l].skip_from
    if j < 0:
        return None
    if j > l:
        raise ValueError("a skip reads an earlier tensor")
    if j == 0:
        return [np.asarray(x, dtype=f32)] + [None] * (M - 1)
    return [acts[j - 1][m] for m in range(M)]


def chain_grids(layers: Sequence[ChainLayer], grid):
    """The token grid (N, H, W) entering every layer, and the one leaving the last."""
    grids = [tuple(grid)]
    for ly in layers:
        N, H, W = grids[-1]
        if ly.kh > 0:
            H, W = conv_out_size(H, W, ly.kh, ly.kw, ly.stride, ly.pad)
        grids.append((N, H, W))
    return grids


def chain_forward(layers: Sequence[ChainLayer], x: np.ndarray, split=None, s_x: Optional[float] = None,
                  act_bits: int = 8, grid=None, asymmetric: bool = False):
    """M member chains through L expanded layers, summed after the last one.

    Member m is the whole architecture with, in every layer, only the orders of its own
    cluster; it quantizes each hidden activation with its own dynamic per-tensor scale;
    biases (and a skip from the network input) belong to the first member.  The last
    layer has no activation of its own (act must be "none").  x is [T, C]; with convolution
    layers its tokens form grid = (N, H, W), ordered (n, h, w) (a channels-last image).
    asymmetric: the network input and every member's hidden tensors get asymmetric codes
    (Sec. 4.3), each over its own range.
    Returns dict(y [T_L, O_L], members [M, T_L, O_L], acts: list of L-1 arrays [M, T_l, O_l])."""
    L = len(layers)
    if L < 1:
        raise ValueError("at least one layer")
    K = layers[0].exp.K
    if any(ly.exp.K != K for ly in layers):
        raise ValueError("all layers need the same expansion order")
    if layers[-1].act != "none":
        raise ValueError("the last layer has no activation")
    M = len(member_ranges(K, split))
    x = np.asarray(x, dtype=f32)
    grids = chain_grids(layers, grid if grid is not None else (x.shape[0], 1, 1))
    acts: List[np.ndarray] = []
    for l, ly in enumerate(layers):
        skips = chain_skips(layers, l, x, acts, M)
        if l == 0:
            a = chain_layer_members(ly, x, True, skips, split, s_x, act_bits, grids[0], asymmetric)
        else:
            a = chain_layer_members(ly, acts[l - 1], False, skips, split, None, act_bits, grids[l], asymmetric)
        acts.append(a)
    members = acts.pop()
    return dict(y=sum_members(members), members=members, acts=acts)


# ----------------------------------------------------------------------------
# App. C: data-free error diagnostics (Theorems "dre_upperbound" / "slim_upperbound")
# ----------------------------------------------------------------------------
def power_start_vector(n: int) -> np.ndarray:
    """The fixed start vector of the power iteration: +-1 by a multiplicative integer hash of
    the index (bit 15 of i * 2654435761 mod 2^32), scaled to unit length.  Both sides use the
    same vector so that the iterates can be compared step by step."""
    i = np.arange(n, dtype=np.uint64)
    bit = ((i * np.uint64(2654435761)) & np.uint64(0xFFFFFFFF)) >> np.uint64(15) & np.uint64(1)
    v = np.where(bit == 1, 1.0, -1.0)
    return v / math.sqrt(n)


def spectral_norm(W: np.ndarray, iters: int) -> float:
    """s = largest singular value of W (the theorems' s_l), by `iters` steps of the power
    iteration on W^T W in fp64: v <- W^T (W v) / ||W^T (W v)||, returning ||W v|| for the last
    v (a lower bound of s that converges to it).  A zero matrix gives 0."""
    W = np.asarray(W, dtype=np.float64)
    v = power_start_vector(W.shape[1])
    sigma = 0.0
    for _ in range(int(iters)):
        y = W @ v
        sigma = float(np.linalg.norm(y))
        z = W.T @ y
        nz = float(np.linalg.norm(z))
        if nz == 0.0:
            return 0.0
        v = z / nz
    return float(np.linalg.norm(W @ v))


def lemma_bound_u(exp: Expansion) -> float:
    """u^(K) of a dense expansion (Lemma, Eq. exponential_decrease): the element-wise bound
    (1/q_max)^(K-1) * lambda / 2 with lambda read as the FIRST-order row scale (with the
    order-K scale, as printed, the bound is not the one the proof gives: the tight fact is
    |error| <= s_K / 2 and s_K <= s_1 / (2 q_max)^(K-1)); the layer's figure is its maximum
    over rows.  Holds for every row that is stored at every order."""
    qm = float(q_max(exp.bits))
    s1 = float(np.max(exp.orders[0].scales)) if exp.orders[0].scales.size else 0.0
    return (1.0 / qm) ** (exp.K - 1) * s1 / 2.0


def stored_bound_u(exp: Expansion) -> float:
    """Element-wise error bound of a (possibly sparse) expansion from what is stored: a row's
    error after its LAST stored order k* is at most s_k*/2 and later orders that prune the row
    pass the residual on unchanged.  The layer's figure is the maximum over rows.  This is the
    provable counterpart of Lemma "slim", whose printed numerator (a norm vector N^(K) times an
    indicator) the paper does not define."""
    last = np.zeros(exp.out_features, dtype=np.float64)
    for k in range(1, exp.K + 1):
        rows = exp.rows(k)
        last[rows] = exp.orders[k - 1].scales.astype(np.float64)
    return float(last.max()) / 2.0 if last.size else 0.0


def error_bound_U(s: Sequence[float], u: Sequence[float]) -> float:
    """U = prod_{l=1..L} ( sum_{i=1..l} s_i u_i + 1 ) - 1 (Theorem dre_upperbound; the same
    form with the sparse u gives U_sparse), exactly as printed."""
    if len(s) != len(u):
        raise ValueError("one s and one u per layer")
    U, run = 1.0, 0.0
    for sl, ul in zip(s, u):
        run += float(sl) * float(ul)
        U *= run + 1.0
    return U - 1.0


def order_norms(exp: Expansion, iters: int) -> List[float]:
    """||R^(k)|| for k = 1..K: the spectral norm (power iteration above) of each term of the
    expansion as a real matrix, row scale times codes, pruned rows zero (Eq. 3).  These are the
    operator norms Theorem "ensemble" and its two-layer corollary are written in."""
    out = []
    for k in range(1, exp.K + 1):
        Rk = exp.dense_scales(k).astype(np.float64)[:, None] * exp.dense_codes(k).astype(np.float64)
        out.append(spectral_norm(Rk, iters))
    return out


def error_bound_U_ens(norms: Sequence[Sequence[float]], split, lam: Optional[Sequence[Sequence[float]]] = None) -> float:
    """U_ens of Theorem "ensemble" (App. C) for an L-layer network split into M predictors:

        U_ens = ( sum_{k in cluster 1} ||R_L^(k)|| / 2^(L-1) )
                * ( 1 + sum_{m=2..M} prod_{l=1..L-1} sum_{k in cluster m} ||R_l^(k)|| lam_l^(k) )

    norms[l][k] = ||R_{l+1}^(k+1)|| (L rows of K).  The printed inner sum runs over
    k = K_m..K_{m+1} and writes R_L inside the product over l; read here as "the orders of
    cluster m" and "the weights of layer l".  lam[l][k] stands for the printed
    lambda_{h~_l^(k)} (the scale of the quantized tensor entering the next layer), which the
    paper does not make data-free; None means 1."""
    L = len(norms)
    if L < 1:
        raise ValueError("at least one layer")
    K = len(norms[0])
    if any(len(r) != K for r in norms):
        raise ValueError("one norm per order and layer")
    rngs = member_ranges(K, split)
    lo1, hi1 = rngs[0]
    head = sum(float(norms[L - 1][k - 1]) for k in range(lo1, hi1 + 1)) / (2.0 ** (L - 1))
    tail = 0.0
    for lo, hi in rngs[1:]:
        prod = 1.0
        for l in range(L - 1):
            prod *= sum(float(norms[l][k - 1]) * (1.0 if lam is None else float(lam[l][k - 1])) for k in range(lo, hi + 1))
        tail += prod
    return head * (1.0 + tail)


def first_predictor_size(norms, logit_norm: float, ratio: float, lam=None) -> int:
    """The predictor-size rule of App. A as a procedure: the smallest K_1 for which the
    two-predictor ensemble [K_1, K - K_1] has U_ens <= ratio * logit_norm (the bound
    "vanishes compared to" the amplitude of the logits); K if no split qualifies."""
    K = len(norms[0])
    for K1 in range(1, K):
        if error_bound_U_ens(norms, [K1, K - K1], lam) <= ratio * logit_norm:
            return K1
    return K


# ----------------------------------------------------------------------------
# App. H: operation head-count
# ----------------------------------------------------------------------------
def bit_operations(D: int, d: int, n_i: int, n_o: int, s: int, b: int, k: int):
    """Bit-operation counts (original layer, quantized layer, expansion with k
    b-bit terms) for a d x d conv on D x D x n_i maps, n_o outputs, stride s; a
    fully-connected layer has D = d = s = 1.  log is taken base 2."""
    fp = 32 * math.log2(32)
    ib = b * math.log2(b)
    mults = d * d * n_i * n_o / (s * s)
    original = D * D * mults * fp
    rescale = (n_i + n_o / (s * s)) * fp
    quantized = D * D * (rescale + mults * ib)
    expanded = D * D * (rescale + k * mults * ib)
    return original, quantized, expanded


def expansion_macs(exp: Expansion, T: int) -> int:
    """Integer multiply-accumulates one forward over T tokens performs: T * I *
    (number of stored rows over all orders)."""
    return int(T) * exp.in_features * sum(o.codes.shape[0] for o in exp.orders)
