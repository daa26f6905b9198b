"""Pins for the CPU checker: every check here rests on something other than the
checker's own formulas -- a hand-worked example, an exhaustive search, the
paper's bounds, brute-force enumeration, or an independent library routine."""
import itertools
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import pipe_oracle as po
from paper_2311_15806_amd import workloads as wl

f32 = np.float32


def _rand_w(seed, O, I, heavy=False):
    rng = np.random.default_rng(seed)
    if heavy:
        return (rng.standard_t(3, size=(O, I)) * 0.015).astype(f32)
    return (rng.standard_normal((O, I)) * 0.02).astype(f32)


# ---------------------------------------------------------------- hand-worked example
def test_hand_worked_example(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "hand_worked.json")))
    for name in ("ternary", "int4"):
        c = g[name]
        W = np.array(c["W"], dtype=f32)
        res = []
        e = po.expand(W, c["bits"], c["K"], 1.0, 1, residuals=res)
        for k in range(c["K"]):
            assert e.orders[k].codes.tolist() == c["codes"][k], (name, k)
            assert e.orders[k].scales.tolist() == c["scales"][k], (name, k)
            assert res[k].tolist() == c["residual_after"][k], (name, k)
    c = g["ternary"]
    e = po.expand(np.array(c["W"], dtype=f32), 2, 3, 1.0, 1)
    r = po.forward(e, np.array(c["x"], dtype=f32), s_x=c["s_x_static"])
    assert r["Qx"].tolist() == c["Qx"]
    assert r["acc"].tolist() == c["acc"]
    assert r["y"].tolist() == c["y"]
    d = g["dynamic_activation"]
    Qx, sx = po.quantize_activations(np.array(d["x"], dtype=f32))
    assert Qx.tolist() == d["Qx"]
    assert sx == f32(2.0) / f32(127.0)


# ---------------------------------------------------------------- Eq. (1): K = 1 is plain quantization
@pytest.mark.parametrize("bits", [8, 6, 4, 3, 2])
def test_k1_is_nearest_code_by_exhaustive_search(bits):
    """For every element the code must be the integer in [-q_max, q_max] whose
    de-quantized value is nearest (searched exhaustively, no rounding formula),
    the row's largest element must sit on +-q_max, and the error is <= s/2."""
    W = _rand_w(bits, 6, 40, heavy=True)
    e = po.expand(W, bits, 1, 1.0, 1)
    q, s = e.orders[0].codes, e.orders[0].scales
    qm = 2 ** (bits - 1) - 1
    cand = np.arange(-qm, qm + 1)
    for o in range(W.shape[0]):
        j = np.argmax(np.abs(W[o]))
        assert abs(int(q[o, j])) == qm
        assert math.isclose(float(s[o]) * qm, float(abs(W[o, j])), rel_tol=1e-6)
        for i in range(W.shape[1]):
            d = np.abs(float(W[o, i]) - float(s[o]) * cand)
            best = d.min()
            got = abs(float(W[o, i]) - float(s[o]) * int(q[o, i]))
            assert got <= best * (1 + 1e-5) + 1e-12
            assert got <= float(s[o]) / 2 * (1 + 1e-5)


def test_zero_row_and_zero_matrix():
    W = _rand_w(1, 4, 8)
    W[2] = 0
    e = po.expand(W, 4, 3, 1.0, 1)
    for o in e.orders:
        assert o.scales[2] == 0 and not o.codes[2].any()
    e0 = po.expand(np.zeros((4, 8), f32), 2, 2, 0.5, 2)
    assert all(not o.codes.any() and not o.scales.any() for o in e0.orders)
    # exact ties in the scores go to the lower group index
    assert e0.orders[1].group_ids.tolist() == [0]


@pytest.mark.parametrize("a", [8, 6, 4, 2])
def test_activation_codes_are_nearest_on_the_a_bit_grid(a):
    """Q(x) with a-bit activations (Sec. 4: A8, A6, A4): the code is the integer of
    [-(2^(a-1)-1), 2^(a-1)-1] nearest to x / s_x (exhaustive search), the largest |x| sits on the
    last code with the dynamic scale, a static scale clamps, and the hand-worked dynamic example of
    the golden file holds at a = 8."""
    rng = np.random.default_rng(40 + a)
    x = (rng.standard_normal((5, 33)) * 1.7).astype(f32)
    qa = 2 ** (a - 1) - 1
    Q, s = po.quantize_activations(x, None, a)
    assert abs(int(Q.reshape(-1)[np.argmax(np.abs(x))])) == qa
    assert math.isclose(float(s) * qa, float(np.abs(x).max()), rel_tol=1e-6)
    cand = np.arange(-qa, qa + 1)
    for v, q in zip(x.reshape(-1), Q.reshape(-1)):
        d = np.abs(float(v) - float(s) * cand)
        assert abs(float(v) - float(s) * int(q)) <= d.min() * (1 + 1e-5) + 1e-12
    Qs, ss = po.quantize_activations(x, 0.25, a)
    assert ss == f32(0.25) and int(np.abs(Qs).max()) <= qa
    big = np.abs(x) >= 0.25 * (qa + 0.5)
    assert np.all(np.abs(Qs[big]) == qa)
    # fewer bits are a coarser grid of the same range: the de-quantized error bound s/2 scales with it
    assert np.abs(x - s * Q.astype(f32)).max() <= float(s) / 2 * (1 + 1e-5)


def test_forward_with_narrow_activations_is_the_textbook_layer():
    """W4/A4 and W4/A6 forward = integer matmul of the a-bit activation codes with the weight codes
    (torch int64), scaled: pins that act_bits reaches the contraction and nothing else changes."""
    W = _rand_w(45, 16, 24)
    x = np.random.default_rng(46).standard_normal((7, 24)).astype(f32)
    e = po.expand(W, 4, 2, 1.0, 8)
    for a in (4, 6):
        r = po.forward(e, x, act_bits=a)
        Q, s = po.quantize_activations(x, None, a)
        assert np.array_equal(r["Qx"], Q) and int(np.abs(Q).max()) == 2 ** (a - 1) - 1
        want = np.zeros((7, 16))
        for k in (1, 2):
            acc = (torch.from_numpy(Q).long() @ torch.from_numpy(e.dense_codes(k)).long().T).numpy()
            want += e.dense_scales(k).astype(np.float64)[None, :] * acc
        want *= float(s)
        assert np.allclose(r["y64"], want, rtol=1e-12, atol=0)
        assert np.allclose(r["y"], want, rtol=1e-5, atol=1e-7)


# ---------------------------------------------------------------- Lemma (exponential convergence)
@pytest.mark.parametrize("bits,K", [(8, 3), (6, 3), (4, 4), (3, 5), (2, 6)])
def test_lemma_bound_dense(bits, K):
    """Per element: |w - sum_k w^(k)| <= s_K/2, scales shrink by >= 2*q_max per
    order, hence the Lemma's bound (1/q_max)^(K-1) * s_1 / 2; the error norm
    never grows with the order."""
    W = _rand_w(10 + bits, 32, 96, heavy=True)
    qm = 2 ** (bits - 1) - 1
    res = []
    e = po.expand(W, bits, K, 1.0, 8, residuals=res)
    eps = 1 + 4 * 2.0 ** -23
    # the fp32 product s*q rounds once per order: at most 2^-24 of the row's largest weight
    ulp = np.abs(W.astype(np.float64)).max(axis=1, keepdims=True) * 2.0 ** -23
    prev_norm = np.linalg.norm(W.astype(np.float64))
    prev_rowmax = np.abs(W.astype(np.float64)).max(axis=1)
    for k in range(1, K + 1):
        s_k = e.orders[k - 1].scales.astype(np.float64)
        err = np.abs(W.astype(np.float64) - e.reconstruct(k))
        assert np.all(err <= (s_k[:, None] / 2) * eps + k * ulp)
        s1 = e.orders[0].scales.astype(np.float64)
        assert np.all(err <= ((1.0 / qm) ** (k - 1)) * (s1[:, None] / 2) * eps + k * ulp)
        if k > 1:
            s_prev = e.orders[k - 2].scales.astype(np.float64)
            assert np.all(s_k <= s_prev / (2 * qm) * eps)
        # the tracked fp32 residual is the true error up to fp32 rounding
        assert np.allclose(res[k - 1], W.astype(np.float64) - e.reconstruct(k),
                           rtol=0, atol=float(np.abs(W).max()) * 2.0 ** -21)
        norm = np.linalg.norm(err)
        assert norm <= prev_norm
        prev_norm = norm
        # row-wise infinity norm of the error shrinks by 2*q_max = 2^b - 2 per order
        rowmax = err.max(axis=1)
        assert np.all(rowmax <= prev_rowmax / (2 * qm) * (1 + 1e-5) + k * ulp[:, 0])
        prev_rowmax = rowmax


# ---------------------------------------------------------------- masks
@pytest.mark.parametrize("bits", [4, 2])
def test_gamma_one_equals_dense(bits):
    W = _rand_w(20, 48, 64)
    a = po.expand(W, bits, 3, 1.0, 16)
    b = po.expand(W, bits, 3, 1.0, 4)        # grouping is irrelevant when nothing is pruned
    for k in range(3):
        assert a.orders[k].group_ids.tolist() == list(range(3))
        assert np.array_equal(a.dense_codes(k + 1), b.dense_codes(k + 1))
        assert np.array_equal(a.dense_scales(k + 1), b.dense_scales(k + 1))
    # and order-by-order it is the plain quantizer applied to the running residual
    E = W.copy()
    for k in range(3):
        q, s = po.quantize_rows(E, bits)
        assert np.array_equal(q, a.orders[k].codes)
        E = (E - (s[:, None] * q.astype(f32))).astype(f32)


def test_sparse_expansion_structure():
    W = _rand_w(21, 64, 80, heavy=True)
    G, gamma, K, bits = 8, 0.5, 4, 4
    res = []
    e = po.expand(W, bits, K, gamma, G, residuals=res)
    assert e.orders[0].group_ids.tolist() == list(range(8))        # R^1 is dense
    prev = res[0]
    for k in range(2, K + 1):
        gids = e.orders[k - 1].group_ids
        assert len(gids) == 4 and len(set(gids.tolist())) == 4
        assert list(gids) == sorted(gids)
        kept = e.rows(k)
        pruned = np.setdiff1d(np.arange(64), kept)
        # pruned rows hand their residual on bit-for-bit; kept rows obey |e| <= s/2
        assert np.array_equal(res[k - 1][pruned], prev[pruned])
        s = e.orders[k - 1].scales
        assert np.all(np.abs(res[k - 1][kept]) <= s[:, None] / 2 * (1 + 1e-6) + 1e-30)
        prev = res[k - 1]
    # the sparse expansion never does worse than stopping at order 1 and never
    # better than the dense one of the same order
    d = po.expand(W, bits, K, 1.0, G)
    err = lambda ex: np.linalg.norm(W - ex.reconstruct())
    assert err(d) <= err(e) <= np.linalg.norm(W - e.reconstruct(1))


def test_mask_is_energy_optimal_by_enumeration():
    """Tiny layers: enumerate every mask with n_keep groups; the chosen one removes
    the most residual energy (energy computed here from the residual itself)."""
    for seed, (O, G, gamma) in enumerate([(8, 2, 0.5), (6, 1, 0.34), (8, 2, 0.25), (10, 2, 0.6)]):
        W = _rand_w(30 + seed, O, 12, heavy=True)
        res = []
        e = po.expand(W, 4, 2, gamma, G, residuals=res)
        n_g = O // G
        keep = math.ceil(gamma * n_g - 1e-9)
        assert len(e.orders[1].group_ids) == keep == po.n_keep(gamma, n_g)
        E2 = (W.astype(np.float64) - e.reconstruct(1))
        energy = [float((E2[g * G:(g + 1) * G] ** 2).sum()) for g in range(n_g)]
        best = max(itertools.combinations(range(n_g), keep), key=lambda c: sum(energy[g] for g in c))
        assert sorted(best) == e.orders[1].group_ids.tolist()


# ---------------------------------------------------------------- unstructured masks (Sec. 3.1)
@pytest.mark.parametrize("bits", [8, 4, 2])
def test_unstructured_mask_structure(bits):
    """Orders k >= 2 keep exactly ceil(gamma * O * I) entries; pruned entries have code 0 and hand
    their residual on bit for bit; kept entries obey |e| <= s/2; every kept magnitude is at least
    every pruned one; gamma = 1 is the dense expansion."""
    W = _rand_w(40, 48, 72, heavy=True)
    K, gamma = 4, 0.3
    res, masks = [], []
    e = po.expand(W, bits, K, gamma, 16, residuals=res, masks=masks, mask="unstructured")
    keep = math.ceil(gamma * W.size - 1e-6)
    assert len(masks) == K - 1
    prev = res[0]
    for k in range(2, K + 1):
        M = masks[k - 2]
        assert M.sum() == keep
        o = e.orders[k - 1]
        assert o.group_ids.tolist() == list(range(3))            # every row is stored
        assert not np.any(o.codes[~M])
        assert np.array_equal(res[k - 1][~M], prev[~M])
        assert np.all(np.abs(res[k - 1])[M] <= (o.scales[:, None] / 2 * (1 + 1e-6) + 1e-30 + 0 * prev)[M])
        assert np.abs(prev)[M].min() >= np.abs(prev)[~M].max()
        # the scale of a row is its largest kept magnitude over q_max (independent quantizer)
        amax = np.where(M, np.abs(prev), 0).max(axis=1)
        assert np.array_equal(o.scales, (amax / f32(po.q_max(bits))).astype(f32))
        prev = res[k - 1]
    d = po.expand(W, bits, K, 1.0, 16)
    u1 = po.expand(W, bits, K, 1.0, 16, mask="unstructured")
    for k in range(K):
        assert np.array_equal(d.orders[k].codes, u1.orders[k].codes)
        assert np.array_equal(d.orders[k].scales, u1.orders[k].scales)
    assert np.array_equal(e.orders[0].codes, d.orders[0].codes)      # R^1 is dense either way


def test_unstructured_mask_by_enumeration_and_ties():
    """Tiny layers: of all masks with n_keep entries the chosen one keeps the most residual
    magnitude; among equal magnitudes the lower flat index wins."""
    for seed, (O, I, gamma) in enumerate([(2, 5, 0.5), (3, 4, 0.34), (2, 6, 0.25)]):
        W = _rand_w(50 + seed, O, I, heavy=True)
        masks = []
        e = po.expand(W, 4, 2, gamma, 1, masks=masks, mask="unstructured")
        E2 = np.abs(W.astype(np.float64) - e.reconstruct(1)).ravel()
        keep = po.n_keep(gamma, O * I)
        best = max(itertools.combinations(range(O * I), keep), key=lambda c: sum(E2[i] for i in c))
        assert sorted(best) == np.flatnonzero(masks[0].ravel()).tolist()
    E = np.array([[0.5, -0.25, 0.25], [0.25, -0.5, 0.125]], dtype=f32)
    assert np.flatnonzero(po.select_entries(E, 3).ravel()).tolist() == [0, 1, 4]     # first of the three 0.25s
    assert np.flatnonzero(po.select_entries(E, 4).ravel()).tolist() == [0, 1, 2, 4]
    assert po.select_entries(E, 6).all() and po.select_entries(E, 1).ravel().tolist() == [True] + [False] * 5


@pytest.mark.parametrize("bits", [8, 4, 2])
def test_unstructured_expansion_beats_the_dense_one_at_equal_budget(bits):
    """Sec. 3.1: at a matched budget of operations the sparse expansion is closer to the
    weights than the standard one.  Budget of two dense orders: K = 3 with half the entries kept
    in orders 2 and 3, against the dense K = 2."""
    for seed, heavy in [(60, False), (61, True)]:
        W = _rand_w(seed, 64, 96, heavy=heavy)
        dense2 = po.expand(W, bits, 2, 1.0, 16)
        sparse3 = po.expand(W, bits, 3, 0.5, 16, mask="unstructured")
        stored = sum(int(np.count_nonzero(sparse3.dense_codes(k))) for k in (2, 3))
        assert stored <= W.size                                       # no more entries than one dense order
        assert np.linalg.norm(W - sparse3.reconstruct()) < np.linalg.norm(W - dense2.reconstruct())


def test_n_keep_rounding():
    assert po.n_keep(0.25, 172) == 43 and po.n_keep(0.5, 344) == 172
    assert po.n_keep(0.5, 16) == 8 and po.n_keep(0.5, 96) == 48 and po.n_keep(0.5, 24) == 12
    assert po.n_keep(0.3, 10) == 3 and po.n_keep(0.31, 10) == 4 and po.n_keep(1.0, 7) == 7
    assert po.n_keep(0.01, 10) == 1


# ---------------------------------------------------------------- integer contraction
@pytest.mark.parametrize("a", [8, 6, 4])
def test_asymmetric_activation_codes(a):
    """The affine quantizer: every code is the nearest grid point (exhaustive search over the
    2^a codes), zero is represented exactly, in-range values are off by at most s/2, and a
    non-negative tensor gets a grid twice as fine as the symmetric one."""
    rng = np.random.default_rng(70 + a)
    x = (rng.standard_normal((5, 40)) * 1.7 + 0.6).astype(f32)
    x[0, 0] = 0.0
    Q, s, z = po.quantize_activations_asymmetric(x, a)
    qa = 2 ** a - 1
    assert Q.min() >= 0 and Q.max() <= qa and 0 <= z <= qa
    grid = (np.arange(qa + 1) - z).astype(np.float64) * float(s)
    best = np.abs(x.astype(np.float64)[..., None] - grid).min(axis=-1)
    mine = np.abs(x.astype(np.float64) - (Q.astype(np.float64) - z) * float(s))
    assert np.all(mine <= best + 1e-6 * float(s))                      # nearest code (ties aside)
    assert Q[0, 0] == z                                                # zero is exact
    inside = (x >= grid[0]) & (x <= grid[-1])
    assert np.all(mine[inside] <= float(s) / 2 * (1 + 1e-5))
    assert abs(float(s) - float(x.max() - x.min()) / qa) <= 1e-6 * float(s)
    r = np.maximum(x, 0)                                               # after a ReLU
    Qr, sr, zr = po.quantize_activations_asymmetric(r, a)
    _, ss = po.quantize_activations(r, None, a)
    assert zr == 0 and abs(float(sr) / float(ss) - (2 ** (a - 1) - 1) / qa) < 1e-6
    Q0, s0, z0 = po.quantize_activations_asymmetric(np.zeros((2, 3), f32), a)
    assert not Q0.any() and s0 == 0 and z0 == 0


def test_asymmetric_forward_is_the_textbook_affine_layer():
    """K = 1: the integer layer on (Q(x) - z) by an independent int64 einsum; shifting the codes by
    any constant c and adding c * (row sums of the weight codes) back gives the same accumulators
    (the identity a kernel with signed 8-bit operands relies on); with 8-bit weights and K = 3 the
    output converges to s * (Q(x) - z) W^T."""
    rng = np.random.default_rng(75)
    W = _rand_w(76, 32, 48)
    x = np.maximum(rng.standard_normal((9, 48)), 0).astype(f32) * 2.0
    e = po.expand(W, 4, 1, 1.0, 16)
    r = po.forward_asymmetric(e, x)
    Qc = r["Qx"].astype(np.int64) - r["z"]
    ref = np.einsum("ti,oi->to", Qc, e.orders[0].codes.astype(np.int64))
    assert np.array_equal(r["acc"][0], ref)
    c = 128 - r["z"]
    shifted = np.einsum("ti,oi->to", r["Qx"].astype(np.int64) - 128, e.orders[0].codes.astype(np.int64))
    assert np.array_equal(shifted + c * e.orders[0].codes.astype(np.int64).sum(axis=1)[None, :], ref)
    y = float(r["s_x"]) * (e.orders[0].scales.astype(np.float64)[None, :] * ref)
    assert np.allclose(r["y64"], y, rtol=1e-12, atol=0)
    e8 = po.expand(W, 8, 3, 1.0, 16)
    r8 = po.forward_asymmetric(e8, x, split=[1, 2])
    full = float(r8["s_x"]) * ((r8["Qx"].astype(np.float64) - r8["z"]) @ W.astype(np.float64).T)
    assert np.abs(r8["y64"] - full).max() <= 1e-5 * np.abs(full).max()
    # and the affine codes halve the input error of the symmetric ones on a non-negative tensor
    es = po.forward(e8, x)
    exact = x.astype(np.float64) @ W.astype(np.float64).T
    assert np.abs(r8["y64"] - exact).mean() < 0.75 * np.abs(es["y64"] - exact).mean()


def test_asymmetric_conv_is_torch_conv_on_centred_codes():
    """The asymmetric conv layer: accumulators equal torch's conv2d (fp64, exact on these integers)
    of Q(x) - z with zero padding, and on a post-ReLU input the layer is closer to the
    full-precision convolution than with symmetric codes."""
    rng = np.random.default_rng(78)
    C, O, H = 8, 16, 7
    W4 = (rng.standard_normal((O, C, 3, 3)) * 0.2).astype(f32)
    x = np.maximum(rng.standard_normal((2, C, H, H)), 0).astype(f32)
    e = po.expand(W4.reshape(O, -1), 8, 2, 1.0, 16)
    for stride, pad in [(1, 1), (2, 0)]:
        r = po.forward_conv2d_asymmetric(e, x, 3, 3, stride, pad)
        Qc = torch.from_numpy((r["Qx"].astype(np.int64) - r["z"]).astype(np.float64))
        for k in range(2):
            wk = torch.from_numpy(e.orders[k].codes.astype(np.float64).reshape(O, C, 3, 3))
            ref = torch.nn.functional.conv2d(Qc, wk, stride=stride, padding=pad).permute(0, 2, 3, 1).reshape(-1, O)
            assert np.array_equal(r["acc"][k], ref.numpy().astype(np.int64))
        full = torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64)), torch.from_numpy(W4.astype(np.float64)),
                                          stride=stride, padding=pad).permute(0, 2, 3, 1).reshape(-1, O).numpy()
        sym = po.forward_conv2d(e, x, 3, 3, stride, pad)
        assert np.abs(r["y64"] - full).mean() < 0.75 * np.abs(sym["y64"] - full).mean()


def test_contraction_against_torch_int64_and_loops():
    rng = np.random.default_rng(40)
    Qx = rng.integers(-127, 128, size=(7, 333), dtype=np.int8)
    q = rng.integers(-127, 128, size=(11, 333), dtype=np.int8)
    got = po.contract(Qx, q)
    ref = (torch.from_numpy(Qx).to(torch.int64) @ torch.from_numpy(q).to(torch.int64).T).numpy()
    assert got.dtype == np.int32 and np.array_equal(got, ref)
    for t, r in [(0, 0), (3, 5), (6, 10)]:
        assert int(got[t, r]) == sum(int(Qx[t, i]) * int(q[r, i]) for i in range(333))
    ones = po.contract(np.ones((2, 500), np.int8), np.ones((3, 500), np.int8))
    assert np.all(ones == 500)
    # worst case magnitude at the largest in_features of the configs stays exact
    big = po.contract(np.full((1, 11008), 127, np.int8), np.full((1, 11008), -127, np.int8))
    assert int(big[0, 0]) == -127 * 127 * 11008


def test_k1_forward_is_textbook_quantized_linear():
    """One int8 order: y = s_x * s_w[o] * sum_i Qx*Qw, recomputed with Python ints."""
    W = _rand_w(41, 5, 24)
    x = np.random.default_rng(42).standard_normal((3, 24)).astype(f32)
    e = po.expand(W, 8, 1, 1.0, 1)
    r = po.forward(e, x)
    sx = float(np.abs(x).max() / f32(127))
    for t in range(3):
        for o in range(5):
            sw = float(np.abs(W[o]).max() / f32(127))
            acc = sum(int(round(float(x[t, i]) / sx)) * int(round(float(W[o, i]) / sw)) for i in range(24))
            assert int(r["acc"][0, t, o]) == acc
            assert math.isclose(float(r["y"][t, o]), sx * sw * acc, rel_tol=1e-5, abs_tol=1e-7)


def test_forward_converges_to_full_precision_weights():
    """int8, K = 4, dense: the expansion reproduces W to ~(1/254)^3, so the output
    equals s_x * Qx W^T (fp64) down to fp32 resolution; lower orders converge at
    the Lemma's rate."""
    W = _rand_w(43, 24, 128)
    x = np.random.default_rng(44).standard_normal((9, 128)).astype(f32)
    prev = None
    for K in (1, 2, 3, 4):
        e = po.expand(W, 8, K, 1.0, 8)
        r = po.forward(e, x)
        target = float(r["s_x"]) * (r["Qx"].astype(np.float64) @ W.astype(np.float64).T)
        err = np.abs(r["y64"] - target).max() / np.abs(target).max()
        if prev is not None:
            # geometric decrease until the fp32 rounding of the residuals (~2^-24) is reached
            assert err < max(prev / 50, 2e-7)
        prev = err
    assert prev < 2e-7
    assert np.abs(r["y"] - target).max() <= 1e-5 * np.abs(target).max()


# ---------------------------------------------------------------- ensemble members (Sec. 3.2)
def test_single_layer_ensemble_is_exact_partition():
    W = _rand_w(50, 32, 64, heavy=True)
    x = np.random.default_rng(51).standard_normal((5, 64)).astype(f32)
    b = np.random.default_rng(52).standard_normal(32).astype(f32)
    e = po.expand(W, 4, 4, 0.5, 8)
    full = po.forward(e, x, bias=b)
    for split in ([2, 2], [1, 3], [1, 1, 2], [1, 1, 1, 1]):
        ens = po.forward(e, x, split=split, bias=b)
        assert np.array_equal(ens["acc"], full["acc"])          # accumulators ignore the split
        assert np.allclose(ens["y64"], full["y64"], rtol=1e-12, atol=1e-12)   # linearity
        assert np.allclose(ens["y"], full["y"], rtol=1e-5, atol=1e-6)
        mem = po.forward(e, x, split=split, bias=b, reduce_members=False)
        assert mem["y"].shape == (len(split), 5, 32)
    with pytest.raises(ValueError):
        po.forward(e, x, split=[2, 1])


def test_bias_only_in_first_member():
    W = _rand_w(53, 16, 32)
    x = np.random.default_rng(54).standard_normal((4, 32)).astype(f32)
    b = np.arange(16, dtype=f32)
    e = po.expand(W, 4, 2, 1.0, 4)
    with_b = po.forward(e, x, split=[1, 1], bias=b, reduce_members=False)["y"]
    no_b = po.forward(e, x, split=[1, 1], reduce_members=False)["y"]
    assert np.allclose(with_b[0] - no_b[0], b[None, :], atol=1e-5)
    assert np.array_equal(with_b[1], no_b[1])
    # a member whose weights are all zero outputs exactly 0, bias or not
    z = po.expand(np.zeros((16, 32), f32), 4, 2, 1.0, 4)
    out = po.forward(z, x, split=[1, 1], bias=b, reduce_members=False)["y"]
    assert np.array_equal(out[0], np.broadcast_to(b, (4, 16))) and not out[1].any()


# ---------------------------------------------------------------- convolution
def test_conv_direct_equals_im2col_and_torch():
    rng = np.random.default_rng(60)
    for (N, C, H, Wd, O, kh, kw, stride, pad) in [(2, 3, 6, 5, 4, 3, 3, 1, 1), (1, 2, 7, 7, 3, 3, 2, 2, 0),
                                                   (2, 5, 8, 6, 4, 1, 1, 2, 0), (1, 3, 13, 11, 4, 7, 7, 2, 3)]:
        Qx = rng.integers(-127, 128, size=(N, C, H, Wd), dtype=np.int8)
        q = rng.integers(-7, 8, size=(O, C * kh * kw), dtype=np.int8)
        direct = po.conv2d_acc_direct(Qx, q, kh, kw, stride, pad)
        gemm = po.contract(po.im2col(Qx, kh, kw, stride, pad), q)
        assert np.array_equal(direct, gemm)
        ref = torch.nn.functional.conv2d(torch.from_numpy(Qx).double(),
                                         torch.from_numpy(q).double().reshape(O, C, kh, kw),
                                         stride=stride, padding=pad)
        ref = ref.permute(0, 2, 3, 1).reshape(-1, O).numpy()
        assert np.array_equal(direct.astype(np.float64), ref)


def test_conv_forward_matches_linear_on_im2col():
    w = wl.scaled(wl.C2, out_div=8, in_div=32, tokens=196)
    spec, c = w.layers[0], w.conv
    W, x = wl.make_weight(w, 0), wl.make_input(w)
    e = po.expand(W, spec.bits, spec.K, spec.gamma, spec.group)
    conv = po.forward_conv2d(e, x, c["kh"], c["kw"], c["stride"], c["pad"], split=list(w.split))
    cols = po.im2col(x, c["kh"], c["kw"], c["stride"], c["pad"])
    lin = po.forward(e, cols, split=list(w.split))
    assert np.array_equal(conv["acc"], lin["acc"]) and np.array_equal(conv["y"], lin["y"])


def test_depthwise_against_torch_grouped_conv():
    """Depthwise accumulators equal torch's grouped conv2d (groups = C) on the integer codes, and
    the expanded depthwise layer converges to the full-precision depthwise conv."""
    rng = np.random.default_rng(66)
    for (N, C, H, Wd, kh, kw, stride, pad) in [(2, 5, 7, 6, 3, 3, 1, 1), (1, 4, 9, 9, 3, 3, 2, 1), (2, 3, 11, 8, 5, 5, 2, 2)]:
        Qx = rng.integers(-127, 128, size=(N, C, H, Wd), dtype=np.int8)
        q = rng.integers(-7, 8, size=(C, kh * kw), dtype=np.int8)
        got = po.depthwise_acc_direct(Qx, q, kh, kw, stride, pad)
        ref = torch.nn.functional.conv2d(torch.from_numpy(Qx).double(), torch.from_numpy(q).double().reshape(C, 1, kh, kw),
                                         stride=stride, padding=pad, groups=C)
        assert np.array_equal(got.astype(np.float64), ref.permute(0, 2, 3, 1).reshape(-1, C).numpy())
    C, kh, kw = 16, 3, 3
    W = rng.standard_normal((C, kh * kw)).astype(f32)
    x = rng.standard_normal((2, C, 8, 8)).astype(f32)
    b = rng.standard_normal(C).astype(f32)
    e = po.expand(W, 8, 3, 1.0, 8)
    r = po.forward_depthwise2d(e, x, kh, kw, 1, 1, bias=b, split=[2, 1])
    full = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(W).double().reshape(C, 1, kh, kw),
                                      torch.from_numpy(b).double(), padding=1, groups=C)
    full = full.permute(0, 2, 3, 1).reshape(-1, C).numpy()
    assert np.abs(r["y"] - full).max() < 0.02 * np.abs(full).max()      # the int8 activation grid is all that is left
    parts = po.forward_depthwise2d(e, x, kh, kw, 1, 1, bias=b, split=[2, 1], reduce_members=False)["y"]
    assert np.array_equal(r["y"], (parts[0] + parts[1]).astype(f32))


def test_batchnorm_fold_equals_conv_then_batchnorm():
    """The folded layer computes what torch's conv2d followed by batch_norm (inference mode)
    computes, for a conv and for a fully-connected layer, with and without a bias."""
    rng = np.random.default_rng(65)
    O, C, kh, kw = 6, 3, 3, 3
    Wc = rng.standard_normal((O, C * kh * kw)).astype(f32)
    x = rng.standard_normal((2, C, 7, 5)).astype(f32)
    gamma, beta = (1 + 0.3 * rng.standard_normal(O)).astype(f32), rng.standard_normal(O).astype(f32)
    mean, var = rng.standard_normal(O).astype(f32), (0.5 + rng.random(O)).astype(f32)
    for b in (None, rng.standard_normal(O).astype(f32)):
        Wf, bf = po.fold_batchnorm(Wc, b, gamma, beta, mean, var, 1e-5)
        t = lambda a: torch.from_numpy(np.asarray(a)).double()
        z = torch.nn.functional.conv2d(t(x), t(Wc).reshape(O, C, kh, kw), None if b is None else t(b), padding=1)
        ref = torch.nn.functional.batch_norm(z, t(mean), t(var), t(gamma), t(beta), False, 0.0, 1e-5)
        got = torch.nn.functional.conv2d(t(x), t(Wf).reshape(O, C, kh, kw), t(bf), padding=1)
        assert torch.allclose(got, ref, rtol=1e-5, atol=1e-5)
    # identity statistics leave the layer alone
    Wi, bi = po.fold_batchnorm(Wc, None, np.ones(O, f32), np.zeros(O, f32), np.zeros(O, f32), np.ones(O, f32), 0.0)
    assert np.array_equal(Wi, Wc) and not bi.any()


# ---------------------------------------------------------------- MLP ensemble
def test_mlp_single_member_is_plain_composition():
    rng = np.random.default_rng(70)
    W1, W2 = _rand_w(71, 32, 24), _rand_w(72, 8, 32)
    x = rng.standard_normal((6, 24)).astype(f32)
    e1, e2 = po.expand(W1, 4, 2, 1.0, 8), po.expand(W2, 4, 2, 1.0, 8)
    out = po.mlp_forward(e1, e2, "gelu", x)
    h = po.forward(e1, x)["y"]
    # GELU pinned to torch's erf form (independent library routine)
    g = torch.nn.functional.gelu(torch.from_numpy(h).double()).numpy()
    assert np.allclose(out["h"][0], g, rtol=1e-6, atol=1e-7)
    y = po.forward(e2, out["h"][0])["y"]
    assert np.array_equal(out["y"], y)
    # gated: SiLU pinned to torch
    W1g = _rand_w(73, 64, 24)
    e1g = po.expand(W1g, 4, 2, 1.0, 8)
    og = po.mlp_forward(e1g, e2, "gated", x)
    y1 = po.forward(e1g, x)["y"]
    hg = (torch.nn.functional.silu(torch.from_numpy(y1[:, :32]).double())
          * torch.from_numpy(y1[:, 32:]).double()).numpy()
    assert np.allclose(og["h"][0], hg, rtol=1e-6, atol=1e-8)


def test_mlp_ensemble_members_use_only_their_orders():
    """Member 2 of split [1,1] must equal a network built from R^2 alone, without
    biases; with a ReLU-like regime (large positive pre-activations) the ensemble
    approaches the full expansion as the paper's approximation states."""
    rng = np.random.default_rng(74)
    W1, W2 = _rand_w(75, 32, 24), _rand_w(76, 8, 32)
    x = rng.standard_normal((6, 24)).astype(f32)
    b1 = rng.standard_normal(32).astype(f32)
    e1, e2 = po.expand(W1, 4, 2, 1.0, 8), po.expand(W2, 4, 2, 1.0, 8)
    out = po.mlp_forward(e1, e2, "gelu", x, split=[1, 1], bias1=b1)
    # rebuild member 2 by hand from the order-2 terms only
    Qx, sx = po.quantize_activations(x)
    y1 = f32(sx) * (e1.dense_scales(2)[None, :] * po.contract(Qx, e1.dense_codes(2)).astype(f32))
    h = po.gelu(y1)
    Qh, sh = po.quantize_activations(h)
    y2 = f32(sh) * (e2.dense_scales(2)[None, :] * po.contract(Qh, e2.dense_codes(2)).astype(f32))
    assert np.allclose(out["members"][1], y2, rtol=1e-6, atol=1e-9)
    assert np.array_equal(out["y"], (out["members"][0] + out["members"][1]).astype(f32))
    full = po.mlp_forward(e1, e2, "gelu", x, bias1=b1)["y"]
    assert np.abs(out["y"] - full).max() < 0.15 * np.abs(full).max()


# ---------------------------------------------------------------- L-layer member chains
def _frac(v):
    from fractions import Fraction
    return float(Fraction(v))


def test_chain_worked_example(golden_dir):
    """Two small networks worked in exact rationals from App. B: pins the member-wise skip,
    the first-member-only bias and input skip, the per-member dynamic activation scales
    and the sum after the last layer."""
    g = json.load(open(os.path.join(golden_dir, "chain_worked.json")))
    exps = {}
    for name in ("W0", "W1", "W2"):
        e = po.expand(np.array(g[name], dtype=f32), g["bits"], g["K"], 1.0, 1)
        for k in range(g["K"]):
            assert e.orders[k].codes.tolist() == g["expansion"][name]["codes"][k], (name, k)
            want = [_frac(v) for v in g["expansion"][name]["scales"][k]]
            assert np.allclose(e.orders[k].scales, want, rtol=1e-6, atol=0), (name, k)
        exps[name] = e
    x = np.array(g["x"], dtype=f32)
    bias = {"W0": np.array(g["b0"], dtype=f32), "W1": None, "W2": np.array(g["b2"], dtype=f32)}
    for case, names in (("case_A", ("W0", "W1", "W2")), ("case_B", ("W0", "W1"))):
        c = g[case]
        layers = [po.ChainLayer(exps[n], bias[n], d["act"], d["skip_from"], d.get("skip_pre_act", True))
                  for n, d in zip(names, c["layers"])]
        r = po.chain_forward(layers, x, split=g["split"])
        for m, key in enumerate(("member_1", "member_2")):
            mm = c[key]
            assert np.allclose(r["acts"][0][m][0], [_frac(v) for v in mm["a1"]], rtol=1e-5, atol=1e-9), (case, key)
            Qa, _ = po.quantize_activations(r["acts"][0][m])
            assert Qa[0].tolist() == mm["Q_a1"], (case, key)
            if "a2" in mm:
                assert np.allclose(r["acts"][1][m][0], [_frac(v) for v in mm["a2"]], rtol=1e-5, atol=1e-9)
                Qa, _ = po.quantize_activations(r["acts"][1][m])
                assert Qa[0].tolist() == mm["Q_a2"], (case, key)
            assert np.allclose(r["members"][m][0], [_frac(v) for v in mm["y"]], rtol=1e-5, atol=1e-9), (case, key)
        assert np.allclose(r["y"][0], [_frac(v) for v in c["y"]], rtol=1e-5, atol=1e-9), case


def _chain_net(seed, widths, K, bits, skips, acts):
    rng = np.random.default_rng(seed)
    layers, Ws, bs = [], [], []
    for l in range(len(widths) - 1):
        W = (rng.standard_normal((widths[l + 1], widths[l])) / math.sqrt(widths[l])).astype(f32)
        b = (3.0 * rng.standard_normal(widths[l + 1])).astype(f32)
        Ws.append(W)
        bs.append(b)
        sf, pre = skips[l]
        layers.append(po.ChainLayer(po.expand(W, bits, K, 1.0, 8), b, acts[l], sf, pre))
    return layers, Ws, bs


def _float_net(Ws, bs, skips, acts, x):
    """The full-precision network the chain expands, in fp64 (textbook forward pass)."""
    tensors = [x.astype(np.float64)]
    for l, (W, b) in enumerate(zip(Ws, bs)):
        z = tensors[l] @ W.astype(np.float64).T + b
        sf, pre = skips[l]
        r = tensors[sf] if sf >= 0 else 0.0
        if pre:
            z = z + r
        if acts[l] == "relu":
            z = np.maximum(z, 0.0)
        elif acts[l] == "gelu":
            z = torch.nn.functional.gelu(torch.from_numpy(z)).numpy()
        if not pre:
            z = z + r
        tensors.append(z)
    return tensors


@pytest.mark.parametrize("split", [None, [2, 2], [1, 1, 2]])
def test_chain_converges_to_the_full_precision_network(split):
    """With 8-bit orders and K = 4 the expansion is the full-precision weight to ~1e-7, so the
    chain must reproduce the fp64 network up to the int8 activation grid (~1 % of a layer's
    range).  Biases three times the pre-activations and skips from the input and from hidden
    tensors make any misplaced bias or skip (all members, wrong tensor, wrong side of the
    activation) an error many times that."""
    widths = [24, 32, 32, 32, 16]
    skips = [(-1, True), (1, True), (0, False), (-1, True)]
    skips[2] = (2, False)
    acts = ["relu", "relu", "gelu", "none"]
    layers, Ws, bs = _chain_net(80, widths, 4, 8, skips, acts)
    rng = np.random.default_rng(81)
    x = (4.0 * rng.standard_normal((7, 24))).astype(f32)
    ref = _float_net(Ws, bs, skips, acts, x)
    r = po.chain_forward(layers, x, split=split)
    for l in range(3):
        tot = r["acts"][l].astype(np.float64).sum(axis=0)
        assert np.abs(tot - ref[l + 1]).max() < 0.03 * np.abs(ref[l + 1]).max(), l
    assert np.abs(r["y"] - ref[4]).max() < 0.03 * np.abs(ref[4]).max()
    # the same with the first layer skipping from the network input itself
    widths2 = [32, 32, 16]
    skips2 = [(0, True), (-1, True)]
    acts2 = ["relu", "none"]
    layers2, Ws2, bs2 = _chain_net(82, widths2, 4, 8, skips2, acts2)
    x2 = (4.0 * rng.standard_normal((7, 32))).astype(f32)
    ref2 = _float_net(Ws2, bs2, skips2, acts2, x2)
    r2 = po.chain_forward(layers2, x2, split=split)
    assert np.abs(r2["y"] - ref2[2]).max() < 0.03 * np.abs(ref2[2]).max()


def test_chain_single_member_is_layer_by_layer_forward():
    """M = 1: the chain is the pinned single-layer forward applied L times with the
    activation and the skip between (written out here for one fixed architecture)."""
    skips = [(-1, True), (1, True), (-1, True)]
    acts = ["relu", "relu", "none"]
    layers, _, bs = _chain_net(83, [24, 32, 32, 8], 2, 4, skips, acts)
    x = np.random.default_rng(84).standard_normal((5, 24)).astype(f32)
    r = po.chain_forward(layers, x)
    a1 = np.maximum(po.forward(layers[0].exp, x, bias=bs[0])["y"], 0)
    a2 = np.maximum((po.forward(layers[1].exp, a1, bias=bs[1])["y"] + a1).astype(f32), 0)
    y = po.forward(layers[2].exp, a2, bias=bs[2])["y"]
    assert np.array_equal(r["acts"][0][0], a1) and np.array_equal(r["acts"][1][0], a2)
    assert np.array_equal(r["y"], y)
    # two layers with GELU between: the pinned MLP routine
    l2 = [po.ChainLayer(layers[0].exp, bs[0], "gelu"), po.ChainLayer(layers[1].exp, bs[1], "none")]
    m = po.mlp_forward(layers[0].exp, layers[1].exp, "gelu", x, split=[1, 1], bias1=bs[0], bias2=bs[1])
    c = po.chain_forward(l2, x, split=[1, 1])
    assert np.array_equal(c["y"], m["y"]) and np.array_equal(c["acts"][0], m["h"])


def test_chain_with_given_scales_is_the_pinned_layer_with_its_static_scale():
    """Static activation ranges inside a chain: layer l quantizes member m's tensor with the given scale
    s_in[m] instead of max|tensor|/127 -- written out with the pinned single-layer routine and its s_x."""
    skips = [(-1, True), (1, True), (-1, True)]
    acts = ["relu", "relu", "none"]
    layers, _, bs = _chain_net(92, [24, 32, 32, 8], 2, 4, skips, acts)
    x = np.random.default_rng(93).standard_normal((5, 24)).astype(f32)
    layers[1].s_in = [0.05]
    layers[2].s_in = [0.11]
    r = po.chain_forward(layers, x, s_x=0.03)
    a1 = np.maximum(po.forward(layers[0].exp, x, s_x=0.03, bias=bs[0])["y"], 0)
    a2 = np.maximum((po.forward(layers[1].exp, a1, s_x=0.05, bias=bs[1])["y"] + a1).astype(f32), 0)
    y = po.forward(layers[2].exp, a2, s_x=0.11, bias=bs[2])["y"]
    assert np.array_equal(r["acts"][0][0], a1) and np.array_equal(r["acts"][1][0], a2) and np.array_equal(r["y"], y)
    # a scale too small clips at +-127: the result differs from the dynamic one
    assert not np.array_equal(r["y"], po.chain_forward([po.ChainLayer(l.exp, l.bias, l.act, l.skip_from, l.skip_pre_act) for l in layers], x, s_x=0.03)["y"])
    # two members: each with its own given scale; with the scales the dynamic run found, nothing changes
    dyn = po.chain_forward([po.ChainLayer(l.exp, l.bias, l.act, l.skip_from, l.skip_pre_act) for l in layers], x, split=[1, 1])
    found = [[float(np.abs(dyn["acts"][l][m]).max()) / 127.0 for m in range(2)] for l in range(2)]
    given = [po.ChainLayer(l.exp, l.bias, l.act, l.skip_from, l.skip_pre_act, s_in=None if i == 0 else [f32(f32(np.abs(dyn["acts"][i - 1][m]).max()) / f32(127)) for m in range(2)])
             for i, l in enumerate(layers)]
    same = po.chain_forward(given, x, split=[1, 1])
    assert np.array_equal(same["y"], dyn["y"]) and found[0][1] < found[0][0]


def test_mlp_with_given_hidden_scales_is_the_chain_with_given_scales():
    """pipe_mlp_forward's static form: with GELU it is the two-layer chain whose second layer has s_in (pinned
    above); gated, member m's last layer is the pinned single layer with s_x = s_h[m]."""
    rng = np.random.default_rng(94)
    I, H, O, T = 24, 32, 16, 6
    W1 = (rng.standard_normal((2 * H, I)) / math.sqrt(I)).astype(f32)
    W2 = (rng.standard_normal((O, H)) / math.sqrt(H)).astype(f32)
    x = rng.standard_normal((T, I)).astype(f32)
    e1, e2, e1g = po.expand(W1, 4, 2, 1.0, 8), po.expand(W2, 4, 2, 1.0, 8), po.expand(W1[:H], 4, 2, 1.0, 8)
    m2 = po.mlp_forward(e1g, e2, "gelu", x, split=[1, 1], s_x=0.03, s_h=[0.02, 0.004])
    c2 = po.chain_forward([po.ChainLayer(e1g, None, "gelu"), po.ChainLayer(e2, None, "none", s_in=[0.02, 0.004])], x, split=[1, 1], s_x=0.03)
    assert np.array_equal(m2["y"], c2["y"])
    r = po.mlp_forward(e1, e2, "gated", x, split=[1, 1], s_x=0.03, s_h=[0.05, 0.01])
    for m in range(2):
        one2 = po.expand((e2.dense_scales(m + 1)[:, None] * e2.dense_codes(m + 1)).astype(f32), 4, 1, 1.0, 8)
        assert np.allclose(r["members"][m], po.forward(one2, r["h"][m], s_x=[0.05, 0.01][m])["y"], rtol=1e-5, atol=1e-7)


def test_chain_members_are_independent_networks():
    """Member 2 of split [1,1] equals a network built from the order-2 terms alone, with no
    bias anywhere, fed the same input; member 1 does not change when order 2 is altered."""
    skips = [(-1, True), (1, True), (-1, True)]
    acts = ["relu", "relu", "none"]
    layers, _, bs = _chain_net(85, [24, 32, 32, 8], 2, 4, skips, acts)
    x = np.random.default_rng(86).standard_normal((5, 24)).astype(f32)
    r = po.chain_forward(layers, x, split=[1, 1])

    def order2(e, a):
        Qa, sa = po.quantize_activations(a)
        return f32(sa) * (e.dense_scales(2)[None, :] * po.contract(Qa, e.dense_codes(2)).astype(f32))

    a1 = np.maximum(order2(layers[0].exp, x), 0)
    a2 = np.maximum((order2(layers[1].exp, a1) + a1).astype(f32), 0)
    y2 = order2(layers[2].exp, a2)
    assert np.allclose(r["acts"][1][1], a2, rtol=1e-6, atol=1e-9)
    assert np.allclose(r["members"][1], y2, rtol=1e-6, atol=1e-9)
    assert np.array_equal(r["y"], (r["members"][0] + r["members"][1]).astype(f32))
    one = po.chain_forward([po.ChainLayer(po.expand(
        (ly.exp.dense_scales(1)[:, None] * ly.exp.dense_codes(1)).astype(f32), 4, 1, 1.0, 8), ly.bias, ly.act,
        ly.skip_from, ly.skip_pre_act) for ly in layers], x)
    assert np.allclose(r["members"][0], one["y"], rtol=1e-5, atol=1e-7)


def test_asymmetric_chain_is_the_pinned_asymmetric_layer_applied_member_wise():
    """Asymmetric codes in front of every layer of a chain (Sec. 4.3).  One member: the pinned
    single-layer routine applied L times with activation and skip between.  Two members: member 2
    is the network of the order-2 terms alone on codes minus their zero point (written out with an
    int64 einsum and the quantizer's own outputs), it carries no bias, and the sum is the members'."""
    skips = [(-1, True), (1, True), (-1, True)]
    acts = ["relu", "relu", "none"]
    layers, _, bs = _chain_net(87, [24, 32, 32, 8], 2, 4, skips, acts)
    x = np.random.default_rng(88).standard_normal((5, 24)).astype(f32)
    r = po.chain_forward(layers, x, asymmetric=True)
    a1 = np.maximum(po.forward_asymmetric(layers[0].exp, x, bias=bs[0])["y"], 0)
    a2 = np.maximum((po.forward_asymmetric(layers[1].exp, a1, bias=bs[1])["y"] + a1).astype(f32), 0)
    y = po.forward_asymmetric(layers[2].exp, a2, bias=bs[2])["y"]
    assert np.array_equal(r["acts"][0][0], a1) and np.array_equal(r["acts"][1][0], a2)
    assert np.array_equal(r["y"], y)
    # after a ReLU the zero point is 0 and the codes span the whole range
    Q2, s2, z2 = po.quantize_activations_asymmetric(a1)
    assert z2 == 0 and Q2.max() == 255
    assert not np.array_equal(r["y"], po.chain_forward(layers, x)["y"])

    r2 = po.chain_forward(layers, x, split=[1, 1], asymmetric=True)

    def order2(e, a):
        Q, s, z = po.quantize_activations_asymmetric(a)
        acc = np.einsum("ti,oi->to", Q.astype(np.int64) - z, e.dense_codes(2).astype(np.int64))
        return f32(s) * (e.dense_scales(2)[None, :] * acc.astype(f32))

    b1 = np.maximum(order2(layers[0].exp, x), 0)
    b2 = np.maximum((order2(layers[1].exp, b1) + b1).astype(f32), 0)
    y2 = order2(layers[2].exp, b2)
    assert np.allclose(r2["acts"][1][1], b2, rtol=1e-6, atol=1e-9)
    assert np.allclose(r2["members"][1], y2, rtol=1e-6, atol=1e-9)
    assert np.array_equal(r2["y"], (r2["members"][0] + r2["members"][1]).astype(f32))
    with pytest.raises(ValueError):
        po.chain_forward(layers, x, s_x=0.1, asymmetric=True)


def test_asymmetric_mlp_is_the_pinned_layers_and_activation():
    """The two-layer ensemble under asymmetric codes: with GELU it is the asymmetric chain of two layers
    (pinned above); gated, member m is the pinned asymmetric layer (its own orders, bias in the first
    member), torch's SiLU times up, and the pinned asymmetric layer again on its own hidden tensor."""
    rng = np.random.default_rng(91)
    I, H, O, T = 24, 32, 16, 6
    W1 = (rng.standard_normal((2 * H, I)) / math.sqrt(I)).astype(f32)
    W2 = (rng.standard_normal((O, H)) / math.sqrt(H)).astype(f32)
    b1 = rng.standard_normal(2 * H).astype(f32)
    b2 = rng.standard_normal(O).astype(f32)
    x = (rng.standard_normal((T, I)) + 0.4).astype(f32)
    e1, e2 = po.expand(W1, 4, 2, 1.0, 8), po.expand(W2, 4, 2, 1.0, 8)
    r = po.mlp_forward(e1, e2, "gated", x, split=[1, 1], bias1=b1, bias2=b2, asymmetric=True)
    ys = []
    for m, sp in enumerate(([1], [1])):
        one1 = po.expand((e1.dense_scales(m + 1)[:, None] * e1.dense_codes(m + 1)).astype(f32), 4, 1, 1.0, 8)
        one2 = po.expand((e2.dense_scales(m + 1)[:, None] * e2.dense_codes(m + 1)).astype(f32), 4, 1, 1.0, 8)
        y1 = po.forward_asymmetric(one1, x, bias=b1 if m == 0 else None)["y"]
        g, u = torch.from_numpy(y1[:, :H].astype(np.float64)), torch.from_numpy(y1[:, H:].astype(np.float64))
        h = (torch.nn.functional.silu(g) * u).numpy().astype(f32)
        assert np.allclose(r["h"][m], h, rtol=2e-6, atol=1e-7)
        ys.append(po.forward_asymmetric(one2, r["h"][m], bias=b2 if m == 0 else None)["y"])
        assert np.allclose(r["members"][m], ys[m], rtol=1e-5, atol=1e-6)
    assert np.array_equal(r["y"], (r["members"][0] + r["members"][1]).astype(f32))
    # GELU: the chain of two layers
    W1g = W1[:H]
    e1g = po.expand(W1g, 4, 2, 1.0, 8)
    m2 = po.mlp_forward(e1g, e2, "gelu", x, split=[1, 1], bias1=b1[:H], bias2=b2, asymmetric=True)
    c2 = po.chain_forward([po.ChainLayer(e1g, b1[:H], "gelu"), po.ChainLayer(e2, b2, "none")], x, split=[1, 1], asymmetric=True)
    assert np.array_equal(m2["y"], c2["y"]) and np.array_equal(m2["h"], c2["acts"][0])
    with pytest.raises(ValueError):
        po.mlp_forward(e1, e2, "gated", x, s_x=0.1, asymmetric=True)


@pytest.mark.parametrize("a", [4, 6])
def test_asymmetric_chain_is_closer_to_the_float_network_after_relus(a):
    """Why the comparison of Sec. 4.3 is made under asymmetric quantization: a tensor that left a
    ReLU uses only half of a symmetric grid.  On a ReLU network with a-bit activations and an
    expansion that is exact to 1e-7 the asymmetric chain must be clearly closer to the fp64 network."""
    widths = [32, 48, 48, 16]
    skips = [(-1, True)] * 3
    acts = ["relu", "relu", "none"]
    layers, Ws, bs = _chain_net(89, widths, 4, 8, skips, acts)
    for ly in layers:
        ly.bias = (ly.bias / 6.0).astype(f32)
    bs = [ly.bias for ly in layers]
    x = np.abs(np.random.default_rng(90).standard_normal((64, 32))).astype(f32)   # e.g. the output of an earlier ReLU
    ref = _float_net(Ws, bs, skips, acts, x)[-1]
    e_sym = np.abs(po.chain_forward(layers, x, split=[2, 2], act_bits=a)["y"] - ref).mean()
    e_asym = np.abs(po.chain_forward(layers, x, split=[2, 2], act_bits=a, asymmetric=True)["y"] - ref).mean()
    assert e_asym < 0.7 * e_sym, (e_asym, e_sym)


def test_conv_chain_is_layer_by_layer_conv_and_converges_to_torch():
    """A residual conv stack as member chains: with one member it is the pinned conv forward
    applied layer by layer (ReLU, skip); with 8-bit orders it reproduces torch's fp64 ConvNet."""
    rng = np.random.default_rng(87)
    N, H, W, C = 2, 8, 8, 8
    geo = [(16, C, 3, 1, 1), (16, 16, 3, 1, 1), (16, 16, 3, 1, 1), (24, 16, 3, 2, 1), (16, 24, 1, 1, 0)]   # O, Cin, k, stride, pad
    Ws = [(rng.standard_normal((o, c * k * k)) * math.sqrt(2.0 / (c * k * k))).astype(f32) for o, c, k, _, _ in geo]
    bs = [(0.5 * rng.standard_normal(o)).astype(f32) for o, *_ in geo]
    acts = ["relu", "relu", "relu", "relu", "none"]
    skip = [-1, -1, 1, -1, -1]          # layer 2 adds the tensor that entered layer 1: a residual block
    x = rng.standard_normal((N, C, H, W)).astype(f32)
    xt = np.ascontiguousarray(x.transpose(0, 2, 3, 1)).reshape(N * H * W, C)

    def layers(bits, K):
        return [po.ChainLayer(po.expand(Wl, bits, K, 1.0, 8), b, a, sk, True, k, k, st, pd)
                for Wl, b, a, sk, (o, c, k, st, pd) in zip(Ws, bs, acts, skip, geo)]

    # one member, 4-bit: composition of the pinned single-layer conv forward
    L4 = layers(4, 2)
    r = po.chain_forward(L4, xt, grid=(N, H, W))
    to_nchw = lambda a, g: a.reshape(g[0], g[1], g[2], -1).transpose(0, 3, 1, 2)
    grids = po.chain_grids(L4, (N, H, W))
    a0 = np.maximum(po.forward_conv2d(L4[0].exp, x, 3, 3, 1, 1, bias=bs[0])["y"], 0)
    a1 = np.maximum(po.forward_conv2d(L4[1].exp, to_nchw(a0, grids[1]), 3, 3, 1, 1, bias=bs[1])["y"], 0)
    a2 = np.maximum((po.forward_conv2d(L4[2].exp, to_nchw(a1, grids[2]), 3, 3, 1, 1, bias=bs[2])["y"] + a0).astype(f32), 0)
    assert np.array_equal(r["acts"][0][0], a0) and np.array_equal(r["acts"][1][0], a1) and np.array_equal(r["acts"][2][0], a2)
    assert grids[-1] == (N, 4, 4) and r["y"].shape == (N * 16, 16)
    # 8-bit, K = 4, two members: torch's ConvNet up to the activation grid
    t = lambda a: torch.from_numpy(np.asarray(a)).double()
    h = t(x)
    saved = {}
    for l, (Wl, b, (o, c, k, st, pd)) in enumerate(zip(Ws, bs, geo)):
        saved[l] = h
        z = torch.nn.functional.conv2d(h, t(Wl).reshape(o, c, k, k), t(b), stride=st, padding=pd)
        if skip[l] >= 0:
            z = z + saved[skip[l]]
        h = torch.relu(z) if acts[l] == "relu" else z
    ref = h.permute(0, 2, 3, 1).reshape(-1, 16).numpy()
    r8 = po.chain_forward(layers(8, 4), xt, split=[2, 2], grid=(N, H, W))
    assert np.abs(r8["y"] - ref).max() < 0.03 * np.abs(ref).max()


def test_asymmetric_conv_chain_is_the_pinned_asymmetric_conv_layer_by_layer():
    """Asymmetric codes (Sec. 4.3) in front of the convolutions of a member chain: with one member it is the
    pinned single-layer routine (whose padding is the real value 0) applied layer by layer with ReLU and a
    skip; with two members the sum is the members'; and after ReLUs, at 4-bit activations, it is closer
    to torch's fp64 ConvNet than the symmetric chain."""
    rng = np.random.default_rng(187)
    N, H, W, C = 2, 7, 6, 8
    geo = [(16, C, 3, 1, 1), (16, 16, 3, 1, 1), (16, 16, 3, 1, 1), (24, 16, 3, 2, 1), (8, 24, 0, 1, 0)]   # O, Cin, k, stride, pad
    Ws = [(rng.standard_normal((o, c * max(k, 1) ** 2)) * math.sqrt(2.0 / (c * max(k, 1) ** 2))).astype(f32) for o, c, k, _, _ in geo]
    bs = [(0.2 * rng.standard_normal(o)).astype(f32) for o, *_ in geo]
    acts = ["relu", "relu", "relu", "relu", "none"]
    skip = [-1, -1, 1, -1, -1]
    x = np.abs(rng.standard_normal((N, C, H, W))).astype(f32)
    xt = np.ascontiguousarray(x.transpose(0, 2, 3, 1)).reshape(N * H * W, C)

    def layers(bits, K):
        return [po.ChainLayer(po.expand(Wl, bits, K, 1.0, 8), b, a, sk, True, k, k, st, pd)
                for Wl, b, a, sk, (o, c, k, st, pd) in zip(Ws, bs, acts, skip, geo)]

    L4 = layers(4, 2)
    grids = po.chain_grids(L4, (N, H, W))
    to_nchw = lambda a, g: a.reshape(g[0], g[1], g[2], -1).transpose(0, 3, 1, 2)
    r = po.chain_forward(L4, xt, grid=(N, H, W), asymmetric=True)
    a0 = np.maximum(po.forward_conv2d_asymmetric(L4[0].exp, x, 3, 3, 1, 1, bias=bs[0])["y"], 0)
    a1 = np.maximum(po.forward_conv2d_asymmetric(L4[1].exp, to_nchw(a0, grids[1]), 3, 3, 1, 1, bias=bs[1])["y"], 0)
    a2 = np.maximum((po.forward_conv2d_asymmetric(L4[2].exp, to_nchw(a1, grids[2]), 3, 3, 1, 1, bias=bs[2])["y"] + a0).astype(f32), 0)
    a3 = np.maximum(po.forward_conv2d_asymmetric(L4[3].exp, to_nchw(a2, grids[3]), 3, 3, 2, 1, bias=bs[3])["y"], 0)
    y = po.forward_asymmetric(L4[4].exp, a3, bias=bs[4])["y"]
    assert all(np.array_equal(r["acts"][i][0], a) for i, a in enumerate([a0, a1, a2, a3]))
    assert np.array_equal(r["y"], y)
    assert not np.array_equal(r["y"], po.chain_forward(L4, xt, grid=(N, H, W))["y"])
    r2 = po.chain_forward(L4, xt, split=[1, 1], grid=(N, H, W), asymmetric=True)
    assert np.array_equal(r2["y"], (r2["members"][0] + r2["members"][1]).astype(f32))
    # against torch's fp64 ConvNet, 8-bit weights (K = 4), 4-bit activations
    t = lambda a: torch.from_numpy(np.asarray(a)).double()
    h, saved = t(x), {}
    for l, (Wl, b, (o, c, k, st, pd)) in enumerate(zip(Ws, bs, geo)):
        saved[l] = h
        kk = max(k, 1)
        z = torch.nn.functional.conv2d(h, t(Wl).reshape(o, c, kk, kk), t(b), stride=st, padding=pd)
        if skip[l] >= 0:
            z = z + saved[skip[l]]
        h = torch.relu(z) if acts[l] == "relu" else z
    ref = h.permute(0, 2, 3, 1).reshape(-1, 8).numpy()
    L8 = layers(8, 4)
    e_sym = np.abs(po.chain_forward(L8, xt, split=[2, 2], grid=(N, H, W), act_bits=4)["y"] - ref).mean()
    e_asym = np.abs(po.chain_forward(L8, xt, split=[2, 2], grid=(N, H, W), act_bits=4, asymmetric=True)["y"] - ref).mean()
    assert e_asym < 0.8 * e_sym, (e_asym, e_sym)


# ---------------------------------------------------------------- App. C: diagnostics
def test_spectral_norm_against_svd_and_closed_forms():
    rng = np.random.default_rng(90)
    for shape in [(24, 40), (64, 17), (5, 5)]:
        W = rng.standard_normal(shape)
        sv = np.linalg.svd(W, compute_uv=False)
        got = po.spectral_norm(W, 400)
        assert got <= sv[0] * (1 + 1e-12)                       # a Rayleigh quotient never exceeds s
        assert math.isclose(got, sv[0], rel_tol=1e-6)
        few = po.spectral_norm(W, 3)
        assert few <= got * (1 + 1e-12)                          # and grows with the iterations
    # rank one: s = |a| |b| after a single step; diagonal: the largest |entry|
    a, b = rng.standard_normal(9), rng.standard_normal(13)
    assert math.isclose(po.spectral_norm(np.outer(a, b), 2), np.linalg.norm(a) * np.linalg.norm(b), rel_tol=1e-12)
    d = np.diag([0.5, -3.0, 2.0, 1.0])
    assert math.isclose(po.spectral_norm(d, 200), 3.0, rel_tol=1e-9)
    assert po.spectral_norm(np.zeros((4, 6)), 5) == 0.0
    v0 = po.power_start_vector(1000)
    assert math.isclose(float(np.linalg.norm(v0)), 1.0, rel_tol=1e-12) and 350 < int((v0 > 0).sum()) < 650


@pytest.mark.parametrize("bits,K", [(8, 2), (4, 3), (2, 5)])
def test_error_bounds_hold_element_wise(bits, K):
    """u of the Lemma bounds every element's error of a dense expansion; the stored-order bound
    does the same for a sparse one and is never looser than it has to be (some element comes
    within a factor 2q_max of it); hence ||W - W^(K)||_2 <= sqrt(O I) u."""
    W = _rand_w(91 + bits, 64, 96, heavy=True)
    dense = po.expand(W, bits, K, 1.0, 16)
    err = np.abs(W.astype(np.float64) - dense.reconstruct())
    slack = np.abs(W).max() * 2.0 ** -21
    assert err.max() <= po.lemma_bound_u(dense) + slack
    assert err.max() <= po.stored_bound_u(dense) + slack
    assert po.stored_bound_u(dense) <= po.lemma_bound_u(dense) * (1 + 1e-6)
    sparse = po.expand(W, bits, K, 0.5, 16)
    errs = np.abs(W.astype(np.float64) - sparse.reconstruct())
    assert errs.max() <= po.stored_bound_u(sparse) + slack
    assert np.linalg.svd(W - sparse.reconstruct(), compute_uv=False)[0] <= math.sqrt(W.size) * po.stored_bound_u(sparse) + slack
    if K > 1:
        assert po.stored_bound_u(sparse) >= po.stored_bound_u(dense)   # pruning cannot tighten the bound


def test_U_closed_forms():
    # one layer: U = s u; two layers, as in the theorem's proof: s_A u_A + (s_A u_A + s_B u_B) + s_A u_A (s_A u_A + s_B u_B)
    assert math.isclose(po.error_bound_U([3.0], [0.01]), 0.03)
    a, b = 2.0 * 0.05, 4.0 * 0.01
    assert math.isclose(po.error_bound_U([2.0, 4.0], [0.05, 0.01]), (a + 1) * (a + b + 1) - 1)
    assert po.error_bound_U([1.0, 1.0, 1.0], [0.0, 0.0, 0.0]) == 0.0
    # more orders shrink u by q_max per order, hence U
    W = _rand_w(95, 32, 48)
    us = [po.lemma_bound_u(po.expand(W, 4, K, 1.0, 16)) for K in (1, 2, 3)]
    assert math.isclose(us[1], us[0] / 7, rel_tol=1e-6) and math.isclose(us[2], us[0] / 49, rel_tol=1e-6)
    s = po.spectral_norm(W, 200)
    Us = [po.error_bound_U([s, s], [u, u]) for u in us]
    assert Us[0] > Us[1] > Us[2] > 0


# ---------------------------------------------------------------- App. H
def test_operation_head_count_closed_form():
    o, q, e = po.bit_operations(D=1, d=1, n_i=4096, n_o=11008, s=1, b=4, k=3)
    assert o == 4096 * 11008 * 32 * 5
    assert q == (4096 + 11008) * 160 + 4096 * 11008 * 8
    assert e - q == 2 * 4096 * 11008 * 8
    o2, q2, _ = po.bit_operations(D=14, d=3, n_i=256, n_o=256, s=1, b=8, k=1)
    assert o2 == 14 * 14 * 9 * 256 * 256 * 160 and q2 == 196 * (512 * 160 + 9 * 65536 * 24)
    # MAC counter against T*I*O*(1+(K-1)*gamma)
    ex = po.expand(_rand_w(80, 64, 32), 4, 3, 0.5, 8)
    assert po.expansion_macs(ex, 10) == 10 * 32 * 64 * 2


# ---------------------------------------------------------------- generator sanity for the configs
def test_workload_shapes_and_seeding():
    for cfg, w in wl.WORKLOADS.items():
        for l in w.layers:
            assert l.out_features % l.group == 0
            assert sum(w.split) == l.K
    a = wl.make_weight(wl.C1, 0)
    b = wl.make_weight(wl.C1, 0)
    assert a.dtype == f32 and a.shape == (256, 256) and np.array_equal(a, b)
    assert abs(float(a.std()) - 0.02) < 1e-3
    x = wl.make_input(wl.scaled(wl.C2, 8, 32, 196))
    assert x.min() == 0.0 and x.shape == (1, 8, 14, 14)


def test_order_norms_against_svd_of_the_order_matrices():
    """||R^(k)|| of every order against numpy's SVD of the matrix that the (separately pinned)
    partial reconstructions differ by; pruned rows contribute nothing."""
    rng = np.random.default_rng(95)
    W = (rng.standard_normal((48, 40)) * 0.1).astype(f32)
    for bits, K, gamma in [(4, 3, 0.5), (2, 4, 0.25), (8, 2, 1.0)]:
        e = po.expand(W, bits, K, gamma, 8)
        got = po.order_norms(e, 600)
        assert len(got) == K
        for k in range(1, K + 1):
            Rk = e.reconstruct(k) - (e.reconstruct(k - 1) if k > 1 else 0.0)
            sv = np.linalg.svd(Rk, compute_uv=False)[0]
            assert got[k - 1] <= sv * (1 + 1e-12) and math.isclose(got[k - 1], sv, rel_tol=1e-5), (bits, k)
        assert all(got[k] < got[k - 1] for k in range(1, K))      # the residual shrinks with every order
    # the first order of a fine expansion is W up to the grid: Weyl's inequality
    e8 = po.expand(W, 8, 2, 1.0, 8)
    n8 = po.order_norms(e8, 600)
    assert abs(n8[0] - np.linalg.svd(W.astype(np.float64), compute_uv=False)[0]) <= n8[1] * (1 + 1e-6) + np.linalg.svd(W - e8.reconstruct(), compute_uv=False)[0]


def test_U_ens_worked_examples_and_predictor_size_rule(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "uens_worked.json")))
    for c in g["cases"]:
        assert math.isclose(po.error_bound_U_ens(c["norms"], c["split"], c["lam"]), c["U"], rel_tol=1e-12), c["name"]
    r = g["k1_rule"]
    K = len(r["norms"][0])
    for K1, U in enumerate(r["U_by_K1"], start=1):
        assert math.isclose(po.error_bound_U_ens(r["norms"], [K1, K - K1]), U, rel_tol=1e-12)
    for q in r["queries"]:
        assert po.first_predictor_size(r["norms"], q["logit_norm"], q["ratio"]) == q["K1"], q
    # scaling every lambda of one hidden layer by c scales every ensembling term by c
    norms = [[3, 1, 0.5, 0.25], [2, 1, 0.5, 0.125], [8, 2, 1, 1]]
    ones = [[1.0] * 4, [1.0] * 4]
    base = po.error_bound_U_ens(norms, [2, 1, 1], ones)
    scaled = po.error_bound_U_ens(norms, [2, 1, 1], [[3.0] * 4, [1.0] * 4])
    head = (8 + 2) / 4
    assert math.isclose(scaled - head, 3.0 * (base - head), rel_tol=1e-12)
    with pytest.raises(ValueError):
        po.error_bound_U_ens(norms, [2, 1])


def test_expansion_with_another_rounding_operator():
    """The rounding operator is a plug-in (Sec. 4.5).  Round-to-nearest passed in as an operator
    reproduces the built-in expansion bit for bit; truncation toward zero still telescopes
    (W = sum of the terms + last residual, exactly in fp32 steps) with the one-step error
    |residual| < s instead of s/2, and orders computed from it still shrink the error."""
    rng = np.random.default_rng(97)
    W = (rng.standard_normal((32, 40)) * 0.05).astype(f32)
    calls = []

    def rne(k, E, s, qm):
        calls.append((k, E.shape))
        return np.rint(E / np.where(s > 0, s, 1).astype(f32)[:, None])

    a = po.expand(W, 4, 3, 0.5, 8)
    b = po.expand(W, 4, 3, 0.5, 8, operator=rne)
    assert [c[0] for c in calls] == [1, 2, 3] and calls[0][1] == (32, 40) and calls[1][1] == (16, 40)
    for oa, ob in zip(a.orders, b.orders):
        assert np.array_equal(oa.group_ids, ob.group_ids) and np.array_equal(oa.scales, ob.scales)
        assert np.array_equal(oa.codes, ob.codes)

    trunc = lambda k, E, s, qm: np.trunc(E / np.where(s > 0, s, 1).astype(f32)[:, None])
    res = []
    t = po.expand(W, 4, 3, 1.0, 8, residuals=res, operator=trunc)
    for k in range(1, 4):
        sk = t.dense_scales(k).astype(np.float64)[:, None]
        assert np.all(np.abs(res[k - 1]) <= sk * (1 + 1e-6))            # less than one step
        assert np.all(np.abs(t.dense_codes(k)) <= 7)
    assert np.abs(res[0]).max() > a.dense_scales(1).max() / 2          # and really not nearest
    assert np.allclose(W.astype(np.float64), t.reconstruct() + res[-1], rtol=0, atol=1e-7)
    errs = [np.abs(W - t.reconstruct(k)).max() for k in (1, 2, 3)]
    assert errs[2] < errs[1] < errs[0]
    # codes out of range are clamped; a wrong shape is refused
    big = po.expand(W, 4, 1, 1.0, 8, operator=lambda k, E, s, qm: np.full(E.shape, 100))
    assert np.all(big.orders[0].codes == 7)
    with pytest.raises(ValueError):
        po.expand(W, 4, 1, 1.0, 8, operator=lambda k, E, s, qm: np.zeros((1, 1)))
