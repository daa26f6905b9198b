"""GPU parity on seeded random configurations: layer shapes, bit widths, expansion orders, sparsity,
group sizes, batch sizes (all three contraction kernels and the resident decode launch), member
groupings, bias, static or dynamic input scale.  Every case goes through the C ABI and is held to
the same bars as the fixed cases: expansion and int32 accumulators bit-exact, fp32 within 1e-3."""
import math

import numpy as np
import pytest
import torch

from oracle import pipe_oracle as po
from _parity import assert_close_fp32, assert_expansion_equal, dev

pytestmark = pytest.mark.gpu

f32 = np.float32
ACT = {"none": 0, "gelu": 1, "relu": 3}


@pytest.fixture(scope="module")
def pipe():
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2311_15806_amd.binding as b
    return b


def _split(rng, K):
    if K == 1 or rng.random() < 0.3:
        return None
    M = int(rng.integers(2, min(K, 4) + 1))
    cuts = sorted(rng.choice(np.arange(1, K), size=M - 1, replace=False).tolist())
    return [b - a for a, b in zip([0] + cuts, cuts + [K])]


def _layer(rng, O=None, I=None, bits=None, K=None):
    bits = bits or int(rng.choice([2, 3, 4, 5, 8]))
    K = K or int(rng.choice([1, 2, 3, 4, 4, 5, 7, 12]))
    gamma = float(rng.choice([0.25, 0.34, 0.5, 0.75, 1.0]))
    if O is None:
        group = int(rng.choice([16, 32, 48, 64]))
        O = group * int(rng.integers(1, 13))
    else:
        group = int(rng.choice([g for g in (16, 32, 48, 64) if O % g == 0]))
    if I is None:
        I = int(rng.choice([16, 64, 100, 200, 256, 333, 512, 700, 1040, 1500]))
    if rng.random() < 0.5:
        W = (rng.standard_t(3, size=(O, I)) * 0.015).astype(f32)
    else:
        W = (rng.standard_normal((O, I)) * 0.05).astype(f32)
    return W, bits, K, gamma, group


def _expand(pipe, W, bits, K, gamma, group):
    """Both expansions, or (None, None) when a mask decision of the checker sits on a near-tie."""
    gaps = []
    o = po.expand(W, bits, K, gamma, group, gaps=gaps)
    if not all(g > 1e-9 for g in gaps):
        return None, None
    g = pipe.pipe_expand(dev(W), bits, K, gamma, group)
    assert_expansion_equal(g, o)
    return o, g


def _linear(pipe, rng):
    W, bits, K, gamma, group = _layer(rng)
    O, I = W.shape
    T = int(rng.choice([1, 2, 7, 16, 17, 33, 64, 100, 129, 200, 257, 400]))
    o, g = _expand(pipe, W, bits, K, gamma, group)
    if o is None:
        return
    x = rng.standard_normal((T, I)).astype(f32)
    if rng.random() < 0.5:
        x[:, int(rng.integers(0, I))] *= 20.0
    split = _split(rng, K)
    b = rng.standard_normal(O).astype(f32) if rng.random() < 0.5 else None
    bd = None if b is None else dev(b)
    s_x = 0.0 if rng.random() < 0.7 else float(np.abs(x).max() / 127.0 * rng.uniform(0.5, 1.5))
    pipe.pipe_set_kernel(int(rng.choice([0, 0, 1, 2])))
    try:
        ref = po.forward(o, x, s_x=s_x if s_x > 0 else None, split=split, bias=b)
        assert_close_fp32(pipe.pipe_forward(g, dev(x), s_x=s_x, split=split, bias=bd).cpu().numpy(), ref["y"])
        acc, qx, _ = pipe.pipe_forward_acc(g, dev(x), s_x=s_x)
        assert np.array_equal(qx.cpu().numpy(), ref["Qx"])
        assert np.array_equal(acc.cpu().numpy(), ref["acc"])
        refm = po.forward(o, x, s_x=s_x if s_x > 0 else None, split=split, bias=b, reduce_members=False)
        ym = pipe.pipe_forward(g, dev(x), s_x=s_x, split=split, bias=bd, reduce_members=False).cpu().numpy()
        assert_close_fp32(ym, refm["y"])
        if rng.random() < 0.4:
            ra = po.forward_asymmetric(o, x, split=split, bias=b)
            assert_close_fp32(pipe.pipe_forward_asymmetric(g, dev(x), split=split, bias=bd).cpu().numpy(), ra["y"])
    finally:
        pipe.pipe_set_kernel(0)
        g.free()


def _mlp(pipe, rng):
    kind = "gated" if rng.random() < 0.5 else "gelu"
    bits, K = int(rng.choice([2, 4, 8])), int(rng.choice([2, 3, 4]))
    H, I, O2 = 32 * int(rng.integers(1, 10)), int(rng.choice([64, 128, 200, 512])), 16 * int(rng.integers(1, 12))
    O1 = 2 * H if kind == "gated" else H
    W1, _, _, gm1, G1 = _layer(rng, O1, I, bits, K)
    W2, _, _, gm2, G2 = _layer(rng, O2, H, bits, K)
    T = int(rng.choice([1, 3, 16, 40, 129, 150]))
    o1, e1 = _expand(pipe, W1, bits, K, gm1, G1)
    if o1 is None:
        return
    o2, e2 = _expand(pipe, W2, bits, K, gm2, G2)
    if o2 is None:
        e1.free()
        return
    x = rng.standard_normal((T, I)).astype(f32)
    split = _split(rng, K)
    b1 = rng.standard_normal(O1).astype(f32) * 0.1 if rng.random() < 0.5 else None
    b2 = rng.standard_normal(O2).astype(f32) * 0.1 if rng.random() < 0.5 else None
    bd1, bd2 = (None if b1 is None else dev(b1)), (None if b2 is None else dev(b2))
    act = pipe.PIPE_ACT_SILU_GATED if kind == "gated" else pipe.PIPE_ACT_GELU
    pipe.pipe_set_decode_resident(int(rng.choice([0, 1, 2])))
    try:
        asym = rng.random() < 0.3
        fn = pipe.pipe_mlp_forward_asymmetric if asym else pipe.pipe_mlp_forward
        y, h = fn(e1, e2, act, dev(x), split=split, bias1=bd1, bias2=bd2, return_hidden=True)
        y, h = y.cpu().numpy(), h.cpu().numpy()
        ref = po.mlp_forward(o1, o2, kind, x, split=split, bias1=b1, bias2=b2, asymmetric=asym)
        assert h.shape == ref["h"].shape
        for m in range(h.shape[0]):
            # asymmetric codes: two large terms cancel in the kernels' evaluation, so the error follows the tensor's scale
            d = np.abs(h[m].astype(np.float64) - ref["h"][m])
            assert d.max() <= 2e-5 * np.abs(ref["h"][m]).max() + 1e-30
            assert_close_fp32(h[m], ref["h"][m], tol=1e-3 if asym else 2e-5)
        # the last layer of the checker on the GPU's own hidden activations
        assert_close_fp32(y, po.mlp_second_layer(o2, h, split, b2, 8, asym)["y"])
        assert pipe.pipe_resident_status() == 0
    finally:
        pipe.pipe_set_decode_resident(1)
        e1.free()
        e2.free()


def _chain(pipe, rng):
    bits, K, L = int(rng.choice([2, 4, 8])), int(rng.choice([1, 2, 3, 4, 6])), int(rng.integers(1, 6))
    widths = [16 * int(rng.integers(1, 14)) for _ in range(L + 1)]
    if rng.random() < 0.5:
        widths = [widths[0]] * (L + 1)   # equal widths: skips become possible
    T = int(rng.choice([1, 5, 16, 30, 140]))
    olayers, glayers, gpu = [], [], []
    for l in range(L):
        W, _, _, gm, G = _layer(rng, widths[l + 1], widths[l], bits, K)
        o, g = _expand(pipe, W, bits, K, gm, G)
        if o is None:
            for e in gpu:
                e.free()
            return
        gpu.append(g)
        b = rng.standard_normal(widths[l + 1]).astype(f32) * 0.1 if rng.random() < 0.5 else None
        act = "none" if l == L - 1 else str(rng.choice(["relu", "gelu", "none"]))
        skip, pre = -1, True
        cands = [j for j in range(l + 1) if widths[j] == widths[l + 1]]
        if cands and rng.random() < 0.4:
            skip, pre = int(rng.choice(cands)), bool(rng.random() < 0.5)
        olayers.append(po.ChainLayer(o, b, act, skip, pre))
        glayers.append((g, None if b is None else dev(b), ACT[act], skip, pre))
    x = rng.standard_normal((T, widths[0])).astype(f32)
    split = _split(rng, K)
    M = 1 if split is None else len(split)
    pipe.pipe_set_decode_resident(int(rng.choice([0, 1, 2])))
    try:
        y, acts = pipe.pipe_chain_forward(glayers, dev(x), split=split, return_acts=True)
        y, acts = y.cpu().numpy(), [a.cpu().numpy() for a in (acts or [])]
        for l in range(L):   # layer l of the checker on the GPU's own earlier tensors
            skips = po.chain_skips(olayers, l, x, acts, M)
            if l == 0:
                ref = po.chain_layer_members(olayers[0], x, True, skips, split, None)
            else:
                ref = po.chain_layer_members(olayers[l], acts[l - 1], False, skips, split)
            if l < L - 1:
                assert acts[l].shape == ref.shape
                for m in range(M):
                    assert_close_fp32(acts[l][m], ref[m], tol=2e-5)
            else:
                assert_close_fp32(y, po.sum_members(ref))
        assert pipe.pipe_resident_status() == 0
    finally:
        pipe.pipe_set_decode_resident(1)
        for e in gpu:
            e.free()


def _conv(pipe, rng):
    bits, K = int(rng.choice([2, 4, 8])), int(rng.choice([1, 2, 3, 4]))
    implicit = rng.random() < 0.6   # tap-major expansion (input channels a multiple of 64), else the patch-matrix path
    C = 64 * int(rng.integers(1, 4)) if implicit else int(rng.choice([3, 16, 24, 40, 64]))
    kh = int(rng.choice([1, 3, 3, 5]))
    stride, pad = int(rng.choice([1, 1, 2])), int(rng.choice([0, 1, 2]))
    H, Wd, N = int(rng.integers(max(kh, 4), 20)), int(rng.integers(max(kh, 4), 20)), int(rng.integers(1, 5))
    group = int(rng.choice([16, 32]))
    O, gamma = group * int(rng.integers(1, 10)), float(rng.choice([0.25, 0.5, 1.0]))
    Wt = (rng.standard_normal((O, C * kh * kh)) * math.sqrt(2.0 / (C * kh * kh))).astype(f32)
    x = np.maximum(rng.standard_normal((N, C, H, Wd)), 0).astype(f32)
    b = rng.standard_normal(O).astype(f32) if rng.random() < 0.5 else None
    bd = None if b is None else dev(b)
    gaps = []
    ora = po.expand(Wt, bits, K, gamma, group, gaps=gaps)
    if not all(g > 1e-9 for g in gaps):
        return
    g = pipe.pipe_expand_conv2d(dev(Wt), C, kh, kh, bits, K, gamma, group) if implicit else pipe.pipe_expand(dev(Wt), bits, K, gamma, group)
    try:
        assert_expansion_equal(g, ora)
        split = _split(rng, K)
        nhwc = rng.random() < 0.5
        xin = dev(np.ascontiguousarray(x.transpose(0, 2, 3, 1)) if nhwc else x)
        ref = po.forward_conv2d(ora, x, kh, kh, stride, pad, split=split, bias=b)
        acc, _, _ = pipe.pipe_forward_conv2d_acc(g, xin, kh, kh, stride, pad, nhwc=nhwc)
        assert np.array_equal(acc.cpu().numpy(), ref["acc"])
        y = pipe.pipe_forward_conv2d(g, xin, kh, kh, stride, pad, nhwc=nhwc, split=split, bias=bd).cpu().numpy()
        assert_close_fp32(y, ref["y"])
        if not implicit and rng.random() < 0.5:
            ra = po.forward_conv2d_asymmetric(ora, x, kh, kh, stride, pad, split=split, bias=b)
            ya = pipe.pipe_forward_conv2d_asymmetric(g, xin, kh, kh, stride, pad, nhwc=nhwc, split=split, bias=bd).cpu().numpy()
            assert_close_fp32(ya, ra["y"])
    finally:
        g.free()


CASES = {"linear": _linear, "mlp": _mlp, "chain": _chain, "conv": _conv}


@pytest.mark.parametrize("seed", [101, 102, 103, 104])
@pytest.mark.parametrize("kind", sorted(CASES))
def test_random_configurations(pipe, kind, seed):
    rng = np.random.default_rng(seed * 7 + sorted(CASES).index(kind))
    for _ in range(12):
        CASES[kind](pipe, rng)
