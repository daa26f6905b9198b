"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

Configs 1 to 4 are compared whole (every token, every output channel, every order).  The
gated MLP of config 5 at 4096 tokens is compared on a stratified sample -- one seeded token
out of every 16-token block, so every token tile and every block of a tile holds a checked
row -- each sampled row being an independent dot product the checker computes one by one.
Integer state (codes, scales, Q(x), int32 accumulators) is bit-exact on all five configs;
fp32 output within 1e-3 relative."""
import numpy as np
import pytest
import torch

from oracle import pipe_oracle as po
from paper_2311_15806_amd import workloads as wl
from _parity import assert_close_fp32, assert_expansion_equal, dev, oracle_expand

pytestmark = pytest.mark.gpu
f32 = np.float32


@pytest.fixture(scope="module")
def pipe():
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2311_15806_amd.binding as b
    return b


def _stratified_tokens(T, seed, block=16):
    """One seeded token out of every `block` consecutive tokens (all of them when T <= 256), plus
    the first and last token and the two sides of the first 64-token tile boundary."""
    if T <= 256:
        return np.arange(T)
    rng = np.random.default_rng(seed)
    starts = np.arange(0, T, block)
    idx = np.minimum(starts + rng.integers(0, block, size=starts.size), T - 1)
    return np.unique(np.concatenate([idx, [0, T - 1, 63, 64]]))


def _rows(exp, acc_rows_by_order):
    """Scatter per-order [n, stored_rows] accumulators into [K, n, O] (pruned rows 0)."""
    n = acc_rows_by_order[0].shape[0]
    acc = np.zeros((exp.K, n, exp.out_features), dtype=np.int32)
    for k in range(1, exp.K + 1):
        acc[k - 1][:, exp.rows(k)] = acc_rows_by_order[k - 1]
    return acc


def _oracle_rows(exp, Qx_rows, s_x, split=None, bias=None):
    acc = _rows(exp, [po.contract(Qx_rows, o.codes) for o in exp.orders])
    ys = po.dequantize(exp, acc, s_x, split, bias, f32)
    return acc, ys


def test_c1_full(pipe):
    w = wl.C1
    spec = w.layers[0]
    W, x = wl.make_weight(w, 0), wl.make_input(w)
    ora = oracle_expand(W, spec)
    ref = po.forward(ora, x)
    g = pipe.pipe_expand(dev(W), spec.bits, spec.K, spec.gamma, spec.group)
    assert_expansion_equal(g, ora)
    acc, qx, sx = pipe.pipe_forward_acc(g, dev(x))
    assert np.array_equal(qx.cpu().numpy(), ref["Qx"]) and np.array_equal(acc.cpu().numpy(), ref["acc"])
    assert_close_fp32(pipe.pipe_forward(g, dev(x)).cpu().numpy(), ref["y"])
    g.free()


def test_c2_full_conv(pipe):
    w = wl.C2
    spec, c = w.layers[0], w.conv
    W, x = wl.make_weight(w, 0), wl.make_input(w)
    ora = oracle_expand(W, spec)
    # the config's form: the convolution as an implicit GEMM (no patch matrix)
    g = pipe.pipe_expand_conv2d(dev(W), c["C"], c["kh"], c["kw"], spec.bits, spec.K, spec.gamma, spec.group)
    assert_expansion_equal(g, ora)
    # the checker's conv on its im2col matrix (direct conv == im2col GEMM is pinned on the CPU)
    Qx, sx = po.quantize_activations(x)
    cols = po.im2col(Qx, c["kh"], c["kw"], c["stride"], c["pad"])
    acc, ys = _oracle_rows(ora, cols, sx, split=list(w.split))
    # integer state of the convolution: Q(x), scale and every order's accumulators against the
    # checker's direct convolution (no patch matrix), whole tensor
    acc_g, qx_g, sx_g = pipe.pipe_forward_conv2d_acc(g, dev(x), c["kh"], c["kw"], c["stride"], c["pad"])
    assert np.array_equal(sx_g.cpu().numpy().view(np.uint32), np.array([sx], f32).view(np.uint32))
    assert np.array_equal(qx_g.cpu().numpy(), Qx)
    acc_direct = _rows(ora, [po.conv2d_acc_direct(Qx, o.codes, c["kh"], c["kw"], c["stride"], c["pad"]) for o in ora.orders])
    assert np.array_equal(acc_g.cpu().numpy(), acc_direct)
    assert np.array_equal(acc, acc_direct)
    del acc_g
    y = pipe.pipe_forward_conv2d(g, dev(x), c["kh"], c["kw"], c["stride"], c["pad"], split=list(w.split)).cpu().numpy()
    assert y.shape == (w.tokens, spec.out_features)
    assert_close_fp32(y, po.sum_members(ys))
    ym = pipe.pipe_forward_conv2d(g, dev(x), c["kh"], c["kw"], c["stride"], c["pad"], split=list(w.split),
                                  reduce_members=False).cpu().numpy()
    assert_close_fp32(ym, ys)
    # the explicit-gather path on a plain expansion of the same weight: same integers, same output bits
    ge = pipe.pipe_expand(dev(W), spec.bits, spec.K, spec.gamma, spec.group)
    assert_expansion_equal(ge, ora)
    acc_e, _, _ = pipe.pipe_forward_conv2d_acc(ge, dev(x), c["kh"], c["kw"], c["stride"], c["pad"])
    assert np.array_equal(acc_e.cpu().numpy(), acc_direct)
    ye = pipe.pipe_forward_conv2d(ge, dev(x), c["kh"], c["kw"], c["stride"], c["pad"], split=list(w.split)).cpu().numpy()
    assert np.array_equal(y, ye)
    g.free(); ge.free()


def test_c3_full_mlp(pipe):
    w = wl.C3
    l1, l2 = w.layers
    W1, W2, x = wl.make_weight(w, 0), wl.make_weight(w, 1), wl.make_input(w)
    o1, o2 = oracle_expand(W1, l1), oracle_expand(W2, l2)
    g1 = pipe.pipe_expand(dev(W1), l1.bits, l1.K, l1.gamma, l1.group)
    g2 = pipe.pipe_expand(dev(W2), l2.bits, l2.K, l2.gamma, l2.group)
    assert_expansion_equal(g1, o1)
    assert_expansion_equal(g2, o2)
    ref = po.mlp_forward(o1, o2, "gelu", x)
    y, h = pipe.pipe_mlp_forward(g1, g2, pipe.PIPE_ACT_GELU, dev(x), return_hidden=True)
    hg = h.cpu().numpy()
    assert_close_fp32(hg, ref["h"], tol=1e-5)
    ref2 = po.mlp_second_layer(o2, hg)
    assert_close_fp32(y.cpu().numpy(), ref2["y"])
    # bit-exact first layer: same Q(x), scale and accumulators, every token
    acc, qx, sx = pipe.pipe_forward_acc(g1, dev(x))
    assert np.array_equal(qx.cpu().numpy(), ref["Qx"])
    assert np.array_equal(sx.cpu().numpy().view(np.uint32), np.array([ref["s_x"]], f32).view(np.uint32))
    assert np.array_equal(acc.cpu().numpy(), po.forward_acc(o1, ref["Qx"]))
    del acc
    # bit-exact second layer on the GPU's own hidden activation (its codes depend on the
    # device's erf, so the checker quantizes the same fp32 tensor)
    acc2, qh, sh = pipe.pipe_forward_acc(g2, h[0])
    assert np.array_equal(qh.cpu().numpy(), ref2["Qh"][0])
    assert np.array_equal(sh.cpu().numpy().view(np.uint32), ref2["s_h"][:1].view(np.uint32))
    assert np.array_equal(acc2.cpu().numpy(), po.forward_acc(o2, ref2["Qh"][0]))
    g1.free(); g2.free()


@pytest.fixture(scope="module")
def c4(pipe):
    w = wl.C4
    spec = w.layers[0]
    W = wl.make_weight(w, 0)
    ora = oracle_expand(W, spec)
    g = pipe.pipe_expand(dev(W), spec.bits, spec.K, spec.gamma, spec.group)
    yield w, ora, g
    g.free()


def test_c4_expand_bit_exact(pipe, c4):
    w, ora, g = c4
    assert_expansion_equal(g, ora)
    assert g.macs_per_token() == po.expansion_macs(ora, 1) == 4096 * 19264


@pytest.mark.parametrize("T", [1, 16, 64, 128, 256, 2048, 4096])
def test_c4_forward(pipe, c4, T):
    w, ora, g = c4
    x = wl.make_input(wl.with_tokens(w, T))
    xd = dev(x)
    Qx, sx = po.quantize_activations(x)
    acc_ref, ys = _oracle_rows(ora, Qx, sx)          # every token
    acc, qx, sxg = pipe.pipe_forward_acc(g, xd)
    assert np.array_equal(sxg.cpu().numpy().view(np.uint32), np.array([sx], f32).view(np.uint32))
    assert np.array_equal(qx.cpu().numpy(), Qx)
    for k in range(ora.K):                           # order by order: bounds the host copies
        assert np.array_equal(acc[k].cpu().numpy(), acc_ref[k]), "order %d" % (k + 1)
    del acc, acc_ref
    y = pipe.pipe_forward(g, xd)
    assert_close_fp32(y.cpu().numpy(), ys[0])
    # properties that hold at any size: pruned (order, group) pairs contribute nothing, and the
    # whole output is finite and reproducible
    y2 = pipe.pipe_forward(g, xd)
    assert torch.equal(y, y2) and bool(torch.isfinite(y).all())


@pytest.fixture(scope="module")
def c5(pipe):
    w = wl.C5
    l1, l2 = w.layers
    W1, W2 = wl.make_weight(w, 0), wl.make_weight(w, 1)
    o1, o2 = oracle_expand(W1, l1), oracle_expand(W2, l2)
    g1 = pipe.pipe_expand(dev(W1), l1.bits, l1.K, l1.gamma, l1.group)
    g2 = pipe.pipe_expand(dev(W2), l2.bits, l2.K, l2.gamma, l2.group)
    yield w, o1, o2, g1, g2
    g1.free(); g2.free()


def test_c5_expand_bit_exact(pipe, c5):
    w, o1, o2, g1, g2 = c5
    assert_expansion_equal(g1, o1)
    assert_expansion_equal(g2, o2)


@pytest.mark.parametrize("T", [1, 16, 100, 4096])
def test_c5_gated_mlp(pipe, c5, T):
    w, o1, o2, g1, g2 = c5
    split = list(w.split)
    x = wl.make_input(wl.with_tokens(w, T))
    y, h = pipe.pipe_mlp_forward(g1, g2, pipe.PIPE_ACT_SILU_GATED, dev(x), split=split, return_hidden=True)
    hg = h.cpu().numpy()                                       # [M, T, H]
    M, H = len(split), o2.in_features
    sel = _stratified_tokens(T, 5)
    seld = torch.from_numpy(sel).to("cuda:0")
    # layer 1 on the sampled tokens: integer contraction, member-wise epilogue, SiLU(gate)*up
    Qx, sx = po.quantize_activations(x)
    acc1_ref, y1 = _oracle_rows(o1, Qx[sel], sx, split=split)          # [K, n, 2H], [M, n, 2H]
    # integer state of layer 1: Q(x) and the scale whole, the accumulators of every order on the sample
    acc1, qx1, sx1 = pipe.pipe_forward_acc(g1, dev(x))
    assert np.array_equal(sx1.cpu().numpy().view(np.uint32), np.array([sx], f32).view(np.uint32))
    assert np.array_equal(qx1.cpu().numpy(), Qx)
    assert np.array_equal(acc1[:, seld].cpu().numpy(), acc1_ref)
    del acc1, qx1
    h_ref = np.stack([po.silu_mul(y1[m][:, :H], y1[m][:, H:]) for m in range(M)])
    assert_close_fp32(hg[:, sel], h_ref, tol=1e-5)
    # layer 2 on the GPU's own hidden activations (scale = max over ALL tokens of the member)
    members = []
    for m in range(M):
        Qh, sh = po.quantize_activations(hg[m])
        acc2 = _rows(o2, [po.contract(Qh[sel], o.codes) for o in o2.orders])
        # integer state of layer 2 for this member's tensor: codes and scale whole, accumulators on the sample
        acc2_g, qh_g, sh_g = pipe.pipe_forward_acc(g2, h[m])
        assert np.array_equal(sh_g.cpu().numpy().view(np.uint32), np.array([sh], f32).view(np.uint32))
        assert np.array_equal(qh_g.cpu().numpy(), Qh)
        assert np.array_equal(acc2_g[:, seld].cpu().numpy(), acc2)
        del acc2_g, qh_g
        members.append(po.dequantize(o2, acc2, sh, split, None, f32)[m])
    y_ref = po.sum_members(np.stack(members))
    assert_close_fp32(y.cpu().numpy()[sel], y_ref)


def test_c4_weight_with_unstructured_mask(pipe):
    """The 11008 x 4096 layer expanded with an unstructured mask (Sec. 3.1): 45 million entries per
    selection, so every level of the builder's radix select holds bins far beyond 16 bits; codes
    and scales equal the checker's bit for bit, and a decode-sized forward its accumulators."""
    w = wl.with_tokens(wl.C4, 16)
    spec = w.layers[0]
    W, x = wl.make_weight(w, 0), wl.make_input(w)
    K = 3
    ora = po.expand(W, spec.bits, K, spec.gamma, spec.group, mask="unstructured")
    g = pipe.pipe_expand_unstructured(dev(W), spec.bits, K, spec.gamma, spec.group)
    assert_expansion_equal(g, ora)
    ref = po.forward(ora, x)
    acc, _, _ = pipe.pipe_forward_acc(g, dev(x))
    assert np.array_equal(acc.cpu().numpy(), ref["acc"])
    assert_close_fp32(pipe.pipe_forward(g, dev(x)).cpu().numpy(), ref["y"])
    g.free()
