"""The resident decode launch (one launch walks all layers of a chain or of the two-layer MLP for
batches of at most 16 tokens) against the per-layer launches, bit for bit, and against the CPU
checker layer by layer; its bounded waits; graph replays."""
import numpy as np
import pytest
import torch

from oracle import pipe_oracle as po
from paper_2311_15806_amd import workloads as wl

from _parity import assert_close_fp32, dev, oracle_expand

pytestmark = pytest.mark.gpu
ACT = {"none": 0, "gelu": 1, "relu": 3}


@pytest.fixture(scope="module")
def pipe():
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2311_15806_amd.binding as b
    b.pipe_set_decode_resident(True)        # the resident launch wherever it applies, not only where it is the default
    yield b
    b.pipe_set_decode_resident(1)
    b.pipe_set_resident_spin_limit(0)


def _both(pipe, fn):
    """fn() with the resident launch and with the per-layer launches."""
    pipe.pipe_set_decode_resident(True)
    a = fn()
    assert pipe.pipe_resident_status() == 0
    pipe.pipe_set_decode_resident(False)
    try:
        b = fn()
    finally:
        pipe.pipe_set_decode_resident(True)
    return a, b


def _expand_all(pipe, w):
    return [pipe.pipe_expand(dev(wl.make_weight(w, l)), s.bits, s.K, s.gamma, s.group) for l, s in enumerate(w.layers)]


@pytest.mark.parametrize("T", [1, 5, 16])
@pytest.mark.parametrize("bits,K,split", [(2, 4, None), (4, 4, [2, 2]), (8, 2, [1, 1]), (4, 3, None), (2, 4, [1, 3])])
def test_resident_chain_equals_per_layer_launches(pipe, bits, K, split, T):
    w = wl.residual_stack(192, 2, 96, bits, K, 0.5, 16, T, split or (K,))
    gs = _expand_all(pipe, w)
    bs = [dev(wl.make_bias(w, l)) for l in range(len(w.layers))]
    layers = [(g, b, ACT[c[0]], c[1], c[2]) for g, b, c in zip(gs, bs, w.chain)]
    x = dev(wl.make_input(w))
    for s_x in (0.0, 0.04):
        (y1, a1), (y2, a2) = _both(pipe, lambda: pipe.pipe_chain_forward(layers, x, s_x=s_x, split=split, return_acts=True))
        assert torch.equal(y1, y2)
        for u, v in zip(a1, a2):
            assert torch.equal(u, v)
    for g in gs:
        g.free()


def test_resident_chain_variants(pipe):
    """Skips from the network input and from earlier tensors, before and after the activation, GELU,
    ragged widths (in_features not a multiple of 256, fewer code tiles than worker waves)."""
    spec = lambda o, i: wl.LayerSpec(o, i, 4, 4, 0.5, 16)
    layers = (spec(112, 112), spec(112, 112), spec(80, 112), spec(80, 80), spec(1040, 80), spec(48, 1040))
    chain = (("relu", 0, False), ("gelu", 0, True), ("none", -1, True), ("relu", 3, True), ("gelu", -1, True), ("none", -1, True))
    w = wl.Workload(name="resident_variants", config=6, kind="chain", layers=layers, tokens=11, split=(2, 2),
                    w_dist=dict(kind=0, std=0.13), x_dist=dict(kind=0), chain=chain)
    gs = _expand_all(pipe, w)
    gl = [(g, dev(wl.make_bias(w, l)), ACT[c[0]], c[1], c[2]) for l, (g, c) in enumerate(zip(gs, w.chain))]
    x = dev(wl.make_input(w))
    for split in (None, [2, 2], [3, 1]):
        (y1, a1), (y2, a2) = _both(pipe, lambda: pipe.pipe_chain_forward(gl, x, split=split, return_acts=True))
        assert torch.equal(y1, y2)
        for u, v in zip(a1, a2):
            assert torch.equal(u, v)
    for g in gs:
        g.free()


@pytest.mark.parametrize("kind,T", [("gelu", 1), ("gelu", 16), ("gated", 1), ("gated", 7), ("gated", 16)])
def test_resident_mlp_equals_per_layer_launches(pipe, kind, T):
    base = wl.C3 if kind == "gelu" else wl.C5
    w = wl.scaled(base, out_div=8, in_div=8, tokens=T)
    split = list(w.split) if len(w.split) > 1 else None
    es = _expand_all(pipe, w)
    act = pipe.PIPE_ACT_GELU if kind == "gelu" else pipe.PIPE_ACT_SILU_GATED
    x = dev(wl.make_input(w))
    b1, b2 = dev(wl.make_bias(w, 0)), dev(wl.make_bias(w, 1))
    (y1, h1), (y2, h2) = _both(pipe, lambda: pipe.pipe_mlp_forward(es[0], es[1], act, x, split=split, bias1=b1, bias2=b2,
                                                                    return_hidden=True))
    assert torch.equal(h1, h2) and torch.equal(y1, y2)
    for e in es:
        e.free()


@pytest.mark.parametrize("T", [1, 16])
def test_resident_stack_of_llm_sized_layers_against_the_checker(pipe, T):
    """A stack of layers shaped like the 7B linear layer scaled by four (2752 x 1024 and back, ternary,
    K = 4): every layer against the checker fed the GPU's own earlier tensors, and the whole stack
    against the per-layer launches bit for bit."""
    up, down = wl.LayerSpec(2752, 1024, 2, 4, 0.25, 64), wl.LayerSpec(1024, 2752, 2, 4, 0.25, 64)
    specs = (up, down, up, down)
    chain = (("relu", -1, True), ("none", 0, True), ("relu", -1, True), ("none", -1, True))
    w = wl.Workload(name="resident_stack", config=7, kind="chain", layers=specs, tokens=T, split=(4,),
                    w_dist=dict(kind=1, df=3.0, scale=0.015, outlier_frac=0.01, outlier_mul=8.0),
                    x_dist=dict(kind=0, outlier_frac=0.005, outlier_mul=20.0), chain=chain)
    Ws = [wl.make_weight(w, l) for l in range(4)]
    ora = [oracle_expand(W, s) for W, s in zip(Ws, specs)]
    gs = [pipe.pipe_expand(dev(W), s.bits, s.K, s.gamma, s.group) for W, s in zip(Ws, specs)]
    olayers = [po.ChainLayer(o, None, c[0], c[1], c[2]) for o, c in zip(ora, chain)]
    gl = [(g, None, ACT[c[0]], c[1], c[2]) for g, c in zip(gs, chain)]
    x = wl.make_input(w)
    (y1, a1), (y2, a2) = _both(pipe, lambda: pipe.pipe_chain_forward(gl, dev(x), return_acts=True))
    assert torch.equal(y1, y2)
    acts = [a.cpu().numpy() for a in a1]
    for l in range(4):
        skips = po.chain_skips(olayers, l, x, acts, 1)
        ref = po.chain_layer_members(olayers[l], x if l == 0 else acts[l - 1], l == 0, skips, None, None)
        got = acts[l][0] if l < 3 else y1.cpu().numpy()
        assert_close_fp32(got, ref[0] if l < 3 else po.sum_members(ref), tol=2e-5 if l < 3 else 1e-3)
    for g in gs:
        g.free()


def test_resident_waits_are_bounded(pipe):
    """With a spin limit of one poll a workgroup gives up waiting at once: the launch still ends (every
    workgroup runs to its end), the status word reports it, and the next launch with the default
    limit is correct again."""
    w = wl.residual_stack(192, 2, 96, 4, 4, 0.5, 16, 8, (4,))
    gs = _expand_all(pipe, w)
    layers = [(g, None, ACT[c[0]], c[1], c[2]) for g, c in zip(gs, w.chain)]
    x = dev(wl.make_input(w))
    good = pipe.pipe_chain_forward(layers, x).clone()
    assert pipe.pipe_resident_status() == 0
    pipe.pipe_set_resident_spin_limit(1)
    try:
        for _ in range(3):
            pipe.pipe_chain_forward(layers, x)
        st = pipe.pipe_resident_status()          # synchronizes: the launches have ended
    finally:
        pipe.pipe_set_resident_spin_limit(0)
    assert st in (0, 1, 2)                        # a single poll may or may not have been enough
    again = pipe.pipe_chain_forward(layers, x)
    assert pipe.pipe_resident_status() == 0
    assert torch.equal(again, good)
    for g in gs:
        g.free()


def test_resident_chain_graph_replays(pipe):
    w = wl.residual_stack(192, 2, 96, 2, 4, 0.5, 16, 16, (2, 2))
    gs = _expand_all(pipe, w)
    layers = [(g, None, ACT[c[0]], c[1], c[2]) for g, c in zip(gs, w.chain)]
    xs = [dev(wl.make_input(w)) * s for s in (1.0, 0.25, 5.0)]
    eager = [pipe.pipe_chain_forward(layers, xi, split=[2, 2]).clone() for xi in xs]
    x = xs[0].clone()
    out = torch.empty_like(eager[0])
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        pipe.pipe_prepare_chain(layers, 16, split=[2, 2])
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        pipe.pipe_chain_forward(layers, x, split=[2, 2], out=out)
    for rep in range(6):
        i = rep % 3
        x.copy_(xs[i])
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager[i]), "replay %d differs" % rep
    for g in gs:
        g.free()


def _launches(pipe, fn):
    """(result of fn(), number of contraction launches it made)."""
    pipe.pipe_timing_read()
    pipe.pipe_timing_enable(True)
    try:
        out = fn()
        torch.cuda.synchronize()
    finally:
        pipe.pipe_timing_enable(False)
    return out, pipe.pipe_timing_read()[1]


def test_resident_limits_layers_and_descriptor_space(pipe):
    """At the limits of the resident launch: 16 layers run as one launch, 17 as per-layer launches; a
    chain whose unit descriptors fill most of a workgroup's table runs resident, one that overflows
    it falls back.  Same results either way."""
    torch.manual_seed(3)
    mk = lambda o, i: pipe.pipe_expand(torch.randn(o, i, device="cuda:0") * (1.5 / i ** 0.5), 4, 2, 1.0, 16)
    x = torch.randn(4, 96, device="cuda:0")
    es = [mk(96, 96) for _ in range(17)]
    for L, want in ((16, 1), (17, 17)):
        layers = [(e, None, ACT["relu"] if l + 1 < L else ACT["none"], -1, True) for l, e in enumerate(es[:L])]
        pipe.pipe_set_decode_resident(True)
        y1, n1 = _launches(pipe, lambda: pipe.pipe_chain_forward(layers, x))
        assert pipe.pipe_resident_status() == 0 and n1 == want, (L, n1)
        pipe.pipe_set_decode_resident(False)
        try:
            y2, n2 = _launches(pipe, lambda: pipe.pipe_chain_forward(layers, x))
        finally:
            pipe.pipe_set_decode_resident(True)
        assert n2 == L and torch.equal(y1, y2)
    for e in es:
        e.free()
    # 122880 output channels in 4 dense orders: 7680 units, 30 per workgroup on 256 compute units
    wide, narrow = 122880, 64
    up = [pipe.pipe_expand(torch.randn(wide, narrow, device="cuda:0") * 0.2, 2, 4, 1.0, 16) for _ in range(3)]
    down = [pipe.pipe_expand(torch.randn(narrow, wide, device="cuda:0") * 0.004, 2, 4, 1.0, 16) for _ in range(3)]
    x = torch.randn(2, narrow, device="cuda:0")
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    for pairs in (2, 3):
        L = 2 * pairs
        layers = []
        for j in range(pairs):
            layers += [(up[j], None, ACT["relu"], -1, True), (down[j], None, ACT["relu"] if j + 1 < pairs else ACT["none"], -1, True)]
        ints = pairs * (-(-7680 // cus) * 48 + -(-4 // cus) * 48)
        pipe.pipe_set_decode_resident(True)
        y1, n1 = _launches(pipe, lambda: pipe.pipe_chain_forward(layers, x))
        assert pipe.pipe_resident_status() == 0
        assert n1 == (1 if ints <= 4096 else L), (pairs, ints, n1)
        pipe.pipe_set_decode_resident(False)
        try:
            y2, n2 = _launches(pipe, lambda: pipe.pipe_chain_forward(layers, x))
        finally:
            pipe.pipe_set_decode_resident(True)
        assert torch.equal(y1, y2)
    for e in up + down:
        e.free()
