"""GPU parity of the L-layer member chains (App. B "Ensemble of more Layers", Fig. 2) against
the CPU checker, layer by layer: each layer of the checker is fed the tensors the GPU produced
for the previous layers, so both sides quantize identical values and every layer is held to the
single-layer bar; the free-running end-to-end comparison allows for the few codes that a
last-bit difference of an activation can flip."""
import numpy as np
import pytest
import torch

from oracle import pipe_oracle as po
from paper_2311_15806_amd import workloads as wl

from _parity import assert_close_fp32, assert_expansion_equal, dev, oracle_expand

pytestmark = pytest.mark.gpu

ACT = {"none": 0, "gelu": 1, "relu": 3}


@pytest.fixture(scope="module")
def pipe():
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2311_15806_amd.binding as b
    return b


def _build(pipe, w, with_bias=True):
    Ws = [wl.make_weight(w, l) for l in range(len(w.layers))]
    bs = [wl.make_bias(w, l) if with_bias else None for l in range(len(w.layers))]
    ora = [oracle_expand(W, s) for W, s in zip(Ws, w.layers)]
    gpu = [pipe.pipe_expand(dev(W), s.bits, s.K, s.gamma, s.group) for W, s in zip(Ws, w.layers)]
    for g, o in zip(gpu, ora):
        assert_expansion_equal(g, o)
    olayers = [po.ChainLayer(o, b, c[0], c[1], c[2]) for o, b, c in zip(ora, bs, w.chain)]
    glayers = [(g, None if b is None else dev(b), ACT[c[0]], c[1], c[2]) for g, b, c in zip(gpu, bs, w.chain)]
    return olayers, glayers, gpu


def _check_chain(pipe, w, olayers, glayers, x, split, s_x=0.0):
    L = len(olayers)
    y, acts = pipe.pipe_chain_forward(glayers, dev(x), s_x=s_x, split=split, return_acts=True)
    y = y.cpu().numpy()
    acts = [a.cpu().numpy() for a in acts]
    M = 1 if split is None else len(split)
    # teacher-forced: layer l of the checker on the GPU's own earlier tensors
    for l in range(L):
        skips = po.chain_skips(olayers, l, x, acts, M)
        if l == 0:
            ref = po.chain_layer_members(olayers[0], x, True, skips, split, s_x if s_x > 0 else None)
        else:
            ref = po.chain_layer_members(olayers[l], acts[l - 1], False, skips, split)
        if l < L - 1:
            assert acts[l].shape == ref.shape
            for m in range(M):
                assert_close_fp32(acts[l][m], ref[m], tol=2e-5)
        else:
            assert_close_fp32(y, po.sum_members(ref))
    # free-running
    full = po.chain_forward(olayers, x, split=split, s_x=s_x if s_x > 0 else None)
    assert_close_fp32(y, full["y"], tol=3e-2, elementwise=False)
    return y


@pytest.mark.parametrize("tokens", [150, 37, 9])
@pytest.mark.parametrize("bits,K,split", [(4, 4, [2, 2]), (2, 4, [1, 1, 2]), (8, 2, None), (2, 8, [3, 3, 2])])
def test_residual_stack_parity(pipe, bits, K, split, tokens):
    w = wl.residual_stack(128, 2, 64, bits, K, 0.5, 16, tokens, split or (K,))
    olayers, glayers, gpu = _build(pipe, w)
    _check_chain(pipe, w, olayers, glayers, wl.make_input(w), split)
    for g in gpu:
        g.free()


def test_chain_skip_variants_and_static_scale(pipe):
    """Skip from the network input (first member only) before and after the activation, a skip on
    the last layer, GELU inside the chain, ragged widths, and a static input scale."""
    spec = lambda o, i: wl.LayerSpec(o, i, 4, 4, 0.5, 16)
    layers = (spec(112, 112), spec(112, 112), spec(80, 112), spec(80, 80))
    chain = (("relu", 0, False), ("gelu", 0, True), ("none", -1, True), ("none", 3, True))
    w = wl.Workload(name="chain_variants", config=6, kind="chain", layers=layers, tokens=70, split=(2, 1, 1),
                    w_dist=dict(kind=0, std=0.13), x_dist=dict(kind=0), chain=chain)
    olayers, glayers, gpu = _build(pipe, w)
    x = wl.make_input(w)
    for kernel in (0, 1):
        pipe.pipe_set_kernel(kernel)
        try:
            _check_chain(pipe, w, olayers, glayers, x, [2, 1, 1])
            _check_chain(pipe, w, olayers, glayers, x, None, s_x=0.03)
        finally:
            pipe.pipe_set_kernel(0)
    for g in gpu:
        g.free()


def test_chain_of_one_and_two_layers_matches_the_other_entry_points(pipe):
    """L = 1 is pipe_forward, L = 2 with GELU is pipe_mlp_forward: bit-identical outputs."""
    w = wl.scaled(wl.C3, out_div=8, in_div=8, tokens=100)
    l1, l2 = w.layers
    W1, W2, x = wl.make_weight(w, 0), wl.make_weight(w, 1), wl.make_input(w)
    b1, b2 = wl.make_bias(w, 0), wl.make_bias(w, 1)
    g1 = pipe.pipe_expand(dev(W1), l1.bits, l1.K, l1.gamma, l1.group)
    g2 = pipe.pipe_expand(dev(W2), l2.bits, l2.K, l2.gamma, l2.group)
    xd = dev(x)
    for split in (None, [2, 1]):
        y1 = pipe.pipe_forward(g1, xd, split=split, bias=dev(b1))
        c1 = pipe.pipe_chain_forward([(g1, dev(b1), 0, -1, True)], xd, split=split)
        assert np.array_equal(y1.cpu().numpy(), c1.cpu().numpy())
        y2 = pipe.pipe_mlp_forward(g1, g2, pipe.PIPE_ACT_GELU, xd, split=split, bias1=dev(b1), bias2=dev(b2))
        c2 = pipe.pipe_chain_forward([(g1, dev(b1), 1, -1, True), (g2, dev(b2), 0, -1, True)], xd, split=split)
        assert np.array_equal(y2.cpu().numpy(), c2.cpu().numpy())
    g1.free(); g2.free()


def _check_chain_asymmetric(pipe, olayers, glayers, x, split, act_bits=8):
    """Teacher-forced layer by layer, then free-running, as _check_chain, under asymmetric codes."""
    L = len(olayers)
    y, acts = pipe.pipe_chain_forward_asymmetric(glayers, dev(x), split=split, return_acts=True)
    y = y.cpu().numpy()
    acts = [a.cpu().numpy() for a in acts]
    M = 1 if split is None else len(split)
    for l in range(L):
        skips = po.chain_skips(olayers, l, x, acts, M)
        if l == 0:
            ref = po.chain_layer_members(olayers[0], x, True, skips, split, None, act_bits, asymmetric=True)
        else:
            ref = po.chain_layer_members(olayers[l], acts[l - 1], False, skips, split, None, act_bits, asymmetric=True)
        if l < L - 1:
            for m in range(M):
                assert_close_fp32(acts[l][m], ref[m], tol=2e-5)
        else:
            assert_close_fp32(y, po.sum_members(ref))
    full = po.chain_forward(olayers, x, split=split, act_bits=act_bits, asymmetric=True)
    assert_close_fp32(y, full["y"], tol=3e-2, elementwise=False)
    return y


@pytest.mark.parametrize("tokens", [150, 37, 9])
@pytest.mark.parametrize("bits,K,split", [(4, 4, [2, 2]), (2, 4, [1, 1, 2]), (8, 2, None), (2, 8, [3, 3, 2])])
def test_asymmetric_chain_parity(pipe, bits, K, split, tokens):
    """Sec. 4.3's asymmetric codes in front of every layer of a residual stack: every member's hidden
    tensor is quantized over its own range (taken in the producing kernel's epilogue) with its own
    zero point; tiled and weight-streaming kernels, bins of more than 4 orders included."""
    w = wl.residual_stack(128, 2, 64, bits, K, 0.5, 16, tokens, split or (K,))
    olayers, glayers, gpu = _build(pipe, w)
    x = wl.make_input(w)
    y = _check_chain_asymmetric(pipe, olayers, glayers, x, split)
    y_again = pipe.pipe_chain_forward_asymmetric(glayers, dev(x), split=split).cpu().numpy()   # every range slot was cleared
    assert np.array_equal(y, y_again)
    # the symmetric call on the same expansions and workspace is unchanged by the asymmetric one
    _check_chain(pipe, w, olayers, glayers, x, split)
    for g in gpu:
        g.free()


def test_asymmetric_chain_variants(pipe):
    """GELU inside the chain (tensors with a negative part: a zero point between the ends), skips from
    the input and from hidden tensors on both sides of the activation, a one-sided negative input,
    4-bit activations, one layer, and both kernels forced."""
    spec = lambda o, i: wl.LayerSpec(o, i, 4, 4, 0.5, 16)
    layers = (spec(112, 112), spec(112, 112), spec(80, 112), spec(80, 80))
    chain = (("relu", 0, False), ("gelu", 0, True), ("none", -1, True), ("none", 3, True))
    w = wl.Workload(name="chain_variants", config=6, kind="chain", layers=layers, tokens=70, split=(2, 1, 1),
                    w_dist=dict(kind=0, std=0.13), x_dist=dict(kind=0), chain=chain)
    olayers, glayers, gpu = _build(pipe, w)
    x = wl.make_input(w)
    for kernel in (0, 1, 2):
        pipe.pipe_set_kernel(kernel)
        try:
            _check_chain_asymmetric(pipe, olayers, glayers, x, [2, 1, 1])
            _check_chain_asymmetric(pipe, olayers, glayers, -np.abs(x), None)
        finally:
            pipe.pipe_set_kernel(0)
    pipe.pipe_set_activation_bits(4)
    try:
        _check_chain_asymmetric(pipe, olayers, glayers, x, [2, 2], act_bits=4)
    finally:
        pipe.pipe_set_activation_bits(8)
    # one layer: the single-layer entry point
    b0 = glayers[0][1]
    y1 = pipe.pipe_chain_forward_asymmetric([(gpu[0], b0, 0, -1, True)], dev(x), split=[1, 3]).cpu().numpy()
    assert_close_fp32(y1, pipe.pipe_forward_asymmetric(gpu[0], dev(x), split=[1, 3], bias=b0).cpu().numpy(), tol=1e-6)
    assert_close_fp32(y1, po.forward_asymmetric(olayers[0].exp, x, split=[1, 3], bias=olayers[0].bias)["y"])
    # an all-zero input: every layer sees its bias only
    z = np.zeros_like(x)
    _check_chain_asymmetric(pipe, olayers, glayers, z, [2, 1, 1])
    for g in gpu:
        g.free()


@pytest.mark.parametrize("tokens", [150, 37, 9])
@pytest.mark.parametrize("bits,K,split", [(4, 4, [2, 2]), (2, 4, None), (2, 8, [3, 3, 2])])
def test_chain_with_given_scales(pipe, bits, K, split, tokens):
    """Static activation ranges inside a chain (Sec. 4: ranges fixed ahead of time): every member quantizes the
    tensor entering layer l with the given s_in[m].  With the scales a dynamic run found, the result is that
    run's, bit for bit; with other scales (some too small: codes clip) every layer matches the checker fed the
    same tensors.  Tiled, streaming and, for the small batch, the resident kernel."""
    w = wl.residual_stack(128, 2, 64, bits, K, 0.5, 16, tokens, split or (K,))
    olayers, glayers, gpu = _build(pipe, w)
    x = wl.make_input(w)
    M = 1 if split is None else len(split)
    L = len(glayers)
    y_dyn, acts = pipe.pipe_chain_forward(glayers, dev(x), split=split, return_acts=True)
    found = [None] + [[float(np.float32(np.float32(np.abs(acts[l - 1][m].cpu().numpy()).max()) / np.float32(127))) for m in range(M)]
                      for l in range(1, L)]
    given = [g + (0, 0, 1, 0, found[l]) for l, g in enumerate(glayers)]
    for resident in (True, False):
        pipe.pipe_set_decode_resident(resident)
        try:
            y_same = pipe.pipe_chain_forward(given, dev(x), split=split)
            assert pipe.pipe_resident_status() == 0
            assert torch.equal(y_same, y_dyn)
            other = [None] + [[f * (0.5 if (l + m) % 2 else 1.7) for m, f in enumerate(found[l])] for l in range(1, L)]
            g2 = [g + (0, 0, 1, 0, other[l]) for l, g in enumerate(glayers)]
            y2, a2 = pipe.pipe_chain_forward(g2, dev(x), s_x=0.05, split=split, return_acts=True)
        finally:
            pipe.pipe_set_decode_resident(1)
        a2 = [a.cpu().numpy() for a in a2]
        for l in range(L):
            ol = po.ChainLayer(olayers[l].exp, olayers[l].bias, olayers[l].act, olayers[l].skip_from, olayers[l].skip_pre_act,
                               s_in=other[l])
            skips = po.chain_skips(olayers, l, x, a2, M)
            ref = po.chain_layer_members(ol, x, True, skips, split, 0.05) if l == 0 else po.chain_layer_members(ol, a2[l - 1], False, skips, split)
            if l < L - 1:
                for m in range(M):
                    assert_close_fp32(a2[l][m], ref[m], tol=2e-5)
            else:
                assert_close_fp32(y2.cpu().numpy(), po.sum_members(ref))
    with pytest.raises(pipe.PipeError):
        bad = [g + (0, 0, 1, 0, None if l == 0 else [0.0] * M) for l, g in enumerate(glayers)]
        pipe.pipe_chain_forward(bad, dev(x), split=split)
    for g in gpu:
        g.free()


def test_chain_argument_errors(pipe):
    w = wl.residual_stack(64, 1, 32, 4, 2, 1.0, 16, 8, (2,))
    _, glayers, gpu = _build(pipe, w, with_bias=False)
    x = dev(wl.make_input(w))
    bad_last = list(glayers)
    bad_last[-1] = (bad_last[-1][0], None, 3, -1, True)          # activation on the last layer
    with pytest.raises(pipe.PipeError):
        pipe.pipe_chain_forward(bad_last, x)
    bad_skip = list(glayers)
    bad_skip[1] = (bad_skip[1][0], None, 3, 2, True)             # a skip cannot read a later tensor
    with pytest.raises(pipe.PipeError):
        pipe.pipe_chain_forward(bad_skip, x)
    bad_width = list(glayers)
    bad_width[-1] = (bad_width[-1][0], None, 0, 0, True)         # 32 outputs, skip tensor 64 wide
    with pytest.raises(pipe.PipeError):
        pipe.pipe_chain_forward(bad_width, x)
    with pytest.raises(pipe.PipeError):
        pipe.pipe_chain_forward(glayers[:2] + glayers[3:], x, split=[1, 2])   # split does not sum to K
    for g in gpu:
        g.free()


def test_full_width_stack_in_the_benchmark_launch_configuration(pipe):
    """The benchmark's residual stack at full width (8 layers, 2048 wide, ternary, K = 8, [4,4])
    on 1024 tokens with the 64-token tiles the benchmark's 4096 tokens select: every layer against
    the checker on the GPU's own earlier tensors."""
    w = wl.with_tokens(wl.CHAIN, 1024)
    olayers, glayers, gpu = _build(pipe, w, with_bias=False)
    pipe.pipe_set_token_tile(64)
    try:
        _check_chain(pipe, w, olayers, glayers, wl.make_input(w), list(w.split))
    finally:
        pipe.pipe_set_token_tile(0)
    for g in gpu:
        g.free()


def _conv_stack(pipe, geo, acts, skips, bits, K, gamma, group, seed):
    """geo: per layer (O, C_in, k, stride, pad), k = 0 for a layer applied per grid position."""
    rng = np.random.default_rng(seed)
    olayers, glayers, gpu = [], [], []
    for (o, c, k, st, pd), a, sk in zip(geo, acts, skips):
        cols = c * max(k, 1) ** 2
        Wl = (rng.standard_normal((o, cols)) * np.sqrt(2.0 / cols)).astype(np.float32)
        b = (0.3 * rng.standard_normal(o)).astype(np.float32)
        spec = wl.LayerSpec(o, cols, bits, K, gamma, group)
        oe = oracle_expand(Wl, spec)
        ge = pipe.pipe_expand(dev(Wl), bits, K, gamma, group)
        assert_expansion_equal(ge, oe)
        olayers.append(po.ChainLayer(oe, b, a, sk, True, k, k, st, pd))
        glayers.append((ge, dev(b), ACT[a], sk, True, k, k, st, pd))
        gpu.append(ge)
    return olayers, glayers, gpu


@pytest.mark.parametrize("N,H,W", [(2, 12, 12), (1, 5, 7)])
@pytest.mark.parametrize("bits,K,split", [(4, 4, [2, 2]), (2, 4, [1, 3]), (8, 2, None)])
def test_conv_residual_stack_parity(pipe, bits, K, split, N, H, W):
    """A ResNet-like stack as member chains (Fig. 2): 3x3 stem, a residual block of two 3x3
    convolutions, a strided 3x3 convolution that changes the grid, a 1x1 projection given as a
    convolution and one given as a per-position layer; teacher-forced layer by layer, then
    free-running.  Grids of 288/72 and 35/12 tokens exercise both contraction kernels."""
    C0 = 16
    geo = [(32, C0, 3, 1, 1), (32, 32, 3, 1, 1), (32, 32, 3, 1, 1), (48, 32, 3, 2, 1), (32, 48, 1, 1, 0), (16, 32, 0, 1, 0)]
    acts = ["relu", "relu", "relu", "relu", "gelu", "none"]
    skips = [-1, -1, 1, -1, -1, -1]
    olayers, glayers, gpu = _conv_stack(pipe, geo, acts, skips, bits, K, 0.5, 16, seed=300 + bits)
    rng = np.random.default_rng(17)
    x = rng.standard_normal((N, H, W, C0)).astype(np.float32)
    xt = x.reshape(N * H * W, C0)
    y, acts_g = pipe.pipe_chain_forward_conv(glayers, dev(x), split=split, return_acts=True)
    grids = po.chain_grids(olayers, (N, H, W))
    assert tuple(y.shape) == (N, grids[-1][1], grids[-1][2], 16)
    y = y.cpu().numpy().reshape(-1, 16)
    acts_g = [a.cpu().numpy().reshape(a.shape[0], -1, a.shape[-1]) for a in acts_g]
    M = 1 if split is None else len(split)
    L = len(olayers)
    for l in range(L):
        sk = po.chain_skips(olayers, l, xt, acts_g, M)
        if l == 0:
            ref = po.chain_layer_members(olayers[0], xt, True, sk, split, None, 8, grids[0])
        else:
            ref = po.chain_layer_members(olayers[l], acts_g[l - 1], False, sk, split, None, 8, grids[l])
        if l < L - 1:
            assert acts_g[l].shape == ref.shape, (l, acts_g[l].shape, ref.shape)
            for m in range(M):
                assert_close_fp32(acts_g[l][m], ref[m], tol=2e-5)
        else:
            assert_close_fp32(y, po.sum_members(ref))
    full = po.chain_forward(olayers, xt, split=split, grid=(N, H, W))
    assert_close_fp32(y, full["y"], tol=3e-2, elementwise=False)
    # a static input scale, and the same chain again (slots left clean by the first call)
    y2 = pipe.pipe_chain_forward_conv(glayers, dev(x), split=split).cpu().numpy().reshape(-1, 16)
    assert np.array_equal(y, y2)
    ys = pipe.pipe_chain_forward_conv(glayers, dev(x), s_x=0.04, split=split).cpu().numpy().reshape(-1, 16)
    fs = po.chain_forward(olayers, xt, split=split, s_x=0.04, grid=(N, H, W))
    assert_close_fp32(ys, fs["y"], tol=3e-2, elementwise=False)
    for g in gpu:
        g.free()


@pytest.mark.parametrize("N,H,W", [(2, 12, 12), (1, 5, 7)])
@pytest.mark.parametrize("bits,K,split", [(4, 4, [2, 2]), (2, 4, [1, 3]), (8, 2, None)])
def test_asymmetric_conv_chain_parity(pipe, bits, K, split, N, H, W):
    """The ResNet-like stack of test_conv_residual_stack_parity under asymmetric activation codes (Sec. 4.3):
    every member quantizes every element of its own hidden tensor over that tensor's range, and the taps of a
    3x3 window outside the image hold the zero point.  Teacher-forced layer by layer, then free-running; a
    second call (all range slots cleared) and the symmetric call on the same scratch are unchanged."""
    C0 = 16
    geo = [(32, C0, 3, 1, 1), (32, 32, 3, 1, 1), (32, 32, 3, 1, 1), (48, 32, 3, 2, 1), (32, 48, 1, 1, 0), (16, 32, 0, 1, 0)]
    acts = ["relu", "relu", "relu", "relu", "gelu", "none"]
    skips = [-1, -1, 1, -1, -1, -1]
    olayers, glayers, gpu = _conv_stack(pipe, geo, acts, skips, bits, K, 0.5, 16, seed=400 + bits)
    rng = np.random.default_rng(19)
    x = (rng.standard_normal((N, H, W, C0)) + 0.5).astype(np.float32)   # a range with both signs, off centre
    xt = x.reshape(N * H * W, C0)
    y, acts_g = pipe.pipe_chain_forward_conv_asymmetric(glayers, dev(x), split=split, return_acts=True)
    grids = po.chain_grids(olayers, (N, H, W))
    assert tuple(y.shape) == (N, grids[-1][1], grids[-1][2], 16)
    y = y.cpu().numpy().reshape(-1, 16)
    acts_g = [a.cpu().numpy().reshape(a.shape[0], -1, a.shape[-1]) for a in acts_g]
    M = 1 if split is None else len(split)
    L = len(olayers)
    for l in range(L):
        sk = po.chain_skips(olayers, l, xt, acts_g, M)
        if l == 0:
            ref = po.chain_layer_members(olayers[0], xt, True, sk, split, None, 8, grids[0], asymmetric=True)
        else:
            ref = po.chain_layer_members(olayers[l], acts_g[l - 1], False, sk, split, None, 8, grids[l], asymmetric=True)
        if l < L - 1:
            assert acts_g[l].shape == ref.shape, (l, acts_g[l].shape, ref.shape)
            for m in range(M):
                # two large terms cancel in the kernels' evaluation: the error follows the tensor's scale
                d = np.abs(acts_g[l][m].astype(np.float64) - ref[m])
                assert d.max() <= 2e-5 * np.abs(ref[m]).max() + 1e-30
                assert_close_fp32(acts_g[l][m], ref[m])
        else:
            assert_close_fp32(y, po.sum_members(ref))
    full = po.chain_forward(olayers, xt, split=split, grid=(N, H, W), asymmetric=True)
    assert_close_fp32(y, full["y"], tol=3e-2, elementwise=False)
    y2 = pipe.pipe_chain_forward_conv_asymmetric(glayers, dev(x), split=split).cpu().numpy().reshape(-1, 16)
    assert np.array_equal(y, y2)
    ys = pipe.pipe_chain_forward_conv(glayers, dev(x), split=split).cpu().numpy().reshape(-1, 16)
    fs = po.chain_forward(olayers, xt, split=split, grid=(N, H, W))
    assert_close_fp32(ys, fs["y"], tol=3e-2, elementwise=False)
    # the flat entry point has no grid: it refuses convolution layers
    with pytest.raises(pipe.PipeError):
        pipe.pipe_chain_forward_asymmetric(glayers, dev(xt), split=split)
    for g in gpu:
        g.free()


def test_conv_chain_argument_errors(pipe):
    geo = [(32, 16, 3, 1, 1), (32, 32, 3, 2, 1), (16, 32, 0, 1, 0)]
    olayers, glayers, gpu = _conv_stack(pipe, geo, ["relu", "relu", "none"], [-1, -1, -1], 4, 2, 1.0, 16, seed=5)
    x = dev(np.zeros((1, 6, 6, 16), dtype=np.float32))
    # the flat entry point has no grid to convolve over
    with pytest.raises(pipe.PipeError):
        pipe.pipe_chain_forward(glayers, x.reshape(36, 16))
    # a skip across the strided layer joins different grids
    bad = list(glayers)
    bad[1] = bad[1][:3] + (1,) + bad[1][4:]
    with pytest.raises(pipe.PipeError):
        pipe.pipe_chain_forward_conv(bad, x)
    # kernel larger than the (unpadded) grid
    nopad = [glayers[0][:5] + (3, 3, 1, 0)] + glayers[1:]
    with pytest.raises(pipe.PipeError):
        pipe.pipe_chain_forward_conv(nopad, dev(np.zeros((1, 2, 2, 16), dtype=np.float32)))
    y = pipe.pipe_chain_forward_conv(glayers, x)
    assert tuple(y.shape) == (1, 3, 3, 16)
    for g in gpu:
        g.free()
