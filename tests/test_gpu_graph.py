"""A forward captured into a HIP graph replays correctly: every replay, with eager work and
synchronizations between replays, equals the eager result bit for bit.  The library keeps its
scratch per stream, so a capture runs on the stream that was warmed up (or prepared with
pipe_prepare*): a first call on a stream under capture is refused, not served by allocating."""
import numpy as np
import pytest
import torch

from paper_2311_15806_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("T", [1, 7, 200])
def test_forward_graph_replays(T):
    import paper_2311_15806_amd.binding as pipe
    w = wl.scaled(wl.C4, out_div=4, in_div=4)
    spec = w.layers[0]
    W = torch.from_numpy(wl.make_weight(w, 0)).cuda()
    g = pipe.pipe_expand(W, spec.bits, spec.K, spec.gamma, spec.group)
    xs = [torch.from_numpy(wl.make_input(wl.with_tokens(w, T))).cuda() * s for s in (1.0, 0.5, 3.0)]
    x = xs[0].clone()
    out = torch.empty((T, spec.out_features), device="cuda")
    eager = []
    for xi in xs:
        eager.append(pipe.pipe_forward(g, xi).clone())
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        pipe.pipe_forward(g, x, out=out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        pipe.pipe_forward(g, x, out=out)
    for rep in range(6):
        i = rep % 3
        x.copy_(xs[i])
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager[i]), "replay %d differs" % rep
        # eager work of the program between replays (same workspace, other input)
        other = pipe.pipe_forward(g, xs[(i + 1) % 3])
        torch.cuda.synchronize()
        assert torch.equal(other, eager[(i + 1) % 3])
    g.free()


@pytest.mark.parametrize("T", [9, 200])
def test_chain_graph_replays(T):
    """A member chain (quantizers, contractions with fused activation and skip, slot clearing
    inside the kernels) captured once and replayed with other inputs: no replay may depend on
    what the previous one left in the max and code-sum slots."""
    import paper_2311_15806_amd.binding as pipe
    w = wl.residual_stack(128, 2, 64, 4, 4, 0.5, 16, T, (2, 2))
    gs = [pipe.pipe_expand(torch.from_numpy(wl.make_weight(w, l)).cuda(), s.bits, s.K, s.gamma, s.group)
          for l, s in enumerate(w.layers)]
    act = {"none": 0, "gelu": 1, "relu": 3}
    layers = [(g, None, act[c[0]], c[1], c[2]) for g, c in zip(gs, w.chain)]
    xs = [torch.from_numpy(wl.make_input(w)).cuda() * s for s in (1.0, 0.25, 5.0)]
    x = xs[0].clone()
    out = torch.empty((T, w.layers[-1].out_features), device="cuda")
    eager = [pipe.pipe_chain_forward(layers, xi, split=[2, 2]).clone() for xi in xs]
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        pipe.pipe_chain_forward(layers, x, split=[2, 2], out=out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        pipe.pipe_chain_forward(layers, x, split=[2, 2], out=out)
    for rep in range(6):
        i = rep % 3
        x.copy_(xs[i])
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager[i]), "replay %d differs" % rep
        other = pipe.pipe_chain_forward(layers, xs[(i + 1) % 3], split=[2, 2])
        torch.cuda.synchronize()
        assert torch.equal(other, eager[(i + 1) % 3])
    for g in gs:
        g.free()


@pytest.mark.parametrize("kind,T", [("gelu", 1), ("gelu", 11), ("gelu", 300), ("gated", 1), ("gated", 11), ("gated", 300)])
def test_mlp_graph_replays(kind, T):
    """The two-layer MLP call (quantizers, both contractions, hidden maxima raised in layer 1's
    epilogue and consumed by the hidden quantizer, slots cleared inside the kernels) captured once
    and replayed with other inputs, for a single token (layer 1 quantizes its input itself),
    decode-sized and tiled batches."""
    import paper_2311_15806_amd.binding as pipe
    base = wl.C3 if kind == "gelu" else wl.C5
    w = wl.scaled(base, out_div=8, in_div=8, tokens=T)
    split = list(w.split) if w.split else None
    es = [pipe.pipe_expand(torch.from_numpy(wl.make_weight(w, l)).cuda(), s.bits, s.K, s.gamma, s.group)
          for l, s in enumerate(w.layers)]
    act = pipe.PIPE_ACT_GELU if kind == "gelu" else pipe.PIPE_ACT_SILU_GATED
    xs = [torch.from_numpy(wl.make_input(w)).cuda() * s for s in (1.0, 0.3, 4.0)]
    x = xs[0].clone()
    out = torch.empty((T, w.layers[-1].out_features), device="cuda")
    eager = [pipe.pipe_mlp_forward(es[0], es[1], act, xi, split=split).clone() for xi in xs]
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        pipe.pipe_mlp_forward(es[0], es[1], act, x, split=split, out=out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        pipe.pipe_mlp_forward(es[0], es[1], act, x, split=split, out=out)
    for rep in range(6):
        i = rep % 3
        x.copy_(xs[i])
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager[i]), "replay %d differs" % rep
        other = pipe.pipe_mlp_forward(es[0], es[1], act, xs[(i + 1) % 3], split=split)
        torch.cuda.synchronize()
        assert torch.equal(other, eager[(i + 1) % 3])
    for e in es:
        e.free()


@pytest.mark.parametrize("T", [16, 2048])
def test_several_steps_in_one_graph_keep_their_order(T):
    """The benchmark's form of a timed region: K forward steps captured into ONE graph.  Every
    step reads the shared workspace the previous one wrote (activation codes, maxima, code sums),
    so a step that started before its predecessor had finished would change a result.  Steps
    alternate between inputs and write to their own outputs; each must equal its eager result.
    Full-size layer of the headline workload."""
    import paper_2311_15806_amd.binding as pipe
    w = wl.with_tokens(wl.C4, T)
    spec = w.layers[0]
    W = torch.from_numpy(wl.make_weight(w, 0)).cuda()
    g = pipe.pipe_expand(W, spec.bits, spec.K, spec.gamma, spec.group)
    x0 = torch.from_numpy(wl.make_input(w)).cuda()
    xs = [x0, x0 * 0.37, torch.roll(x0, 1, dims=0) * 2.5]
    eager = [pipe.pipe_forward(g, xi).clone() for xi in xs]
    K = 9
    outs = [torch.empty_like(eager[0]) for _ in range(K)]
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        pipe.pipe_forward(g, xs[0], out=outs[0])
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for i in range(K):
            pipe.pipe_forward(g, xs[i % 3], out=outs[i])
    for rep in range(3):
        for o in outs:
            o.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for i in range(K):
            assert torch.equal(outs[i], eager[i % 3]), "replay %d, step %d differs" % (rep, i)
    g.free()


@pytest.mark.parametrize("T", [7, 200])
def test_asymmetric_forward_graph_replays(T):
    """The asymmetric layer (range reduction, quantizer, bias kernel that also clears the range
    slots, contraction) captured once and replayed with inputs of other ranges."""
    import paper_2311_15806_amd.binding as pipe
    w = wl.scaled(wl.C4, out_div=4, in_div=4)
    spec = w.layers[0]
    W = torch.from_numpy(wl.make_weight(w, 0)).cuda()
    g = pipe.pipe_expand(W, spec.bits, spec.K, spec.gamma, spec.group)
    x0 = torch.from_numpy(wl.make_input(wl.with_tokens(w, T))).cuda()
    xs = [torch.relu(x0), x0 * 0.5 + 1.0, -torch.relu(x0) * 3.0]
    x = xs[0].clone()
    out = torch.empty((T, spec.out_features), device="cuda")
    eager = [pipe.pipe_forward_asymmetric(g, xi).clone() for xi in xs]
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        pipe.pipe_forward_asymmetric(g, x, out=out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        pipe.pipe_forward_asymmetric(g, x, out=out)
    for rep in range(6):
        i = rep % 3
        x.copy_(xs[i])
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager[i]), "replay %d differs" % rep
        other = pipe.pipe_forward(g, xs[(i + 1) % 3])          # symmetric eager work on the same workspace
        torch.cuda.synchronize()
    g.free()


def test_conv_graph_replays():
    """The convolution call (range reduction, element-wise codes, code-sum clearing, patch gather,
    contraction) captured once and replayed with other inputs."""
    import paper_2311_15806_amd.binding as pipe
    w = wl.scaled(wl.C2, out_div=4, in_div=4, tokens=4 * 14 * 14)
    spec, c = w.layers[0], w.conv
    W = torch.from_numpy(wl.make_weight(w, 0)).cuda()
    g = pipe.pipe_expand(W, spec.bits, spec.K, spec.gamma, spec.group)
    x0 = torch.from_numpy(wl.make_input(w)).cuda()
    xs = [x0, x0 * 0.3, torch.flip(x0, dims=[0]) * 2.0]
    split = list(w.split)
    args = (c["kh"], c["kw"], c["stride"], c["pad"])
    eager = [pipe.pipe_forward_conv2d(g, xi, *args, split=split).clone() for xi in xs]
    x = xs[0].clone()
    out = torch.empty_like(eager[0])
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        pipe.pipe_forward_conv2d(g, x, *args, split=split, out=out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        pipe.pipe_forward_conv2d(g, x, *args, split=split, out=out)
    for rep in range(6):
        i = rep % 3
        x.copy_(xs[i])
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager[i]), "replay %d differs" % rep
        other = pipe.pipe_forward_conv2d(g, xs[(i + 1) % 3], *args, split=split)
        torch.cuda.synchronize()
        assert torch.equal(other, eager[(i + 1) % 3])
    g.free()


def _c4_quarter(pipe, T):
    w = wl.scaled(wl.C4, out_div=4, in_div=4)
    spec = w.layers[0]
    W = torch.from_numpy(wl.make_weight(w, 0)).cuda()
    x = torch.from_numpy(wl.make_input(wl.with_tokens(w, T))).cuda()
    return spec, W, x


@pytest.mark.parametrize("T", [1, 16, 200])
def test_capture_with_no_prior_eager_call(T):
    """pipe_prepare does what a first call would (scratch of the stream, tile schedule); the very
    first forward of a fresh expansion on a fresh stream is then captured, and every replay equals
    the eager result computed afterwards."""
    import paper_2311_15806_amd.binding as pipe
    spec, W, x0 = _c4_quarter(pipe, T)
    g = pipe.pipe_expand(W, spec.bits, spec.K, spec.gamma, spec.group)
    split = [1, spec.K - 1]
    x = x0.clone()
    out = torch.empty((T, spec.out_features), device="cuda")
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        pipe.pipe_prepare(g, T, split=split)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        pipe.pipe_forward(g, x, split=split, out=out)
    for rep, scale in enumerate((1.0, 0.4, 2.5)):
        x.copy_(x0 * scale)
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        eager = pipe.pipe_forward(g, x, split=split)
        torch.cuda.synchronize()
        assert torch.equal(out, eager), "replay %d differs" % rep
    g.free()


def test_capture_of_mlp_and_chain_with_no_prior_eager_call():
    import paper_2311_15806_amd.binding as pipe
    T = 300
    w = wl.scaled(wl.C5, out_div=8, in_div=8, tokens=T)
    split = list(w.split)
    es = [pipe.pipe_expand(torch.from_numpy(wl.make_weight(w, l)).cuda(), s.bits, s.K, s.gamma, s.group)
          for l, s in enumerate(w.layers)]
    x = torch.from_numpy(wl.make_input(w)).cuda()
    out = torch.empty((T, w.layers[-1].out_features), device="cuda")
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        pipe.pipe_prepare_mlp(es[0], es[1], pipe.PIPE_ACT_SILU_GATED, T, split=split)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        pipe.pipe_mlp_forward(es[0], es[1], pipe.PIPE_ACT_SILU_GATED, x, split=split, out=out)
    for rep in range(2):
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, pipe.pipe_mlp_forward(es[0], es[1], pipe.PIPE_ACT_SILU_GATED, x, split=split))
    for e in es:
        e.free()
    # a member chain on a fresh stream
    wc = wl.residual_stack(128, 2, 64, 4, 4, 0.5, 16, T, (2, 2))
    gs = [pipe.pipe_expand(torch.from_numpy(wl.make_weight(wc, l)).cuda(), s.bits, s.K, s.gamma, s.group)
          for l, s in enumerate(wc.layers)]
    act = {"none": 0, "gelu": 1, "relu": 3}
    layers = [(g, None, act[c[0]], c[1], c[2]) for g, c in zip(gs, wc.chain)]
    xc = torch.from_numpy(wl.make_input(wc)).cuda()
    outc = torch.empty((T, wc.layers[-1].out_features), device="cuda")
    side2 = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side2):
        pipe.pipe_prepare_chain(layers, T, split=[2, 2])
    graph2 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph2, stream=side2):
        pipe.pipe_chain_forward(layers, xc, split=[2, 2], out=outc)
    for rep in range(2):
        outc.zero_()
        graph2.replay()
        torch.cuda.synchronize()
        assert torch.equal(outc, pipe.pipe_chain_forward(layers, xc, split=[2, 2]))
    for g in gs:
        g.free()


def test_unprepared_capture_is_refused_not_served():
    """A first call on a stream under capture would have to allocate: it returns PIPE_ENOTREADY,
    launches nothing, and the same call succeeds once prepared."""
    import paper_2311_15806_amd.binding as pipe
    spec, W, x = _c4_quarter(pipe, 200)
    g = pipe.pipe_expand(W, spec.bits, spec.K, spec.gamma, spec.group)
    out = torch.empty((200, spec.out_features), device="cuda")
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    code = None
    with torch.cuda.graph(graph, stream=side):
        try:
            pipe.pipe_forward(g, x, out=out)
        except pipe.PipeError as exc:
            code = exc.code
    assert code == -6
    with torch.cuda.stream(side):
        pipe.pipe_prepare(g, 200)
    graph2 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph2, stream=side):
        pipe.pipe_forward(g, x, out=out)
    graph2.replay()
    torch.cuda.synchronize()
    assert torch.equal(out, pipe.pipe_forward(g, x))
    g.free()


def test_replay_after_a_larger_eager_call_on_the_same_stream():
    """The scratch of a stream grows for a larger batch; the block a graph captured earlier keeps
    its address (blocks are retired, never freed), so the replay still equals the eager result."""
    import paper_2311_15806_amd.binding as pipe
    spec, W, x_small = _c4_quarter(pipe, 16)
    _, _, x_big = _c4_quarter(pipe, 3000)
    g = pipe.pipe_expand(W, spec.bits, spec.K, spec.gamma, spec.group)
    out = torch.empty((16, spec.out_features), device="cuda")
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        pipe.pipe_prepare(g, 16)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        pipe.pipe_forward(g, x_small, out=out)
    graph.replay()
    torch.cuda.synchronize()
    first = out.clone()
    with torch.cuda.stream(side):
        big = pipe.pipe_forward(g, x_big)          # grows the stream's scratch
        big2 = pipe.pipe_forward(g, x_big * 0.5)   # and uses the new block
    torch.cuda.synchronize()
    out.zero_()
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(out, first) and torch.equal(out, pipe.pipe_forward(g, x_small))
    assert bool(torch.isfinite(big).all()) and bool(torch.isfinite(big2).all())
    g.free()


def test_two_expansions_on_two_streams_at_once():
    """Calls on different streams use disjoint scratch: two expansions driven from two streams
    without any ordering between them give the results of the serial run, bit for bit."""
    import paper_2311_15806_amd.binding as pipe
    spec, W, xa = _c4_quarter(pipe, 300)
    _, _, xb = _c4_quarter(pipe, 16)
    ga = pipe.pipe_expand(W, spec.bits, spec.K, spec.gamma, spec.group)
    gb = pipe.pipe_expand(W * 0.5, spec.bits, spec.K, spec.gamma, spec.group)
    ref_a = [pipe.pipe_forward(ga, xa * s).clone() for s in (1.0, 0.3)]
    ref_b = [pipe.pipe_forward(gb, xb * s).clone() for s in (1.0, 0.3)]
    torch.cuda.synchronize()
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    xs_a, xs_b = [xa * 1.0, xa * 0.3], [xb * 1.0, xb * 0.3]
    torch.cuda.synchronize()
    outs_a, outs_b = [], []
    for rep in range(20):
        with torch.cuda.stream(sa):
            outs_a.append(pipe.pipe_forward(ga, xs_a[rep % 2]))
        with torch.cuda.stream(sb):
            outs_b.append(pipe.pipe_forward(gb, xs_b[rep % 2]))
            outs_b.append(pipe.pipe_forward(gb, xs_b[(rep + 1) % 2]))
    torch.cuda.synchronize()
    for rep in range(20):
        assert torch.equal(outs_a[rep], ref_a[rep % 2]), "stream a, call %d" % rep
        assert torch.equal(outs_b[2 * rep], ref_b[rep % 2]) and torch.equal(outs_b[2 * rep + 1], ref_b[(rep + 1) % 2])
    ga.free(); gb.free()
