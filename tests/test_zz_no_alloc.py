"""The entry point that allocates nothing (pipe_forward_noalloc) against pipe_forward: same
results bit for bit, on calls in a row that share the fixed scratch array, the later ones with
smaller inputs; sizes beyond the array and missing schedules are refused with their own codes."""
import pytest
import torch

from paper_2311_15806_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _layer(pipe, out_div, in_div):
    w = wl.scaled(wl.C4, out_div=out_div, in_div=in_div)
    spec = w.layers[0]
    W = torch.from_numpy(wl.make_weight(w, 0)).cuda()
    return w, spec, pipe.pipe_expand(W, spec.bits, spec.K, spec.gamma, spec.group)


def _x(w, T, scale=1.0):
    return torch.from_numpy(wl.make_input(wl.with_tokens(w, T))).cuda() * scale


def test_no_alloc_matches_forward_on_calls_in_a_row():
    import paper_2311_15806_amd.binding as pipe
    w, spec, g = _layer(pipe, 4, 4)
    split = [1, spec.K - 1]
    bias = torch.linspace(-1.0, 1.0, spec.out_features, device="cuda")
    pipe.pipe_prepare(g, 700, split=split)                    # the tile schedule of this grouping
    # tiled kernel (two launches of the quantizer), then smaller inputs: the streaming kernel with the
    # one-launch quantizer, a ragged block, a single token (quantized inside the contraction)
    for T, scale in ((700, 1.0), (300, 0.25), (64, 3.0), (16, 1.0), (7, 0.5), (1, 2.0), (129, 1.0)):
        x = _x(w, T, scale)
        ref = pipe.pipe_forward(g, x, split=split, bias=bias)
        out = torch.full_like(ref, float("nan"))
        pipe.pipe_forward_noalloc(g, x, out, split=split, bias=bias)
        torch.cuda.synchronize()
        assert torch.equal(out, ref), "T = %d" % T
    # a static scale and members kept apart, after the dynamic calls above
    x = _x(w, 40)
    ref = pipe.pipe_forward(g, x, s_x=0.05, split=split, reduce_members=False)
    out = torch.empty_like(ref)
    pipe.pipe_forward_noalloc(g, x, out, s_x=0.05, split=split, reduce_members=False)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)
    g.free()


def test_no_alloc_limits_and_missing_schedule():
    import paper_2311_15806_amd.binding as pipe
    w, spec, g = _layer(pipe, 4, 1)                               # 4096 input features
    out = torch.empty((2112, spec.out_features), device="cuda")
    with pytest.raises(pipe.PipeError) as ei:                     # 2112 x 4096 bytes > 8 MiB
        pipe.pipe_forward_noalloc(g, _x(w, 2112), out)
    assert ei.value.code == -7
    out = torch.empty((200, spec.out_features), device="cuda")
    with pytest.raises(pipe.PipeError) as ei:                     # no tile schedule yet: it would have to build one
        pipe.pipe_forward_noalloc(g, _x(w, 200), out)
    assert ei.value.code == -6
    x = _x(w, 200)
    ref = pipe.pipe_forward(g, x)                                 # builds it
    pipe.pipe_forward_noalloc(g, x, out)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)
    x = _x(w, 2048)                                               # the largest batch of this width that fits
    out = torch.empty((2048, spec.out_features), device="cuda")
    pipe.pipe_forward_noalloc(g, x, out)
    torch.cuda.synchronize()
    assert torch.equal(out, pipe.pipe_forward(g, x))
    g.free()
