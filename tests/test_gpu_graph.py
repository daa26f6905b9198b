"""A forward captured into a HIP graph replays correctly: every replay, with eager work and
synchronizations between replays, equals the eager result bit for bit."""
import numpy as np
import pytest
import torch

from paper_2311_15806_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("T", [7, 200])
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
    with torch.cuda.graph(graph):
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
