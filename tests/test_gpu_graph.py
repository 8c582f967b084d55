"""The layer entry points under HIP graph capture: they allocate nothing and record only kernel launches,
so a captured forward + backward must replay to the same bits as the eager calls, every time."""
import numpy as np
import pytest
import torch

from paper_2505_14669_amd import synth

pytestmark = pytest.mark.gpu


def test_linear_fwd_bwd_replays_bit_identically_from_a_graph():
    import gpu_util as G
    L = synth.make_layer(1, 0)
    lin = G.Linear(L["x"], L["w"])
    dy = G.to_dev(L["dy"])
    seed = 77

    lin.fwd()
    lin.bwd(dy, seed, 0)
    eager = [G.to_host(t, np.uint32).copy() for t in (lin.y, lin.dx, lin.dw)]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):       # warm-up on the capture stream, as torch asks for
        lin.fwd()
        lin.bwd(dy, seed, 0)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lin.fwd()
        lin.bwd(dy, seed, 0)

    for replay in range(3):
        for t in (lin.y, lin.dx, lin.dw):      # eager work between replays: poison the outputs
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, t, want in zip(("y", "dx", "dw"), (lin.y, lin.dx, lin.dw), eager):
            got = G.to_host(t, np.uint32)
            assert np.array_equal(got, want), f"replay {replay}: {name} differs from the eager result"
