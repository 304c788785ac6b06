"""The hot calls allocate nothing and never synchronise, so a caller may record
them into a HIP graph.  A decode step (smoe_forward) and the five separate calls
are captured and replayed several times with ordinary eager work and
synchronisations between the replays; every replay must reproduce the eager
result bit for bit, and the eager result is checked against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2308_15030_amd import workloads as wl
from harness import Case, max_abs_rel, to_dev, to_host, values

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("fused", [True, False])
def test_layer_replays_from_a_graph(fused):
    cfg = wl.MoEConfig("graph", E=16, K=4, d_model=128, d_ff=256, T=96, dtype=wl.BF16, seed=9)
    c = Case(cfg, router_scale=10.0)
    L, T = c.L, c.T
    fwd = L.forward_fused if fused else L.forward
    x_in = torch.empty_like(c.d_x)
    inputs = [c.d_x, to_dev(wl.hidden_states(cfg.scaled(seed=10), 0)), to_dev(wl.hidden_states(cfg.scaled(seed=11), 0))]
    names = ("slot", "perm", "offsets", "count", "score", "out")

    def eager(x):
        x_in.copy_(x)
        fwd(x_in, T, accumulate=0)
        torch.cuda.synchronize()
        return {n: to_host(getattr(L, n)).copy() for n in names}

    want = [eager(x) for x in inputs]                       # also warms up everything that runs once per bind
    ref = oracle.layer_forward(c.x, c.Wr, *c.slot_weights_host(), c.e2s)
    ok = ~ref["ambiguous"]
    assert np.array_equal(want[0]["slot"][ok], ref["slot"][ok])
    assert max_abs_rel(values(want[0]["out"], cfg.dtype)[ok], values(ref["out"], cfg.dtype)[ok]) <= 2e-2

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            fwd(x_in, T, accumulate=0)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for rep in range(3):
        for i, x in enumerate(inputs):
            for n in names:                                  # eager work between the replays
                getattr(L, n).fill_(0)
            x_in.copy_(x)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for n in names:
                assert np.array_equal(to_host(getattr(L, n)), want[i][n]), (rep, i, n)
    c.L.close()
