"""The four stage calls only enqueue kernels on the caller's stream (no allocation, no memset, no
synchronisation), so a caller may record them into a HIP graph.  The graph is replayed several times, with
eager work and synchronisations between the replays, and every replay must reproduce the eager result."""
import numpy as np
import pytest
import torch

import parity_util as U
from synth import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def g():
    import paper_2509_03136_amd as g
    g.lib()
    assert torch.cuda.is_available()
    return g


@pytest.mark.parametrize("cfg", [1, 5])
def test_stage_calls_replay_from_a_graph(g, cfg):
    wl = W.config(1) if cfg == 1 else W.scaled(W.config(5), lengths=(1100, 333, 2049, 64), n_planted=(8, 3, 200, 1))
    items = U.to_device(W.make_items(wl, "cpu"), DEV)
    b = U.batch_from(g, wl, items)
    pipe = g.Pipeline(b, wl.S, wl.p, ddof=wl.ddof)

    def snapshot():
        torch.cuda.synchronize()
        n = int(pipe.offsets[-1].item())
        return dict(mu=pipe.mu.clone(), q=pipe.q.clone(), rowmask=pipe.rowmask.clone(), union=pipe.union_mask.clone(),
                    budget=pipe.budget.clone(), offsets=pipe.offsets.clone(), k=pipe.k_out[:n].clone(),
                    v=pipe.v_out[:n].clone(), idx=pipe.idx_out[:n].clone())

    def scrub():      # eager work between replays: the outputs are overwritten, so a replay has to produce them again
        for t in (pipe.mu, pipe.var, pipe.q, pipe.rowmask, pipe.union_mask, pipe.budget, pipe.offsets, pipe.k_out, pipe.v_out,
                  pipe.idx_out):
            t.fill_(1)
        torch.cuda.synchronize()

    pipe.run()
    want = snapshot()
    assert int(want["budget"].sum().item()) > 0
    scrub()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):       # one warm-up on the capture stream (first-use set-up must not fall into the capture)
        pipe.run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        pipe.run()
    for rep in range(3):
        scrub()
        graph.replay()
        got = snapshot()
        for key in want:
            assert torch.equal(got[key], want[key]), (rep, key)
