"""The entry point that allocates nothing (gvote_union_compact_static: stage 4 on the library's static
scratch array) against gvote_union_compact on the same row masks: two calls in a row, the second with a
smaller input, every output compared bit for bit."""
import numpy as np
import pytest
import torch

import parity_util as U
from synth import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(g, wl, seed):
    items = W.make_items(wl, "cpu")
    b = U.batch_from(g, wl, U.to_device(items, DEV))
    pipe = g.Pipeline(b, wl.S, wl.p)
    rng = np.random.default_rng(seed)
    words = [torch.tensor((rng.random(n * 32) < 0.03).reshape(n, 32).dot(1 << np.arange(32, dtype=np.int64)).astype(np.uint32).view(np.int32))
             for n in pipe.mask_words]
    pipe.rowmask.copy_(torch.cat(words))
    pipe.compact()                                       # the existing entry point (caller's workspace)
    torch.cuda.synchronize()
    want = [t.clone() for t in (pipe.union_mask, pipe.budget, pipe.offsets, pipe.k_out, pipe.v_out, pipe.idx_out, pipe.overflow)]
    n = int(pipe.offsets[-1].item())
    for t in (pipe.union_mask, pipe.budget, pipe.offsets, pipe.k_out, pipe.v_out, pipe.idx_out):
        t.zero_()
    pipe.overflow.fill_(7)
    g.union_compact_static(b, wl.S, pipe.rowmask, pipe.union_mask, pipe.budget, pipe.offsets, pipe.k_out, pipe.v_out,
                           pipe.idx_out, pipe.capacity, pipe.overflow)
    torch.cuda.synchronize()
    got = (pipe.union_mask, pipe.budget, pipe.offsets, pipe.k_out, pipe.v_out, pipe.idx_out, pipe.overflow)
    assert n > 0 and int(want[6].item()) == 0
    for name, a, c in zip(("union", "budget", "offsets", "k_out", "v_out", "idx", "overflow"), want, got):
        if name in ("k_out", "v_out", "idx"):
            a, c = a[:n], c[:n]
        assert torch.equal(a, c), name
    return n


def test_static_scratch_entry_point_matches_the_workspace_one():
    import paper_2509_03136_amd as g
    g.lib()
    assert torch.cuda.is_available()
    big = W.scaled(W.config(5), lengths=(5000, 2049, 700), n_planted=(20, 5, 3), S=4)
    small = W.scaled(W.config(5), lengths=(333, 64), n_planted=(2, 1), S=4)
    n1 = _both(g, big, 1)
    n2 = _both(g, small, 2)              # smaller input right after: nothing of the first call may leak in
    assert n2 < n1
    # a call too large for the scratch array is refused on the host
    huge = (g.Item * 1)()
    it = huge[0]
    it.hidden, it.hidden_row_stride, it.w_q, it.k, it.v = 0x1000, 4096, 0x2000, 0x3000, 0x4000
    it.kv_tok_stride, it.kv_head_stride, it.L, it.n_skip, it.pos0, it.n_future = 1024, 128, 1 << 30, 4, 1 << 30, 1
    sh = g.Shape(4096, 32, 8, 128, g.BF16, 5e5)
    import ctypes as C
    rc = g.lib().gvote_union_compact_static(C.byref(sh), huge, 1, 4, 0x100, 0x200, 0x300, 0x400, 0x500, 0x600, None,
                                            10, 0x700, None)
    assert rc == 5
