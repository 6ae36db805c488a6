"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
uses (inputs generated on the device, all items in one batch).  The oracle cannot redo whole stacks in
a test's time, so it recomputes SAMPLED outputs (chosen items / query rows, end to end from the same
stored inputs) and the rest is checked through properties that hold at any size: the union is the OR of
the row masks, budgets are its popcounts, offsets their prefix sums, the packed cache is the rows the
union names, in order."""
import sys

import numpy as np
import pytest
import torch

import oracle as O
import parity_util as U
from synth import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module")
def g():
    import paper_2509_03136_amd as g
    g.lib()
    assert torch.cuda.is_available()
    return g


def _run(g, wl):
    items = W.make_items(wl, DEV)
    torch.cuda.synchronize()
    b = U.batch_from(g, wl, items)
    pipe = g.Pipeline(b, wl.S, wl.p, ddof=wl.ddof)
    pipe.fit()
    pipe.sample()
    pipe.select()
    torch.cuda.synchronize()
    pipe.n_fallback = pipe.fallback_rows()      # lives in the workspace: read before the next stage reuses it
    pipe.compact()
    torch.cuda.synchronize()
    return items, pipe


def _offsets(words_per_item):
    return np.concatenate([[0], np.cumsum(words_per_item)])


def _structure_checks(wl, items, pipe, sample_items):
    """Size-independent properties on every item (cheap ones) and on sampled items (bit-level ones)."""
    budget = pipe.budget.cpu().numpy()
    offsets = pipe.offsets.cpu().numpy()
    assert int(pipe.overflow.item()) == 0
    assert np.array_equal(offsets, np.concatenate([[0], np.cumsum(budget.reshape(-1).astype(np.int64))]))
    assert np.all(budget >= 1) and np.all(budget <= np.array(wl.lengths)[:, None])
    moff, uoff = _offsets(pipe.mask_words), _offsets(pipe.union_words)
    for i in sample_items:
        L = wl.lengths[i]
        gm = U.unpack_rows(pipe.rowmask[moff[i]:moff[i + 1]], pipe.rows, L).reshape(wl.S, wl.n_q_heads, L)
        um = U.unpack_rows(pipe.union_mask[uoff[i]:uoff[i + 1]], wl.n_kv_heads, L)
        gu, gb = O.union_vote(gm, wl.n_kv_heads)
        assert np.array_equal(um, gu) and np.array_equal(budget[i], gb)
        assert np.all(gm.sum(-1) >= 1)
        k, v = items[i]["k"], items[i]["v"]
        for h in range(wl.n_kv_heads):
            lo, hi = offsets[i * wl.n_kv_heads + h], offsets[i * wl.n_kv_heads + h + 1]
            idx = torch.tensor(np.nonzero(um[h])[0], device=DEV)
            assert torch.equal(pipe.idx_out[lo:hi].long(), idx)
            assert torch.equal(pipe.k_out[lo:hi], k[idx, h]) and torch.equal(pipe.v_out[lo:hi], v[idx, h])
    return moff


def _oracle_rows(wl, it, rows):
    """Oracle logits of the sampled query rows of one item, from the item's stored inputs."""
    cpu = {k: (v.cpu() if isinstance(v, torch.Tensor) else v) for k, v in it.items()}
    r = U.oracle_item(wl, cpu, upto="q")
    k = U.f32np(cpu["k"]).astype(np.float64)
    G = wl.group
    out = {}
    for (s, h) in rows:
        out[(s, h)] = k[:, h // G, :] @ r["q_tilde"][s, h] / np.sqrt(wl.d_k)
    return r, out


def _check_sampled_rows(wl, it, pipe, item_index, moff, rows):
    L = wl.lengths[item_index]
    ref, lg = _oracle_rows(wl, it, rows)
    gm = U.unpack_rows(pipe.rowmask[moff[item_index]:moff[item_index + 1]], pipe.rows, L).reshape(wl.S, wl.n_q_heads, L)
    tol, p = U.TOL[wl.dtype], U.p32(wl.p)
    boundary = 0
    for (s, h), l in lg.items():
        must, may = U.band_sets(l, p, tol)
        got = gm[s, h]
        assert not (must & ~got).any() and not (got & ~may).any(), (item_index, s, h)
        boundary += int((got ^ O.top_p_select(l, p)).sum())
        m = l.max()
        assert abs(float(pipe.row_max[item_index, s * wl.n_q_heads + h]) - m) <= tol * (1 + abs(m))
    mu = pipe.mu[item_index].cpu().numpy()
    assert np.all(np.abs(mu - ref["mu"]) <= 1e-5 * np.maximum(np.abs(ref["mu"]), np.sqrt(ref["var"])) + 1e-7)
    return boundary


def test_config3_full_stack(g):
    wl = W.config(3)
    say("cfg3 full: 32 layers x 32768")
    items, pipe = _run(g, wl)
    moff = _structure_checks(wl, items, pipe, sample_items=(0, 17))
    assert pipe.n_fallback <= 8
    # two layers end to end against the oracle
    boundary = 0
    for i in (5, 31):
        cpu = {k: (v.cpu() if isinstance(v, torch.Tensor) else v) for k, v in items[i].items()}
        ref = U.oracle_item(wl, cpu)
        L = wl.lengths[i]
        gm = U.unpack_rows(pipe.rowmask[moff[i]:moff[i + 1]], pipe.rows, L).reshape(wl.S, wl.n_q_heads, L)
        boundary += U.check_rowmask_sandwich(gm, ref["logits"], U.p32(wl.p), U.TOL[wl.dtype])
        gb = pipe.budget[i].cpu().numpy()
        say(f"  layer {i}: budget gpu {gb.tolist()} oracle {ref['budget'].tolist()}")
        assert np.all(np.abs(gb - ref["budget"]) <= 0.02 * ref["budget"] + 8)
    rho = float(pipe.offsets[-1].item()) / (sum(wl.lengths) * wl.n_kv_heads)
    say(f"  boundary keys {boundary}, kept fraction {rho:.4f}, compressed bytes {int(pipe.offsets[-1].item()) * wl.d_k * 4}")


def test_config4_long_context_sampled_rows(g):
    wl = W.config(4)
    say("cfg4 full: 28 layers x 131072, S=32, G=7")
    items, pipe = _run(g, wl)
    moff = _structure_checks(wl, items, pipe, sample_items=(3,))
    rows = [(0, 0), (5, 6), (13, 7), (31, 27), (17, 20), (8, 13)]
    boundary = _check_sampled_rows(wl, items[9], pipe, 9, moff, rows)
    boundary += _check_sampled_rows(wl, items[27], pipe, 27, moff, rows[:3])
    rho = float(pipe.offsets[-1].item()) / (sum(wl.lengths) * wl.n_kv_heads)
    say(f"  boundary keys {boundary}, kept fraction {rho:.4f}, fallback rows {pipe.n_fallback}")


def test_config5_ragged_batch(g):
    wl = W.config(5)
    say("cfg5 full: 16 requests", wl.lengths)
    items, pipe = _run(g, wl)
    moff = _structure_checks(wl, items, pipe, sample_items=(0, 7, 15))
    shortest, longest = int(np.argmin(wl.lengths)), int(np.argmax(wl.lengths))
    boundary = 0
    for i in (shortest, 4):
        cpu = {k: (v.cpu() if isinstance(v, torch.Tensor) else v) for k, v in items[i].items()}
        ref = U.oracle_item(wl, cpu)
        L = wl.lengths[i]
        gm = U.unpack_rows(pipe.rowmask[moff[i]:moff[i + 1]], pipe.rows, L).reshape(wl.S, wl.n_q_heads, L)
        boundary += U.check_rowmask_sandwich(gm, ref["logits"], U.p32(wl.p), U.TOL[wl.dtype])
    boundary += _check_sampled_rows(wl, items[longest], pipe, longest, moff, [(0, 0), (7, 13), (15, 31)])
    usage = pipe.budget.cpu().numpy().sum(1) / (np.array(wl.lengths) * wl.n_kv_heads)
    say("  boundary keys", boundary, "usage per request", np.round(usage, 3).tolist())
    assert usage.max() > 2 * usage.min()          # the adaptive budgets really differ across requests
