"""Seeded random sweep of the select stage on the matrix-core path against the oracle: lengths from 33 to 6000 in
ragged batches, 1 to 33 samples, 1 to 8 query heads per KV head, both head sizes, p from 0.3 to 0.99999, keys scaled
from nearly flat to sharply peaked attention, both selection rules.  Same stored queries on both sides, so the masks
must agree in full (the strict check) and TopK must return exactly k keys split at the k-th largest logit."""
import numpy as np
import pytest
import torch

import oracle as O
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


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_shapes_against_the_oracle(g, seed):
    rng = np.random.default_rng(seed)
    second = exact = 0
    for case in range(16):
        dk = int(rng.choice([64, 128]))
        hkv = int(rng.choice([1, 2, 4]))
        G = int(rng.choice([1, 2, 4, 7, 8]))
        S = int(rng.choice([1, 2, 3, 5, 8, 16, 24, 33]))
        n_it = int(rng.choice([1, 2, 3]))
        lengths = tuple(int(x) for x in np.exp(rng.uniform(np.log(33), np.log(6000), n_it)).astype(int))
        p = float(rng.choice([0.3, 0.8, 0.9, 0.95, 0.99, 0.999, 0.9999, 0.99999]))
        kscale = float(rng.choice([0.02, 0.2, 1.0, 1.0, 3.0, 30.0]))
        topk = bool(rng.integers(0, 3) == 0)
        wl = W.scaled(W.config(2), lengths=lengths, n_planted=tuple(max(1, L // 100) for L in lengths), d=256,
                      n_q_heads=hkv * G, n_kv_heads=hkv, d_k=dk, S=S, seed=100 * seed + case)
        items = W.make_items(wl, "cpu")
        items = [dict(it, k=(it["k"].to(torch.float32) * kscale).to(it["k"].dtype)) for it in items]
        refs = [U.oracle_item(wl, it, upto="q") for it in items]
        lgs = [O.scores(r["q_tilde"], U.f32np(it["k"])) for it, r in zip(items, refs)]
        b = U.batch_from(g, wl, U.to_device(items, DEV))
        pipe = g.Pipeline(b, wl.S, p)
        pipe.q.copy_(torch.tensor(np.stack([r["q_tilde"] for r in refs])).to(pipe.q.dtype))
        R = wl.S * wl.n_q_heads
        what = f"seed {seed} case {case}: d_k {dk}, {hkv} x {G} heads, S {S}, L {lengths}, p {p}, keys x {kscale}, topk {topk}"
        print(what, flush=True)
        if topk:
            ks = np.concatenate([rng.integers(1, L + 1, R) for L in lengths]).astype(np.int32)
            g.score_select(b, wl.S, pipe.q, 0.5, pipe.rowmask, mode=g.SELECT_TOPK, k_per_row=torch.tensor(ks, device=DEV),
                           ws=pipe.ws)
        else:
            pipe.select()
        torch.cuda.synchronize()
        off = 0
        for i, it in enumerate(items):
            L = it["L"]
            gm = U.unpack_rows(pipe.rowmask[off:off + pipe.mask_words[i]], pipe.rows, L).reshape(wl.S, wl.n_q_heads, L)
            off += pipe.mask_words[i]
            # (fp32 accumulation: the logit error grows with the logit, about 2^-21 |l|)
            tol = max(U.STAGE_TOL["bf16"], 2.0 ** -21 * float(np.abs(lgs[i]).max()))
            if topk:
                lg, got = lgs[i].reshape(R, L), gm.reshape(R, L)
                for r in range(R):
                    k = min(int(ks[i * R + r]), L)
                    assert got[r].sum() == k, (what, i, r, int(got[r].sum()), k)
                    if k < L:
                        assert lg[r][got[r]].min() >= lg[r][~got[r]].max() - U.logit_slack(lg[r], tol), (what, i, r)
            else:
                pp = U.p32(p)
                close = pp > 0.999
                U.check_rowmask_strict(gm, lgs[i], pp, min(tol, (1 - pp) / 4) if close else tol,
                                       vtol=max((1 - pp) / 2, 1e-6) if close else None)
        second += pipe.refined_rows()
        exact += pipe.fallback_rows()
    print(f"  seed {seed}: rows settled by a second histogram {second}, redone exactly {exact}", flush=True)


@pytest.mark.parametrize("seed", [21, 22])
def test_random_union_compact_against_the_oracle(g, seed):
    """Stage 4 on random row masks (Sec. 3.2 Step 4): row counts S*G that are not multiples of the workgroup's four
    waves, lengths that end inside a mask word and inside a 2048-token chunk, empty and full heads; union masks,
    budgets, offsets and the packed K/V rows bit-exact against the oracle, also through the entry point that keeps
    its scratch in the library."""
    rng = np.random.default_rng(seed)
    for case in range(12):
        dk = int(rng.choice([64, 128]))
        hkv = int(rng.choice([1, 2, 4]))
        G = int(rng.choice([1, 2, 3, 7, 8]))
        S = int(rng.choice([1, 2, 3, 5, 8, 16, 33]))
        n_it = int(rng.choice([1, 2, 5]))
        lengths = tuple(int(x) for x in np.exp(rng.uniform(np.log(33), np.log(9000), n_it)).astype(int))
        density = float(rng.choice([0.0, 0.001, 0.02, 0.3, 1.0]))
        wl = W.scaled(W.config(2), lengths=lengths, n_planted=tuple(1 for _ in lengths), d=64,
                      n_q_heads=hkv * G, n_kv_heads=hkv, d_k=dk, S=S, seed=100 * seed + case)
        items = W.make_items(wl, "cpu")
        print(f"seed {seed} case {case}: d_k {dk}, {hkv} x {G} heads, S {S}, L {lengths}, density {density}", flush=True)
        b = U.batch_from(g, wl, U.to_device(items, DEV))
        pipe = g.Pipeline(b, wl.S, 0.9)
        masks = []
        for L in lengths:
            m = rng.random((S, hkv * G, L)) < density
            if density > 0.0:
                m[rng.integers(0, S), :, L - 1] = True          # the last key of the item, in every head
            if hkv > 1:
                m[:, :G, :] = False                               # an empty head: budget 0
            masks.append(m)
        words = np.concatenate([O.pack_mask_words(m.reshape(pipe.rows, -1)).reshape(-1) for m in masks])
        pipe.rowmask.copy_(torch.tensor(words.view(np.int32)))
        for static in (False, True):
            pipe.k_out.zero_(); pipe.v_out.zero_(); pipe.budget.fill_(-1); pipe.offsets.fill_(-1)
            if static:
                g.union_compact_static(b, wl.S, pipe.rowmask, pipe.union_mask, pipe.budget, pipe.offsets, pipe.k_out,
                                       pipe.v_out, pipe.idx_out, pipe.capacity, pipe.overflow)
            else:
                pipe.compact()
            torch.cuda.synchronize()
            assert int(pipe.overflow.item()) == 0
            budget, offsets = pipe.budget.cpu().numpy(), pipe.offsets.cpu().numpy()
            uoff = 0
            for i, (it, m) in enumerate(zip(items, masks)):
                union, bud = O.union_vote(m, hkv)
                assert np.array_equal(budget[i], bud), (static, i)
                um = U.unpack_rows(pipe.union_mask[uoff:uoff + pipe.union_words[i]], hkv, it["L"])
                uoff += pipe.union_words[i]
                assert np.array_equal(um, union), (static, i)
                ko, vo, idx, _ = O.compact(U.f32np(it["k"]), U.f32np(it["v"]), union)
                lo, hi = offsets[i * hkv], offsets[(i + 1) * hkv]
                assert hi - lo == int(bud.sum())
                assert np.array_equal(U.f32np(pipe.k_out[lo:hi]), ko), (static, i)
                assert np.array_equal(U.f32np(pipe.v_out[lo:hi]), vo), (static, i)
                assert np.array_equal(pipe.idx_out[lo:hi].cpu().numpy(), idx), (static, i)
            assert np.array_equal(offsets, np.concatenate([[0], np.cumsum(budget.reshape(-1))]))
