"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.
Integer / byte / index work is bit-exact; floating point within the tolerance of parity_util.TOL.
Masks: where the stage is fed the oracle's own stored queries, the full sandwich
C(p - tol) <= gpu <= C(p + tol) at STAGE_TOL (check_rowmask_strict); end to end (each side on its own
queries) the cumulative-mass band plus the selection's validity on the oracle's weights and the budgets
within 2 % + 8 keys (check_rowmask_sandwich, check_budgets).  Boundary keys are counted and printed."""
import math
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
    sys.stdout.flush()


@pytest.fixture(scope="module")
def g():
    import paper_2509_03136_amd as g
    g.lib()
    assert torch.cuda.is_available()
    return g


def small_workloads():
    """Shapes of the five configurations, sized so the oracle takes seconds, spanning several
    tiles and a ragged tail."""
    c1, c2, c3, c4, c5 = (W.config(i) for i in range(1, 6))
    return {
        "cfg1": c1,
        "cfg2": c2,
        "cfg3_small": W.scaled(c3, lengths=(3000, 2085), n_planted=(40, 30)),
        "cfg4_small": W.scaled(c4, lengths=(2500,), n_planted=(6,)),
        "cfg5_small": W.scaled(c5, lengths=(1100, 333, 2049, 64), n_planted=(8, 3, 200, 1)),
    }


# ------------------------------------------------------------------ integers
def test_philox_stream_is_bit_exact(g):
    for seed, sid, n in ((0, 0, 16), (0x1234_5678_9ABC_DEF0, 0xFEDC_BA98_7654_3210, 4099), (3, 31, 1 << 16)):
        out = torch.zeros(n, device=DEV, dtype=torch.int32)
        g.philox_u32(seed, sid, n, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy().view(np.uint32)
        assert np.array_equal(got, O.philox_u32_stream(seed, sid, n))


# ------------------------------------------------------------------ stage 1
@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3_small", "cfg5_small"])
def test_fit_gaussian(g, name):
    wl = small_workloads()[name]
    say("fit", name)
    items = W.make_items(wl, "cpu")
    b = U.batch_from(g, wl, U.to_device(items, DEV))
    pipe = g.Pipeline(b, wl.S, wl.p, ddof=wl.ddof)
    for ddof in (1, 0):
        pipe.ddof = ddof
        pipe.fit()
        torch.cuda.synchronize()
        for i, it in enumerate(items):
            mu, var = O.fit_gaussian(U.f32np(it["hidden"]), wl.n_skip, ddof)
            gm, gv = pipe.mu[i].cpu().numpy(), pipe.var[i].cpu().numpy()
            sd = np.sqrt(var)
            assert np.all(np.abs(gm - mu) <= 1e-5 * np.maximum(np.abs(mu), sd) + 1e-7), np.abs(gm - mu).max()
            assert np.all(np.abs(gv - var) <= 1e-5 * var + 1e-9), (np.abs(gv - var) / var).max()


def test_fit_gaussian_edge_cases(g):
    wl = W.scaled(W.config(1), lengths=(2, 3, 70))
    items = W.make_items(wl, "cpu")
    items[0]["n_skip"] = 0
    items[1]["n_skip"] = 1
    items[2]["n_skip"] = 0
    items[2]["hidden"] = items[2]["hidden"] * 0 + 3.25 + torch.arange(70, dtype=torch.float32)[:, None] * 1e3
    b = U.batch_from(g, wl, U.to_device(items, DEV))
    pipe = g.Pipeline(b, wl.S, wl.p)
    pipe.fit()
    torch.cuda.synchronize()
    for i, it in enumerate(items):
        mu, var = O.fit_gaussian(U.f32np(it["hidden"]), it["n_skip"], 1)
        assert np.allclose(pipe.mu[i].cpu().numpy(), mu, rtol=1e-5, atol=1e-6)
        assert np.allclose(pipe.var[i].cpu().numpy(), var, rtol=1e-5, atol=1e-9)
    # strided rows (a view into a wider buffer)
    wide = torch.zeros(70, 512, device=DEV)
    wide[:, :256] = items[2]["hidden"].to(DEV)
    it2 = dict(U.to_device([items[2]], DEV)[0], hidden=wide[:, :256])
    b2 = U.batch_from(g, wl, [it2])
    p2 = g.Pipeline(b2, wl.S, wl.p)
    p2.fit()
    torch.cuda.synchronize()
    assert torch.equal(p2.mu[0], pipe.mu[2]) and torch.equal(p2.var[0], pipe.var[2])


# ------------------------------------------------------------------ stage 2
@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg4_small", "cfg5_small"])
def test_sample_queries_given_oracle_moments(g, name):
    wl = small_workloads()[name]
    say("sample", name)
    items = W.make_items(wl, "cpu")
    b = U.batch_from(g, wl, U.to_device(items, DEV))
    pipe = g.Pipeline(b, wl.S, wl.p, want_h_tilde=True)
    refs = [U.oracle_item(wl, it, upto="q") for it in items]
    pipe.mu.copy_(torch.tensor(np.stack([r["mu"] for r in refs])))
    pipe.var.copy_(torch.tensor(np.stack([r["var"] for r in refs])))
    pipe.sample()
    torch.cuda.synchronize()
    tol = U.TOL[wl.dtype]
    for i, r in enumerate(refs):
        h = U.f32np(pipe.h_tilde[i]).astype(np.float64)
        q = U.f32np(pipe.q[i]).astype(np.float64)
        if wl.dtype == "f32":
            assert np.all(np.abs(h - r["h_tilde"]) <= 1e-5 * (1 + np.abs(r["h_tilde"]))), np.abs(h - r["h_tilde"]).max()
            assert np.all(np.abs(q - r["q_tilde"]) <= 1e-5 * (1 + np.abs(r["q_tilde"]))), np.abs(q - r["q_tilde"]).max()
        else:
            # stored bf16 values: equal except where fp32-vs-fp64 arithmetic lands on the other side of a
            # rounding boundary (then exactly one bf16 step apart)
            hd = h != r["h_tilde"]
            assert hd.mean() < 2e-3, hd.mean()
            # (near a cancellation mu + sigma z ~ 0 the fp32 normal's 1e-6 error is all that is left)
            mag = np.abs(r["mu"].astype(np.float64))[None, :] + np.sqrt(r["var"].astype(np.float64))[None, :] * np.abs(r["z"])
            assert np.all(np.abs(h - r["h_tilde"]) <= 2.0 ** -7 * np.abs(r["h_tilde"]) + 2e-6 * mag)
            qd = np.abs(q - r["q_tilde"])
            scale = np.sqrt((r["q_tilde"] ** 2).mean())
            assert np.all(qd <= 2.0 ** -7 * np.abs(r["q_tilde"]) + tol * scale), qd.max()
            assert (qd > 0).mean() < 0.05, (qd > 0).mean()
        say("  item", i, "max |dq|", float(np.abs(q - r["q_tilde"]).max()))


def test_sample_queries_bias_and_future_average(g):
    wl = W.scaled(W.config(2), lengths=(300,))
    items = W.make_items(wl, "cpu")
    gen = torch.Generator().manual_seed(5)
    bq = (torch.randn(wl.n_q_heads * wl.d_k, generator=gen) * 0.5).to(torch.bfloat16)
    items[0].update(b_q=bq, pos0=1000, n_future=5)
    ref = U.oracle_item(wl, items[0], upto="q", pos0=1000, n_future=5, b_q=bq)
    b = U.batch_from(g, wl, U.to_device(items, DEV))
    pipe = g.Pipeline(b, wl.S, wl.p)
    pipe.mu.copy_(torch.tensor(ref["mu"])[None])
    pipe.var.copy_(torch.tensor(ref["var"])[None])
    pipe.sample()
    torch.cuda.synchronize()
    q = U.f32np(pipe.q[0]).astype(np.float64)
    qd = np.abs(q - ref["q_tilde"])
    scale = np.sqrt((ref["q_tilde"] ** 2).mean())
    assert np.all(qd <= 2.0 ** -7 * np.abs(ref["q_tilde"]) + 2e-3 * scale), qd.max()


# ------------------------------------------------------------------ stage 3
@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3_small", "cfg4_small", "cfg5_small"])
def test_score_select_given_oracle_queries(g, name):
    wl = small_workloads()[name]
    say("select", name)
    items = W.make_items(wl, "cpu")
    refs = [U.oracle_item(wl, it) for it in items]
    b = U.batch_from(g, wl, U.to_device(items, DEV))
    pipe = g.Pipeline(b, wl.S, wl.p)
    pipe.q.copy_(torch.tensor(np.stack([r["q_tilde"] for r in refs])).to(pipe.q.dtype))
    pipe.select()
    torch.cuda.synchronize()
    off = 0
    total_boundary = 0
    for i, (it, r) in enumerate(zip(items, refs)):
        L = it["L"]
        n = pipe.mask_words[i]
        gm = U.unpack_rows(pipe.rowmask[off:off + n], pipe.rows, L).reshape(wl.S, wl.n_q_heads, L)
        off += n
        # same stored inputs on both sides: only fp32-vs-fp64 arithmetic separates them
        stol = U.STAGE_TOL[wl.dtype]
        total_boundary += U.check_rowmask_strict(gm, r["logits"], U.p32(wl.p), stol)
        m = r["logits"].max(-1)
        Z = np.exp(r["logits"] - m[..., None]).sum(-1)
        gmax = pipe.row_max[i].cpu().numpy().reshape(wl.S, wl.n_q_heads)
        gsum = pipe.row_sum[i].cpu().numpy().reshape(wl.S, wl.n_q_heads)
        assert np.all(np.abs(gmax - m) <= stol * (1 + np.abs(m))), np.abs(gmax - m).max()
        assert np.all(np.abs(gsum - Z) <= stol * Z), (np.abs(gsum - Z) / Z).max()
    say("  boundary keys", total_boundary)
    assert total_boundary <= 16


def _select_case(g, wl, items, q_np, p, mode=0, k_per_row=None):
    b = U.batch_from(g, wl, U.to_device(items, DEV))
    pipe = g.Pipeline(b, wl.S, p)
    pipe.q.copy_(torch.tensor(q_np).to(pipe.q.dtype))
    kk = None if k_per_row is None else torch.tensor(k_per_row, dtype=torch.int32, device=DEV)
    g.score_select(b, wl.S, pipe.q, p, pipe.rowmask, mode=mode, k_per_row=kk, row_max=pipe.row_max,
                   row_sum=pipe.row_sum, ws=pipe.ws)
    torch.cuda.synchronize()
    L = items[0]["L"]
    return U.unpack_rows(pipe.rowmask[:pipe.mask_words[0]], pipe.rows, L).reshape(wl.S, wl.n_q_heads, L), pipe


def test_select_degenerate_cases(g):
    wl = W.scaled(W.config(1), lengths=(517,))
    it = W.make_items(wl, "cpu")[0]
    ref = U.oracle_item(wl, it)
    L = 517
    # p = 1 keeps every key, bits beyond L stay 0
    gm, pipe = _select_case(g, wl, [it], ref["q_tilde"][None], 1.0)
    assert gm.all()
    words = pipe.rowmask[:pipe.mask_words[0]].cpu().numpy().view(np.uint32).reshape(pipe.rows, -1)
    assert np.all(words[:, -1] == (1 << (L % 32)) - 1)
    # all keys equal -> uniform attention -> the first ceil(p L) positions
    it0 = dict(it, k=torch.zeros_like(it["k"]))
    gm, _ = _select_case(g, wl, [it0], ref["q_tilde"][None], 0.9)
    want = O.top_p_select(np.zeros(L), U.p32(0.9))
    assert want.sum() == math.ceil(U.p32(0.9) * L)
    assert np.all(gm == want[None, None, :])
    # duplicated keys: exact ties at the cut go to the lower position
    kd = it["k"].clone()
    kd[1::2] = kd[0::2][: kd[1::2].shape[0]]
    itd = dict(it, k=kd)
    lg = O.scores(ref["q_tilde"], U.f32np(kd))
    gm, _ = _select_case(g, wl, [itd], ref["q_tilde"][None], 0.7)
    assert U.check_rowmask_strict(gm, lg, U.p32(0.7), 1e-5) <= 2
    # one dominant key -> a single selected key per row
    kh = it["k"].clone() * 0.01
    kh[100] = 50.0 * torch.tensor(ref["q_tilde"][0].reshape(wl.n_kv_heads, wl.group, wl.d_k)[:, 0], dtype=torch.float32)
    q1 = np.repeat(ref["q_tilde"][:1], wl.S, axis=0)
    q1 = np.repeat(q1.reshape(wl.S, wl.n_kv_heads, wl.group, wl.d_k)[:, :, :1], wl.group, axis=2).reshape(ref["q_tilde"].shape)
    gm, _ = _select_case(g, wl, [dict(it, k=kh)], q1[None], 0.99)
    assert np.all(gm.sum(-1) == 1) and gm[..., 100].all()
    # L = 2 and S = 1
    wl2 = W.scaled(W.config(1), lengths=(2,), S=1)
    it2 = W.make_items(wl2, "cpu")[0]
    it2["n_skip"] = 0
    r2 = U.oracle_item(wl2, it2, n_skip=0)
    gm, _ = _select_case(g, wl2, [it2], r2["q_tilde"][None], 0.9)
    assert np.array_equal(gm, r2["rowmask"])


def test_select_bf16_fallbacks_and_ties(g):
    """bf16 (matrix-core path): cases the histogram cannot settle must fall back to the exact selector."""
    wl = W.scaled(W.config(2), lengths=(1500,), S=4)
    it = W.make_items(wl, "cpu")[0]
    ref = U.oracle_item(wl, it)
    q = ref["q_tilde"][None]
    stol = U.STAGE_TOL["bf16"]
    # the cut lies far below the maximum (p -> 1): beyond the histogram window
    for p in (0.999999, 0.9999999):
        gm, _ = _select_case(g, wl, [it], q, p)
        # (p within 1e-6 of 1: fp32 weights cannot honour a band of (1 - p) / 4 on the mass itself, so the
        # validity asserts use 1e-6; the interval band stays at (1 - p) / 4)
        nb = U.check_rowmask_sandwich(gm, ref["logits"], U.p32(p), min(stol, (1 - U.p32(p)) / 4),
                                      vtol=max((1 - U.p32(p)) / 2, 1e-6))
        say("  p", p, "boundary", nb, "mean row size", gm.sum(-1).mean())
    # all keys equal: every key lands in one bin, candidate lists overflow; ties -> lowest positions
    it0 = dict(it, k=torch.zeros_like(it["k"]))
    gm, _ = _select_case(g, wl, [it0], q, 0.9)
    want = O.top_p_select(np.zeros(1500), U.p32(0.9))
    assert np.all(gm == want[None, None, :])
    # every key duplicated: exact ties inside the boundary bin are resolved towards the lower position
    kd = it["k"].clone()
    kd[1::2] = kd[0::2]
    lg = O.scores(ref["q_tilde"], U.f32np(kd))
    for p in (0.5, 0.95):
        gm, _ = _select_case(g, wl, [dict(it, k=kd)], q, p)
        assert U.check_rowmask_strict(gm, lg, U.p32(p), stol) <= 8
    # flatter attention: hundreds of keys share the cut bin (the larger candidate paths of the resolver)
    for scale in (0.25, 0.05):
        ks = (it["k"].to(torch.float32) * scale).to(it["k"].dtype)
        lg = O.scores(ref["q_tilde"], U.f32np(ks))
        gm, _ = _select_case(g, wl, [dict(it, k=ks)], q, 0.9)
        nb = U.check_rowmask_strict(gm, lg, U.p32(0.9), stol)
        say("  key scale", scale, "boundary", nb, "mean row size", gm.sum(-1).mean())
    # a tiny p: only the arg-max key of each row
    gm, _ = _select_case(g, wl, [it], q, 1e-6)
    assert np.all(gm.sum(-1) == 1)
    assert np.array_equal(gm.argmax(-1), ref["logits"].argmax(-1))


def test_select_topk_mode(g):
    wl = W.scaled(W.config(2), lengths=(700,), S=4)
    it = W.make_items(wl, "cpu")[0]
    ref = U.oracle_item(wl, it)
    R = wl.S * wl.n_q_heads
    ks = (np.arange(R) * 37 % 720) - 5          # includes k < 1 and k > L (clamped to [1, L])
    gm, pipe = _select_case(g, wl, [it], ref["q_tilde"][None], 0.5, mode=1, k_per_row=ks)
    say(f"  TopK with k up to L: {pipe.fallback_rows()} of {R} rows redone by the exact selector (cut below the window)")
    lg = ref["logits"].reshape(R, -1)
    gm = gm.reshape(R, -1)
    bad = 0
    for r in range(R):
        k = int(min(max(ks[r], 1), 700))
        want = O.top_k_select(lg[r], k)
        assert gm[r].sum() == k
        bad += int((gm[r] ^ want).sum())
    assert bad <= 4            # only fp32-vs-fp64 near-ties may swap


# ------------------------------------------------------------------ stage 4
@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg5_small"])
def test_union_compact_given_oracle_masks_is_bit_exact(g, name):
    wl = small_workloads()[name]
    say("compact", name)
    items = W.make_items(wl, "cpu")
    refs = [U.oracle_item(wl, it) for it in items]
    b = U.batch_from(g, wl, U.to_device(items, DEV))
    pipe = g.Pipeline(b, wl.S, wl.p)
    words = np.concatenate([O.pack_mask_words(r["rowmask"].reshape(pipe.rows, -1)).reshape(-1) for r in refs])
    pipe.rowmask.copy_(torch.tensor(words.view(np.int32)))
    pipe.compact()
    torch.cuda.synchronize()
    assert int(pipe.overflow.item()) == 0
    budget = pipe.budget.cpu().numpy()
    offsets = pipe.offsets.cpu().numpy()
    assert np.array_equal(budget, np.stack([r["budget"] for r in refs]))
    assert np.array_equal(offsets, np.concatenate([[0], np.cumsum(budget.reshape(-1))]))
    uoff = 0
    for i, (it, r) in enumerate(zip(items, refs)):
        L = it["L"]
        um = U.unpack_rows(pipe.union_mask[uoff:uoff + pipe.union_words[i]], wl.n_kv_heads, L)
        uoff += pipe.union_words[i]
        assert np.array_equal(um, r["union"])
        lo, hi = offsets[i * wl.n_kv_heads], offsets[(i + 1) * wl.n_kv_heads]
        assert torch.equal(pipe.k_out[lo:hi].cpu(), torch.tensor(r["k_out"]).to(pipe.k_out.dtype))
        assert torch.equal(pipe.v_out[lo:hi].cpu(), torch.tensor(r["v_out"]).to(pipe.v_out.dtype))
        assert np.array_equal(pipe.idx_out[lo:hi].cpu().numpy(), r["idx"])


def test_union_compact_overflow_strides_and_many_items(g):
    wl = W.scaled(W.config(1), lengths=(100,) * 70)           # more items than one launch batch holds
    base = W.make_items(W.scaled(W.config(1), lengths=(100,)), "cpu")[0]
    gen = torch.Generator().manual_seed(9)
    items = []
    for i in range(70):
        kv = torch.randn(100, wl.n_kv_heads, 2, wl.d_k, generator=gen)        # k and v interleaved: strided views
        items.append(dict(base, k=kv[:, :, 0], v=kv[:, :, 1], stream_id=i))
    dev_items = []
    for it in items:
        kv = torch.stack([it["k"], it["v"]], dim=2).to(DEV)
        dev_items.append(dict(it, hidden=it["hidden"].to(DEV), w_q=it["w_q"].to(DEV), k=kv[:, :, 0], v=kv[:, :, 1]))
    b = U.batch_from(g, wl, dev_items)
    pipe = g.Pipeline(b, wl.S, wl.p)
    rng = np.random.default_rng(0)
    rm = rng.random((70, pipe.rows, 100)) < 0.02
    words = np.concatenate([O.pack_mask_words(m).reshape(-1) for m in rm])
    pipe.rowmask.copy_(torch.tensor(words.view(np.int32)))
    pipe.compact()
    torch.cuda.synchronize()
    budget = pipe.budget.cpu().numpy()
    offsets = pipe.offsets.cpu().numpy()
    for i in range(70):
        union, bud = O.union_vote(rm[i].reshape(wl.S, wl.n_q_heads, 100), wl.n_kv_heads)
        assert np.array_equal(budget[i], bud)
        ko, vo, idx, _ = O.compact(items[i]["k"].numpy(), items[i]["v"].numpy(), union)
        lo, hi = offsets[i * wl.n_kv_heads], offsets[(i + 1) * wl.n_kv_heads]
        assert np.array_equal(pipe.k_out[lo:hi].cpu().numpy(), ko)
        assert np.array_equal(pipe.v_out[lo:hi].cpu().numpy(), vo)
        assert np.array_equal(pipe.idx_out[lo:hi].cpu().numpy(), idx)
    # capacity smaller than the total: flag set, budgets complete, rows below the capacity intact
    total = int(offsets[-1])
    cap = total // 2
    small = g.Pipeline(b, wl.S, wl.p, capacity_tokens=cap)
    small.rowmask.copy_(pipe.rowmask)
    small.k_out.fill_(-7.0)
    small.compact()
    torch.cuda.synchronize()
    assert int(small.overflow.item()) == 1
    assert torch.equal(small.budget, pipe.budget) and torch.equal(small.offsets, pipe.offsets)
    assert torch.equal(small.k_out[:cap], pipe.k_out[:cap])


# ------------------------------------------------------------------ whole path
@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3_small", "cfg4_small", "cfg5_small"])
def test_end_to_end_path(g, name):
    wl = small_workloads()[name]
    say("e2e", name)
    items = W.make_items(wl, "cpu")
    refs = [U.oracle_item(wl, it) for it in items]
    b = U.batch_from(g, wl, U.to_device(items, DEV))
    pipe = g.Pipeline(b, wl.S, wl.p, ddof=wl.ddof)
    pipe.run()
    torch.cuda.synchronize()
    tol = U.TOL[wl.dtype]
    budget = pipe.budget.cpu().numpy()
    offsets = pipe.offsets.cpu().numpy()
    assert np.array_equal(offsets, np.concatenate([[0], np.cumsum(budget.reshape(-1))]))
    moff = uoff = 0
    boundary = 0
    for i, (it, r) in enumerate(zip(items, refs)):
        L = it["L"]
        gm = U.unpack_rows(pipe.rowmask[moff:moff + pipe.mask_words[i]], pipe.rows, L).reshape(wl.S, wl.n_q_heads, L)
        moff += pipe.mask_words[i]
        boundary += U.check_rowmask_sandwich(gm, r["logits"], U.p32(wl.p), tol)
        um = U.unpack_rows(pipe.union_mask[uoff:uoff + pipe.union_words[i]], wl.n_kv_heads, L)
        uoff += pipe.union_words[i]
        # the union is exactly the OR of the GPU's own rows; budgets count it; compaction follows it bit for bit
        gu, gb = O.union_vote(gm, wl.n_kv_heads)
        assert np.array_equal(um, gu) and np.array_equal(budget[i], gb)
        assert np.all(gb >= gm.reshape(wl.S, wl.n_kv_heads, wl.group, L).sum(-1).max(axis=(0, 2)))
        ko, vo, idx, _ = O.compact(U.f32np(it["k"]), U.f32np(it["v"]), um)
        lo, hi = offsets[i * wl.n_kv_heads], offsets[(i + 1) * wl.n_kv_heads]
        assert np.array_equal(U.f32np(pipe.k_out[lo:hi]), ko) and np.array_equal(U.f32np(pipe.v_out[lo:hi]), vo)
        assert np.array_equal(pipe.idx_out[lo:hi].cpu().numpy(), idx)
        m = r["logits"].max(-1).reshape(-1)
        assert np.all(np.abs(pipe.row_max[i].cpu().numpy() - m) <= tol * (1 + np.abs(m)))
        say(f"  item {i}: L={L} budget gpu {budget[i].tolist()} oracle {r['budget'].tolist()}")
        U.check_budgets(budget[i], r["budget"])
    say("  boundary keys", boundary)


def test_repeat_runs_are_bit_identical(g):
    """Integer histograms, ordered compaction and fixed-order reductions: the same call twice gives the
    same bits (masks, budgets, packed cache, moments, queries)."""
    wl = small_workloads()["cfg3_small"]
    items = W.make_items(wl, "cpu")
    b = U.batch_from(g, wl, U.to_device(items, DEV))
    outs = []
    for _ in range(2):
        pipe = g.Pipeline(b, wl.S, wl.p, ddof=wl.ddof)
        pipe.run()
        torch.cuda.synchronize()
        n = int(pipe.offsets[-1].item())
        outs.append((pipe.mu.clone(), pipe.var.clone(), pipe.q.clone(), pipe.rowmask.clone(), pipe.union_mask.clone(),
                     pipe.budget.clone(), pipe.k_out[:n].clone(), pipe.idx_out[:n].clone()))
    for a, c in zip(*outs):
        assert torch.equal(a, c)


def test_short_contexts_take_the_general_path(g):
    """bf16 items with fewer than 32 keys (the matrix-core path loads whole 32-key tiles)."""
    wl = W.scaled(W.config(2), lengths=(31, 17, 40), S=4)
    items = W.make_items(wl, "cpu")
    refs = [U.oracle_item(wl, it) for it in items]
    b = U.batch_from(g, wl, U.to_device(items, DEV))
    pipe = g.Pipeline(b, wl.S, wl.p)
    pipe.q.copy_(torch.tensor(np.stack([r["q_tilde"] for r in refs])).to(pipe.q.dtype))
    pipe.select()
    torch.cuda.synchronize()
    off = 0
    for i, (it, r) in enumerate(zip(items, refs)):
        L = it["L"]
        gm = U.unpack_rows(pipe.rowmask[off:off + pipe.mask_words[i]], pipe.rows, L).reshape(wl.S, wl.n_q_heads, L)
        off += pipe.mask_words[i]
        U.check_rowmask_strict(gm, r["logits"], U.p32(wl.p), U.STAGE_TOL[wl.dtype])


def test_algorithm1_mode_real_query_budget_then_topk(g):
    """The paper's Algorithm 1 as printed: the REAL current query's top-p set sizes B_step per head, then
    every synthetic row keeps its B_step largest logits (row-wise TopK), then the union.  Composed from
    gvote_score_select (TOPP, S = 1) -> gvote_count_rows -> gvote_score_select (TOPK) -> gvote_union_compact."""
    wl = W.scaled(W.config(2), lengths=(1800, 700), n_planted=(30, 10), S=8)
    items = W.make_items(wl, "cpu")
    dev_items = U.to_device(items, DEV)
    b = U.batch_from(g, wl, dev_items)
    n, S, hq = len(items), wl.S, wl.n_q_heads
    refs = [U.oracle_item(wl, it) for it in items]
    p = U.p32(wl.p)
    # the real current query of each item: the last token's hidden state through W_q, rotated at L - 1
    q0 = []
    for it in items:
        L = it["L"]
        c, s_ = O.rope_cos_sin(float(np.float32(wl.theta)), wl.d_k, L - 1, 1)
        q0.append(O.project_rope(U.f32np(it["hidden"][L - 1:L]), U.f32np(it["w_q"]), None, c, s_, hq, wl.d_k, wl.dtype))
    q0_dev = torch.tensor(np.stack(q0)).to(torch.bfloat16).to(DEV)                 # [n, 1, H_q, d_k]
    words = [b.words(i) for i in range(n)]
    mask0 = torch.empty(sum(hq * w for w in words), device=DEV, dtype=torch.int32)
    ws = torch.empty(g.workspace_bytes(b, S), device=DEV, dtype=torch.uint8)
    g.score_select(b, 1, q0_dev, p, mask0, ws=ws)
    counts = torch.empty(n, S, hq, device=DEV, dtype=torch.int32)
    g.count_rows(b, 1, mask0, S, counts)
    pipe = g.Pipeline(b, S, p)
    pipe.q.copy_(torch.tensor(np.stack([r["q_tilde"] for r in refs])).to(pipe.q.dtype))
    g.score_select(b, S, pipe.q, p, pipe.rowmask, mode=g.SELECT_TOPK, k_per_row=counts, ws=pipe.ws)
    torch.cuda.synchronize()
    n_fb = pipe.fallback_rows()          # TopK runs on the matrix-core path too (count-weighted histogram)
    say(f"  TopK rows redone by the exact selector: {n_fb} of {n * S * hq} {pipe.fallback_reasons()}")
    assert n_fb <= n * S * hq // 20
    pipe.compact()
    torch.cuda.synchronize()
    counts_h = counts.cpu().numpy()
    off0 = off = uoff = 0
    swaps = 0
    for i, (it, r) in enumerate(zip(items, refs)):
        L = it["L"]
        lg0 = O.scores(q0[i], U.f32np(it["k"]))[0]                      # [H_q, L]
        m0 = U.unpack_rows(mask0[off0:off0 + hq * words[i]], hq, L)
        off0 += hq * words[i]
        U.check_rowmask_strict(m0[None], lg0[None], p, U.STAGE_TOL["bf16"])     # the real query is the oracle's
        for h in range(hq):
            assert np.all(counts_h[i, :, h] == m0[h].sum())
        gm = U.unpack_rows(pipe.rowmask[off:off + pipe.mask_words[i]], pipe.rows, L).reshape(S, hq, L)
        off += pipe.mask_words[i]
        for s in range(S):
            for h in range(hq):
                k = int(counts_h[i, s, h])
                assert gm[s, h].sum() == k
                swaps += int((gm[s, h] ^ O.top_k_select(r["logits"][s, h], k)).sum())
        um = U.unpack_rows(pipe.union_mask[uoff:uoff + pipe.union_words[i]], wl.n_kv_heads, L)
        uoff += pipe.union_words[i]
        gu, gb = O.union_vote(gm, wl.n_kv_heads)
        assert np.array_equal(um, gu) and np.array_equal(pipe.budget[i].cpu().numpy(), gb)
        say(f"  item {i}: B_step per head {counts_h[i, 0].tolist()[:8]}..., union budget {gb.tolist()}")
    assert swaps <= 8          # only fp32-vs-fp64 near-ties may swap


def test_more_items_than_one_launch_table_bf16(g):
    """40 requests in one call: every stage splits the batch into launch tables of 32 items."""
    lengths = tuple(64 + 37 * (i % 9) + i for i in range(40))
    wl = W.scaled(W.config(5), lengths=lengths, n_planted=tuple(1 + i % 4 for i in range(40)), S=4)
    items = W.make_items(wl, "cpu")
    b = U.batch_from(g, wl, U.to_device(items, DEV))
    pipe = g.Pipeline(b, wl.S, wl.p, ddof=wl.ddof)
    pipe.run()
    torch.cuda.synchronize()
    budget = pipe.budget.cpu().numpy()
    offsets = pipe.offsets.cpu().numpy()
    assert np.array_equal(offsets, np.concatenate([[0], np.cumsum(budget.reshape(-1))]))
    moff = np.concatenate([[0], np.cumsum(pipe.mask_words)])
    uoff = np.concatenate([[0], np.cumsum(pipe.union_words)])
    for i in (0, 31, 32, 39):
        it, L = items[i], lengths[i]
        r = U.oracle_item(wl, it)
        gm = U.unpack_rows(pipe.rowmask[moff[i]:moff[i + 1]], pipe.rows, L).reshape(wl.S, wl.n_q_heads, L)
        U.check_rowmask_sandwich(gm, r["logits"], U.p32(wl.p), U.TOL[wl.dtype])
        um = U.unpack_rows(pipe.union_mask[uoff[i]:uoff[i + 1]], wl.n_kv_heads, L)
        gu, gb = O.union_vote(gm, wl.n_kv_heads)
        assert np.array_equal(um, gu) and np.array_equal(budget[i], gb)
        U.check_budgets(budget[i], r["budget"])
        ko, vo, idx, _ = O.compact(U.f32np(it["k"]), U.f32np(it["v"]), um)
        lo, hi = offsets[i * wl.n_kv_heads], offsets[(i + 1) * wl.n_kv_heads]
        assert np.array_equal(U.f32np(pipe.k_out[lo:hi]), ko) and np.array_equal(pipe.idx_out[lo:hi].cpu().numpy(), idx)
        assert np.all(np.abs(pipe.mu[i].cpu().numpy() - r["mu"]) <= 1e-5 * np.maximum(np.abs(r["mu"]), np.sqrt(r["var"])) + 1e-7)
