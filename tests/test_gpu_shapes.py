"""GPU parity on the kernel instantiations that the five benchmark shapes do not reach: head_dim 64 on the
bf16 matrix-core score path, 33..128 samples (the wider projection tiles, several 64-row blocks per KV
group), a hidden size that is not a multiple of the projection's k-slice, more than eight query heads per
KV head on the consumer side, and the failure handling of the first score pass (forced from the host
through the spin-limit test aid; every kernel still exits normally)."""
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


def _stage_by_stage(g, wl):
    """sample (given the oracle's moments) and select (given the oracle's queries) against the oracle."""
    items = W.make_items(wl, "cpu")
    refs = [U.oracle_item(wl, it) for it in items]
    b = U.batch_from(g, wl, U.to_device(items, DEV))
    pipe = g.Pipeline(b, wl.S, wl.p)
    pipe.mu.copy_(torch.tensor(np.stack([r["mu"] for r in refs])))
    pipe.var.copy_(torch.tensor(np.stack([r["var"] for r in refs])))
    pipe.sample()
    torch.cuda.synchronize()
    for i, r in enumerate(refs):
        q = U.f32np(pipe.q[i]).astype(np.float64)
        qd = np.abs(q - r["q_tilde"])
        scale = np.sqrt((r["q_tilde"] ** 2).mean())
        assert np.all(qd <= 2.0 ** -7 * np.abs(r["q_tilde"]) + U.TOL[wl.dtype] * scale), qd.max()
        assert (qd > 0).mean() < 0.05, (qd > 0).mean()
    pipe.q.copy_(torch.tensor(np.stack([r["q_tilde"] for r in refs])).to(pipe.q.dtype))
    pipe.select()
    torch.cuda.synchronize()
    n_fb = pipe.fallback_rows()
    off = boundary = 0
    for i, (it, r) in enumerate(zip(items, refs)):
        L = it["L"]
        gm = U.unpack_rows(pipe.rowmask[off:off + pipe.mask_words[i]], pipe.rows, L).reshape(wl.S, wl.n_q_heads, L)
        off += pipe.mask_words[i]
        boundary += U.check_rowmask_strict(gm, r["logits"], U.p32(wl.p), U.STAGE_TOL[wl.dtype])
        m = r["logits"].max(-1).reshape(-1)
        assert np.all(np.abs(pipe.row_max[i].cpu().numpy() - m) <= U.STAGE_TOL[wl.dtype] * (1 + np.abs(m)))
    pipe.compact()
    torch.cuda.synchronize()
    budget = pipe.budget.cpu().numpy()
    for i, r in enumerate(refs):
        U.check_budgets(budget[i], r["budget"], slack_keys=2 + boundary, rel=0.0)
    return boundary, n_fb


@pytest.mark.parametrize("S", [48, 96, 128])
def test_wide_sample_blocks_and_odd_hidden_size(g, S):
    # d = 832 = 512 + 320: the projection's last k-slice is short (and for S > 96 the slices are 256 wide);
    # S * G = 96 .. 256 query rows per KV head: two to four 64-row blocks in the score passes
    wl = W.scaled(W.config(2), lengths=(1500, 333), n_planted=(20, 4), d=832, n_q_heads=4, n_kv_heads=2, S=S)
    boundary, n_fb = _stage_by_stage(g, wl)
    say(f"  S={S}: boundary keys {boundary}, fallback rows {n_fb}")
    assert boundary <= 8


def test_head_dim_64_on_the_matrix_core_path(g):
    wl = W.scaled(W.config(2), lengths=(2100, 77), n_planted=(30, 2), d=1024, n_q_heads=16, n_kv_heads=4, d_k=64, S=16)
    boundary, n_fb = _stage_by_stage(g, wl)
    say(f"  head_dim 64: boundary keys {boundary}, fallback rows {n_fb}")
    assert boundary <= 8


@pytest.mark.parametrize("S,n", [(5, 21), (16, 7), (40, 3)])
def test_requests_that_share_one_layer_are_projected_together(g, S, n):
    """Items with the same W_q (requests through one layer) go through the projection in groups of up to 96
    columns: odd sample counts (group columns that straddle the 32-column blocks), a last group that is smaller,
    and the same queries as when every item is projected alone."""
    lengths = tuple(64 + 37 * i for i in range(n))
    wl = W.scaled(W.config(5), lengths=lengths, n_planted=(2,) * n, d=512, n_q_heads=4, n_kv_heads=2, S=S)
    items = W.make_items(wl, "cpu")
    assert all(it["w_q"] is items[0]["w_q"] for it in items)
    refs = [U.oracle_item(wl, it, upto="q") for it in items]
    dev_items = U.to_device(items, DEV)
    assert len({it["w_q"].data_ptr() for it in dev_items}) == 1
    b = U.batch_from(g, wl, dev_items)
    pipe = g.Pipeline(b, wl.S, wl.p)
    pipe.mu.copy_(torch.tensor(np.stack([r["mu"] for r in refs])))
    pipe.var.copy_(torch.tensor(np.stack([r["var"] for r in refs])))
    pipe.sample()
    torch.cuda.synchronize()
    q_grouped = pipe.q.clone()
    for i, r in enumerate(refs):
        q = U.f32np(pipe.q[i]).astype(np.float64)
        qd = np.abs(q - r["q_tilde"])
        scale = np.sqrt((r["q_tilde"] ** 2).mean())
        assert np.all(qd <= 2.0 ** -7 * np.abs(r["q_tilde"]) + U.TOL[wl.dtype] * scale), (i, qd.max())
        assert (qd > 0).mean() < 0.05, (i, (qd > 0).mean())
    # every item alone (its own copy of the weights): bit-identical queries
    for i in (0, n - 1):
        solo = dict(dev_items[i], w_q=dev_items[i]["w_q"].clone())
        b1 = U.batch_from(g, wl, [solo])
        p1 = g.Pipeline(b1, wl.S, wl.p)
        p1.mu.copy_(pipe.mu[i:i + 1]); p1.var.copy_(pipe.var[i:i + 1])
        p1.sample()
        torch.cuda.synchronize()
        assert torch.equal(p1.q[0], q_grouped[i]), i


@pytest.mark.parametrize("heads", [(32, 2, 64), (8, 2, 64), (16, 2, 64), (14, 2, 128), (32, 2, 128), (32, 1, 128), (48, 2, 64)],
                         ids=lambda h: f"Hq{h[0]}_Hkv{h[1]}_dk{h[2]}")
def test_decode_attention_group_sizes_and_head_dims(g, heads):
    """Every instantiation of the matrix-core decode kernel (4, 8 or 16 head columns, head_dim 64 and 128) and the
    vector-unit kernel that serves groups of more than 16 heads."""
    hq, hkv, dk = heads
    wl = W.scaled(W.config(2), lengths=(900, 130), n_planted=(10, 2), d=1024, n_q_heads=hq, n_kv_heads=hkv, d_k=dk, S=4)
    items = W.make_items(wl, "cpu")
    b = U.batch_from(g, wl, U.to_device(items, DEV))
    pipe = g.Pipeline(b, wl.S, wl.p, ddof=wl.ddof)
    pipe.run()
    gen = torch.Generator().manual_seed(11)
    q = torch.randn(len(items), wl.n_q_heads, wl.d_k, generator=gen).to(torch.bfloat16)
    q_dev = q.to(DEV)
    out = torch.empty_like(q_dev)
    lse = torch.empty(len(items), wl.n_q_heads, device=DEV, dtype=torch.float32)
    g.decode_attention(b, q_dev, pipe.k_out, pipe.v_out, pipe.offsets, out, pipe.ws, lse)
    torch.cuda.synchronize()
    offs = pipe.offsets.cpu().numpy()
    k_out, v_out = U.f32np(pipe.k_out), U.f32np(pipe.v_out)
    for i in range(len(items)):
        o = offs[i * wl.n_kv_heads:(i + 1) * wl.n_kv_heads + 1]
        want, want_lse = O.decode_attention(U.f32np(q[i]), k_out, v_out, o, wl.n_kv_heads)
        got = U.f32np(out[i]).astype(np.float64)
        scale = np.sqrt((want ** 2).mean())
        assert np.all(np.abs(got - want) <= 2.0 ** -7 * np.abs(want) + 2e-3 * scale + 1e-6), np.abs(got - want).max()
        assert np.all(np.abs(lse[i].cpu().numpy() - want_lse) <= 2e-3 * (1 + np.abs(want_lse)))


def test_cut_below_the_first_window_is_found_in_a_deeper_one(g):
    """A far-reaching p, and one dominant key over a long flat tail: the cut lies more than 12 logit units below
    the row maximum, outside the first 256-bin window.  Such rows get a second (third) window on the same grid
    instead of the exact selector; the masks still match the oracle's on the same stored queries."""
    wl = W.scaled(W.config(2), lengths=(6000, 1300), n_planted=(60, 10), S=8)
    items = W.make_items(wl, "cpu")
    refs = [U.oracle_item(wl, it) for it in items]
    stol = U.STAGE_TOL["bf16"]

    def run(its, q, p):
        b = U.batch_from(g, wl, U.to_device(its, DEV))
        pipe = g.Pipeline(b, wl.S, p)
        pipe.q.copy_(torch.tensor(np.stack(q)).to(pipe.q.dtype))
        pipe.select()
        torch.cuda.synchronize()
        out, off = [], 0
        for i, it in enumerate(its):
            out.append(U.unpack_rows(pipe.rowmask[off:off + pipe.mask_words[i]], pipe.rows, it["L"]).reshape(wl.S, wl.n_q_heads, it["L"]))
            off += pipe.mask_words[i]
        return out, pipe.fallback_rows(), pipe.refined_rows(), pipe.fallback_reasons()

    most = 0
    for p in (0.999, 0.9999, 0.99999, 0.999999):
        masks, n_fb, n_ref, why = run(items, [r["q_tilde"] for r in refs], p)
        nb = deep = 0
        for gm, r in zip(masks, refs):
            nb += U.check_rowmask_strict(gm, r["logits"], U.p32(p), min(stol, (1 - U.p32(p)) / 4),
                                         vtol=max((1 - U.p32(p)) / 2, 1e-6))
            lg = r["logits"]
            cut = np.where(r["rowmask"] if p == wl.p else np.stack([[O.top_p_select(lg[s, h], U.p32(p)) for h in range(wl.n_q_heads)]
                                                                      for s in range(wl.S)]), lg, np.inf).min(-1)
            deep += int((lg.max(-1) - cut > 16.0).sum())       # the first window ends 12 .. 16 units below the maximum
        say(f"  p {p}: rows settled in a deeper window {n_ref} (oracle cuts deeper than 16 units: {deep}), "
            f"redone exactly {n_fb} {why}, boundary keys {nb}")
        assert n_ref >= deep and why[0] == 0
        most = max(most, n_ref)
    assert most > 0
    # one dominant key 13 units above a long, nearly flat rest: the key alone holds 94.5 % of the mass, p = 0.95
    # needs hundreds of tail keys, the cut lies 12.7 units below the maximum
    wl = W.scaled(W.config(2), lengths=(30000,), n_planted=(60,), S=2)
    it = W.make_items(wl, "cpu")[0]
    ref = U.oracle_item(wl, it, upto="q")
    gen = torch.Generator().manual_seed(5)
    kf = (0.42 * torch.randn(it["k"].shape, generator=gen)).to(it["k"].dtype)
    qn = ref["q_tilde"][0].reshape(wl.n_kv_heads, wl.group, wl.d_k)[:, 0]           # one query direction per KV head
    qn = qn / np.linalg.norm(qn, axis=-1, keepdims=True)
    q1 = np.repeat(np.repeat(qn[:, None], wl.group, axis=1).reshape(1, wl.n_q_heads, wl.d_k), wl.S, axis=0) * 8.0
    q1 = U.f32np(torch.tensor(q1).to(torch.bfloat16)).astype(np.float64)
    kf[77] = torch.tensor(qn * (13.2 * np.sqrt(wl.d_k) / 8.0), dtype=torch.float32).to(kf.dtype)
    sink = dict(it, k=kf)
    lg = O.scores(q1, U.f32np(kf))
    masks, n_fb, n_ref, why = run([sink], [q1], 0.95)
    depth = np.array([lg[s, h].max() - lg[s, h][masks[0][s, h]].min() for s in range(wl.S) for h in range(wl.n_q_heads)])
    nb = U.check_rowmask_strict(masks[0], lg, U.p32(0.95), stol)
    say(f"  dominant key: rows settled in a deeper window {n_ref}, redone exactly {n_fb} {why}, boundary keys {nb}, "
        f"mean row size {masks[0].sum(-1).mean():.0f}, cut {depth.min():.2f} .. {depth.max():.2f} units below the maximum")
    assert depth.min() > 12.2 and why[0] == 0


@pytest.mark.parametrize("shape", [dict(S=16), dict(S=24), dict(S=20, d_k=64, n_q_heads=16, n_kv_heads=4, d=1024)],
                         ids=["64_rows", "96_rows", "head_dim_64"])
def test_second_histogram_on_full_and_partial_row_blocks(g, shape):
    """The second histogram pass on blocks of 64 rows (both 32-row halves in use), on a KV group with one full and
    one half-full block, and with head_dim 64; p = 0.9999 sends many rows below their first window."""
    wl = W.scaled(W.config(2), lengths=(2500, 700), n_planted=(30, 8), **shape)
    items = W.make_items(wl, "cpu")
    refs = [U.oracle_item(wl, it) for it in items]
    p = 0.9999
    b = U.batch_from(g, wl, U.to_device(items, DEV))
    pipe = g.Pipeline(b, wl.S, p)
    pipe.q.copy_(torch.tensor(np.stack([r["q_tilde"] for r in refs])).to(pipe.q.dtype))
    pipe.select()
    torch.cuda.synchronize()
    n_fb, n_ref, why = pipe.fallback_rows(), pipe.refined_rows(), pipe.fallback_reasons()
    off = nb = 0
    for i, (it, r) in enumerate(zip(items, refs)):
        gm = U.unpack_rows(pipe.rowmask[off:off + pipe.mask_words[i]], pipe.rows, it["L"]).reshape(wl.S, wl.n_q_heads, it["L"])
        off += pipe.mask_words[i]
        nb += U.check_rowmask_strict(gm, r["logits"], U.p32(p), min(U.STAGE_TOL["bf16"], (1 - U.p32(p)) / 4),
                                     vtol=max((1 - U.p32(p)) / 2, 1e-6))
    say(f"  rows settled by a second histogram {n_ref} of {len(items) * wl.S * wl.n_q_heads}, redone exactly {n_fb} {why}, boundary keys {nb}")
    assert n_ref > 0 and why[0] == 0


def test_large_logits_stay_exact(g):
    """Keys forty and four hundred times larger than the recipe's (and with the sign flipped): logits of several
    hundred to ten thousand units, bin numbers far beyond what the int16 tile bins hold (the histogram grid is
    absolute), windows raised in big jumps."""
    wl = W.scaled(W.config(2), lengths=(3000, 500), n_planted=(40, 6), S=8)
    items = W.make_items(wl, "cpu")
    refs = [U.oracle_item(wl, it, upto="q") for it in items]
    for scale in (40.0, 400.0, -400.0):
        big = [dict(it, k=(it["k"].to(torch.float32) * scale).to(it["k"].dtype)) for it in items]
        lgs = [O.scores(r["q_tilde"], U.f32np(it["k"])) for it, r in zip(big, refs)]
        b = U.batch_from(g, wl, U.to_device(big, DEV))
        pipe = g.Pipeline(b, wl.S, 0.9)
        pipe.q.copy_(torch.tensor(np.stack([r["q_tilde"] for r in refs])).to(pipe.q.dtype))
        pipe.select()
        torch.cuda.synchronize()
        off = nb = 0
        for i, it in enumerate(big):
            gm = U.unpack_rows(pipe.rowmask[off:off + pipe.mask_words[i]], pipe.rows, it["L"]).reshape(wl.S, wl.n_q_heads, it["L"])
            off += pipe.mask_words[i]
            # fp32 accumulation of a 128-term dot product: the logit error grows with the logit (about 2^-21 |l|), and
            # an error of delta in a logit is an error of delta in its share of the mass
            tol = max(U.STAGE_TOL["bf16"], 2.0 ** -21 * float(np.abs(lgs[i]).max()))
            nb += U.check_rowmask_strict(gm, lgs[i], U.p32(0.9), tol)
            m = lgs[i].max(-1).reshape(-1)
            assert np.all(np.abs(pipe.row_max[i].cpu().numpy() - m) <= U.STAGE_TOL["bf16"] * (1 + np.abs(m)))
        say(f"  keys x {scale:g}: largest |logit| {max(np.abs(l).max() for l in lgs):.0f}, boundary keys {nb}, "
            f"redone exactly {pipe.fallback_rows()} {pipe.fallback_reasons()}")


def test_crowded_cut_bin_is_looked_into_with_finer_bins(g):
    """Nearly flat attention over a long context: thousands of keys share the 1/16-logit bin of the cut, more than the
    candidate resolver holds.  The bin is then split into 256 finer ones (a second histogram pass) instead of handing
    the row to the exact selector.  Both selection rules."""
    wl = W.scaled(W.config(2), lengths=(30000, 9000), n_planted=(60, 20), S=2)
    items = W.make_items(wl, "cpu")
    gen = torch.Generator().manual_seed(9)
    stol = U.STAGE_TOL["bf16"]
    flat, qs, lgs = [], [], []
    for it in items:
        ref = U.oracle_item(wl, it, upto="q")
        kf = (0.03 * torch.randn(it["k"].shape, generator=gen)).to(it["k"].dtype)
        flat.append(dict(it, k=kf))
        qs.append(ref["q_tilde"])
        lgs.append(O.scores(ref["q_tilde"], U.f32np(kf)))
    b = U.batch_from(g, wl, U.to_device(flat, DEV))
    pipe = g.Pipeline(b, wl.S, 0.9)
    pipe.q.copy_(torch.tensor(np.stack(qs)).to(pipe.q.dtype))
    pipe.select()
    torch.cuda.synchronize()
    n_fb, n_ref, why = pipe.fallback_rows(), pipe.refined_rows(), pipe.fallback_reasons()
    off = nb = 0
    for i, it in enumerate(flat):
        gm = U.unpack_rows(pipe.rowmask[off:off + pipe.mask_words[i]], pipe.rows, it["L"]).reshape(wl.S, wl.n_q_heads, it["L"])
        off += pipe.mask_words[i]
        nb += U.check_rowmask_strict(gm, lgs[i], U.p32(0.9), stol)
    in_bin = int(((lgs[0][0, 0] * 16 >= np.floor(np.sort(lgs[0][0, 0])[3000] * 16)) & (lgs[0][0, 0] * 16 < np.floor(np.sort(lgs[0][0, 0])[3000] * 16) + 1)).sum())
    say(f"  top-p: rows settled by a second histogram {n_ref}, redone exactly {n_fb} {why}, boundary keys {nb}; "
        f"about {in_bin} of {flat[0]['L']} keys share a 1/16-logit bin")
    assert n_ref > 0 and n_fb == 0
    # the same rows by count (Alg. 1's TopK): k in the crowded region
    R = wl.S * wl.n_q_heads
    ks = torch.tensor(np.tile((np.arange(R) * 131 % 7000 + 1500).astype(np.int32), len(flat)), device=DEV)
    g.score_select(b, wl.S, pipe.q, 0.5, pipe.rowmask, mode=g.SELECT_TOPK, k_per_row=ks, ws=pipe.ws)
    torch.cuda.synchronize()
    n_fb, n_ref = pipe.fallback_rows(), pipe.refined_rows()
    off = 0
    kk = ks.cpu().numpy().reshape(len(flat), R)
    for i, it in enumerate(flat):
        gm = U.unpack_rows(pipe.rowmask[off:off + pipe.mask_words[i]], pipe.rows, it["L"]).reshape(R, it["L"])
        off += pipe.mask_words[i]
        lg = lgs[i].reshape(R, -1)
        for r in range(R):
            k = min(int(kk[i, r]), it["L"])
            assert gm[r].sum() == k, (i, r, gm[r].sum(), k)
            # the k-th largest logit separates the sets up to the score tolerance
            assert lg[r][gm[r]].min() >= (lg[r][~gm[r]].max() if k < it["L"] else -np.inf) - U.logit_slack(lg[r], stol)
    say(f"  top-k: rows settled by a second histogram {n_ref}, redone exactly {n_fb}")
    assert n_ref > 0 and n_fb == 0


def test_first_pass_give_up_path_sends_rows_to_the_exact_selector(g):
    """With a spin limit of 0 a first-pass wave that finishes before its workgroup gives up at once: the
    workgroup publishes no histogram, its rows are flagged and the exact selector redoes them.  The masks
    must still be the oracle's, and the give-up counter must say what happened."""
    wl = W.scaled(W.config(2), lengths=(3000, 1100), n_planted=(40, 10), S=8)
    items = W.make_items(wl, "cpu")
    refs = [U.oracle_item(wl, it) for it in items]
    b = U.batch_from(g, wl, U.to_device(items, DEV))
    pipe = g.Pipeline(b, wl.S, wl.p)
    pipe.q.copy_(torch.tensor(np.stack([r["q_tilde"] for r in refs])).to(pipe.q.dtype))
    old = g.debug_set_spin_limit(0)
    try:
        pipe.select()
        torch.cuda.synchronize()
    finally:
        g.debug_set_spin_limit(old)
    n_fb, why = pipe.fallback_rows(), pipe.fallback_reasons()
    say(f"  spin limit 0: {n_fb} rows redone exactly, by reason {why}")
    assert why[3] > 0 and n_fb >= why[3]
    off = 0
    for i, (it, r) in enumerate(zip(items, refs)):
        L = it["L"]
        gm = U.unpack_rows(pipe.rowmask[off:off + pipe.mask_words[i]], pipe.rows, L).reshape(wl.S, wl.n_q_heads, L)
        off += pipe.mask_words[i]
        U.check_rowmask_strict(gm, r["logits"], U.p32(wl.p), U.STAGE_TOL[wl.dtype])
    pipe.select()                       # and with the default limit nothing gives up
    torch.cuda.synchronize()
    assert pipe.fallback_reasons()[3] == 0
