"""Pins of the CPU oracle against things other than itself: the generator's published known-answer
vectors, closed forms, distribution laws from SciPy, brute-force enumeration and hand-built cases.
Each test is chosen so that a plausible slip in the oracle (dropped term, wrong sign or index,
transposed operand, wrong pairing) makes it fail.  CPU only."""
import itertools
import math
import os

import numpy as np
import pytest
from scipy import stats

import oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- Philox integers
def test_philox_known_answers():
    n = 0
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(x, 16) for x in line.split()]
        out = O.philox4x32_10(np.array(v[:4], dtype=np.uint32), np.array(v[4:6], dtype=np.uint32))
        assert out.tolist() == v[6:]
        n += 1
    assert n == 3


def test_philox_stream_layout_is_random_access():
    # draw e alone == draw e of a bulk fill; block index spills into the second counter word
    seed, sid = 0x1234_5678_9ABC_DEF0, 0x0FED_CBA9_8765_4321
    bulk = O.philox_u32_stream(seed, sid, 1027)
    for e in (0, 1, 5, 1026):
        blk = e >> 2
        ctr = np.array([blk & 0xFFFFFFFF, blk >> 32, sid & 0xFFFFFFFF, sid >> 32], dtype=np.uint32)
        key = np.array([seed & 0xFFFFFFFF, seed >> 32], dtype=np.uint32)
        assert O.philox4x32_10(ctr, key)[e & 3] == bulk[e]
    # the third golden vector read as a stream: ctr=(blk_lo, blk_hi, sid_lo, sid_hi), key=(seed_lo, seed_hi)
    blk = 0x85A308D3_243F6A88
    sid = 0x03707344_13198A2E
    seed = 0x299F31D0_A4093822
    ctr = np.array([[blk & 0xFFFFFFFF, blk >> 32, sid & 0xFFFFFFFF, sid >> 32]], dtype=np.uint32)
    key = np.array([seed & 0xFFFFFFFF, seed >> 32], dtype=np.uint32)
    assert O.philox4x32_10(ctr, key)[0].tolist() == [0xD16CFE09, 0x94FDCCEB, 0x5001E420, 0x24126EA1]
    # first S of S+1 samples are identical (counter-based indexing)
    a = O.standard_normals(7, 3, 4, 64)
    b = O.standard_normals(7, 3, 5, 64)
    assert np.array_equal(a, b[:4])
    assert not np.array_equal(O.standard_normals(7, 4, 4, 64), a)
    assert not np.array_equal(O.standard_normals(8, 3, 4, 64), a)


def test_uniform_is_open_interval_and_exact():
    u = O.uniform_from_u32(np.array([0, 0x1FF, 0x200, 0xFFFFFFFF], dtype=np.uint32))
    assert u[0] == 2.0 ** -24 and u[1] == 2.0 ** -24 and u[2] == 1.5 * 2.0 ** -23
    assert u[3] == 1.0 - 2.0 ** -24
    assert np.all(u.astype(np.float32).astype(np.float64) == u)       # representable in fp32


# ---------------------------------------------------------------- normals
def test_normals_follow_the_standard_normal_law():
    z = O.standard_normals(11, 0, 64, 4096)
    n = z.size
    assert abs(z.mean()) < 5 / math.sqrt(n)
    assert abs(z.var() - 1.0) < 5 * math.sqrt(2.0 / n)
    assert abs((z ** 3).mean()) < 5 * math.sqrt(15.0 / n)
    assert abs((z ** 4).mean() - 3.0) < 5 * math.sqrt(96.0 / n)
    assert stats.kstest(z.reshape(-1)[:100000], "norm").pvalue > 1e-3
    # the two outputs of a pair are uncorrelated, neighbouring pairs too
    flat = z.reshape(-1, 4)
    for a, b in ((0, 1), (2, 3), (0, 2), (1, 3)):
        assert abs(np.corrcoef(flat[:, a], flat[:, b])[0, 1]) < 5 / math.sqrt(flat.shape[0])
    # radius^2 of a pair is chi-square with 2 dof, its angle uniform
    r2 = flat[:, 0] ** 2 + flat[:, 1] ** 2
    assert stats.kstest(r2[:50000], "chi2", args=(2,)).pvalue > 1e-3
    ang = np.arctan2(flat[:, 1], flat[:, 0]) / (2 * np.pi) % 1.0
    assert stats.kstest(ang[:50000], "uniform").pvalue > 1e-3


def test_sample_moments_converge_to_the_fitted_gaussian():
    d = 8
    mu = np.linspace(-2, 2, d).astype(np.float32)
    var = np.linspace(0.25, 4, d).astype(np.float32)
    S = 1 << 16
    h = O.sample_hidden(mu, var, O.standard_normals(5, 9, S, d), "f32")
    assert np.all(np.abs(h.mean(0) - mu) < 5 * np.sqrt(var / S))
    assert np.all(np.abs(h.var(0) / var - 1) < 5 * math.sqrt(2.0 / S))
    # sigma = 0 gives the mean exactly; bf16 storage rounds to 8 significant bits
    h0 = O.sample_hidden(mu, np.zeros(d, np.float32), O.standard_normals(5, 9, 4, d), "f32")
    assert np.array_equal(h0, np.broadcast_to(mu.astype(np.float64), (4, d)))


def test_round_to_dtype():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -7, -3.14159, 0.0, 1e-3, 255.5, 256.5 * 2])
    r = O.round_to_dtype(x, "bf16")
    #   1+2^-8 is a tie -> even (1.0); 1+3*2^-8 is a tie -> even (1+2^-6)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0 + 2 ** -6 and r[3] == 1.0 + 2 ** -7
    assert r[4] == -3.140625 and r[5] == 0.0 and r[7] == 256.0 and r[8] == 512.0
    import torch
    t = torch.tensor(np.random.default_rng(0).standard_normal(20000) * 37.0, dtype=torch.float64)
    want = t.to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    got = O.round_to_dtype(t.numpy(), "bf16")
    assert np.mean(got != want) < 1e-3            # differs only through fp32 double rounding
    assert np.allclose(got, want, rtol=2 ** -7)
    assert np.array_equal(O.round_to_dtype(t.numpy(), "f32"), t.to(torch.float32).to(torch.float64).numpy())


# ---------------------------------------------------------------- moments
@pytest.mark.parametrize("ddof", [0, 1])
def test_moments_closed_form_arithmetic_progression(ddof):
    L, d, n_skip = 1000, 6, 4
    a = np.arange(d, dtype=np.float64) - 2.0
    b = 0.5 + np.arange(d, dtype=np.float64)
    t = np.arange(L, dtype=np.float64)
    h = a[None, :] + b[None, :] * t[:, None]
    h[:n_skip] = 1e6                                    # skipped tokens must not matter
    mu, var = O.fit_gaussian(h, n_skip, ddof)
    n = L - n_skip
    want_mu = a + b * (n_skip + L - 1) / 2.0
    want_var = b ** 2 * (n * n - 1) / 12.0 * (n / (n - ddof))
    assert np.allclose(mu, want_mu, rtol=1e-6)
    assert np.allclose(var, want_var, rtol=1e-6)
    assert mu.dtype == np.float32 and var.dtype == np.float32


def test_moments_recover_generating_gaussian_and_invariances():
    rng = np.random.default_rng(3)
    L, d = 20000, 5
    mu_t = rng.normal(size=d)
    sd_t = rng.uniform(0.5, 1.5, size=d)
    h = mu_t + sd_t * rng.normal(size=(L, d))
    mu, var = O.fit_gaussian(h, 0, 1)
    assert np.all(np.abs(mu - mu_t) < 5 * sd_t / math.sqrt(L))
    assert np.all(np.abs(var / sd_t ** 2 - 1) < 5 * math.sqrt(2.0 / L))
    _, var_shift = O.fit_gaussian(h + 100.0, 0, 1)
    assert np.allclose(var_shift, var, rtol=1e-5)
    mu_c, var_c = O.fit_gaussian(np.full((50, 3), 2.5), 0, 1)
    assert np.all(mu_c == 2.5) and np.all(var_c == 0)


# ---------------------------------------------------------------- RoPE and projection
def test_rope_cos_sin_closed_forms():
    theta, dk = 1.0e4, 8
    c, s = O.rope_cos_sin(theta, dk, 0, 1)
    assert np.array_equal(c, np.ones(4)) and np.array_equal(s, np.zeros(4))          # position 0 = identity
    c, s = O.rope_cos_sin(theta, dk, 5, 1)
    assert np.allclose(c ** 2 + s ** 2, 1.0)
    om = np.array([1.0, 0.1, 0.01, 0.001])                                            # 1e4^(-2i/8)
    assert np.allclose(c, np.cos(5 * om)) and np.allclose(s, np.sin(5 * om))
    # mean over n positions a..a+n-1: cos((a+(n-1)/2) w) sin(n w/2) / (n sin(w/2))
    a, n = 100, 7
    c, s = O.rope_cos_sin(theta, dk, a, n)
    k = np.sin(n * om / 2) / (n * np.sin(om / 2))
    assert np.allclose(c, np.cos((a + (n - 1) / 2) * om) * k)
    assert np.allclose(s, np.sin((a + (n - 1) / 2) * om) * k)


def test_projection_orientation_bias_and_rotation_sign():
    S, d, hq, dk = 2, 6, 2, 2
    h = np.arange(S * d, dtype=np.float64).reshape(S, d) + 1.0
    w = np.zeros((hq * dk, d))
    w[3, 5] = 1.0                       # output 3 (head 1, lane 1) reads channel 5
    w[0, 2] = 2.0                       # output 0 (head 0, lane 0) reads twice channel 2
    one, zero = np.ones(1), np.zeros(1)
    q = O.project_rope(h, w, None, one, zero, hq, dk, "f32")
    assert q.shape == (S, hq, dk)
    assert np.array_equal(q[:, 1, 1], h[:, 5]) and np.array_equal(q[:, 0, 0], 2 * h[:, 2])
    assert np.all(q[:, 0, 1] == 0) and np.all(q[:, 1, 0] == 0)
    qb = O.project_rope(h, w, np.array([0.0, 10.0, 0.0, 0.0]), one, zero, hq, dk, "f32")
    assert np.array_equal(qb[:, 0, 1], np.full(S, 10.0))
    # quarter turn: (x, 0) -> (0, x) for the pair (i, i + d_k/2)
    c, s = O.rope_cos_sin(7.0, 2, 1, 1)                 # d_k = 2: one frequency, omega = 1, angle 1 rad
    assert np.allclose([c[0], s[0]], [math.cos(1.0), math.sin(1.0)])
    q = O.project_rope(h, w, None, np.zeros(1), np.ones(1), hq, dk, "f32")
    assert np.array_equal(q[:, 0, 1], 2 * h[:, 2]) and np.all(q[:, 0, 0] == 0)       # head 0: (x,0)->(0,x)
    assert np.array_equal(q[:, 1, 0], -h[:, 5]) and np.all(q[:, 1, 1] == 0)          # head 1: (0,y)->(-y,0)


def test_rope_relative_position_and_norm():
    rng = np.random.default_rng(1)
    dk, theta = 16, 5.0e5
    q = rng.normal(size=(1, dk))
    k = rng.normal(size=(1, dk))
    eye = np.eye(dk)

    def rot(x, pos):
        c, s = O.rope_cos_sin(theta, dk, pos, 1)
        return O.project_rope(x, eye, None, c, s, 1, dk, "f32")[:, 0, :]
    assert np.allclose(np.linalg.norm(rot(q, 77)), np.linalg.norm(q), rtol=1e-6)
    d1 = (rot(q, 40) @ rot(k, 33).T).item()
    d2 = (rot(q, 1040) @ rot(k, 1033).T).item()
    assert abs(d1 - d2) < 1e-5
    assert abs(d1 - (rot(q, 41) @ rot(k, 33).T).item()) > 1e-4


def test_sigma_zero_makes_every_sample_the_rotated_mean_projection():
    rng = np.random.default_rng(2)
    d, hq, dk, S = 12, 2, 4, 3
    mu = rng.normal(size=d).astype(np.float32)
    w = rng.normal(size=(hq * dk, d))
    h = O.sample_hidden(mu, np.zeros(d, np.float32), O.standard_normals(1, 1, S, d), "f32")
    c, s = O.rope_cos_sin(1e4, dk, 9, 1)
    q = O.project_rope(h, w, None, c, s, hq, dk, "f32")
    lin = (w @ mu.astype(np.float64)).reshape(hq, dk)
    want = np.concatenate([lin[:, :2] * c - lin[:, 2:] * s, lin[:, 2:] * c + lin[:, :2] * s], axis=-1)
    for sidx in range(S):
        assert np.allclose(q[sidx], want, rtol=1e-6, atol=1e-6)


# ---------------------------------------------------------------- scores
def test_scores_one_hot_and_group_mapping():
    S, hq, hkv, dk, L = 2, 4, 2, 4, 5
    k = np.arange(L * hkv * dk, dtype=np.float64).reshape(L, hkv, dk)
    q = np.zeros((S, hq, dk))
    q[0, 0, 1] = 1.0        # head 0 -> kv head 0, picks component 1
    q[0, 3, 2] = 1.0        # head 3 -> kv head 1, picks component 2
    q[1, 2, 0] = -2.0       # head 2 -> kv head 1
    lg = O.scores(q, k)
    assert lg.shape == (S, hq, L)
    assert np.allclose(lg[0, 0], k[:, 0, 1] / 2.0)
    assert np.allclose(lg[0, 3], k[:, 1, 2] / 2.0)
    assert np.allclose(lg[1, 2], -2.0 * k[:, 1, 0] / 2.0)
    assert np.all(lg[1, 0] == 0)
    m, w, Z = O.softmax_weights(lg[0, 0])
    assert m == lg[0, 0].max() and abs((w / Z).sum() - 1) < 1e-12
    m2, w2, Z2 = O.softmax_weights(lg[0, 0] + 123.0)
    assert np.allclose(w2, w) and np.isclose(Z2, Z)


# ---------------------------------------------------------------- top-p selection
def _brute_force_minimal_set(w, p):
    """Smallest cardinality reaching mass p, and the largest mass attainable at that cardinality."""
    L = len(w)
    Z = sum(w)
    for size in range(1, L + 1):
        best = max(sum(c) for c in itertools.combinations(w, size))
        if best >= p * Z:
            return size, best
    return L, Z


@pytest.mark.parametrize("seed", range(12))
def test_top_p_equals_brute_force_subset_enumeration(seed):
    rng = np.random.default_rng(seed)
    L = int(rng.integers(3, 13))
    l = rng.normal(scale=rng.uniform(0.3, 3.0), size=L)
    if seed % 3 == 0:
        l[rng.integers(0, L)] = l[rng.integers(0, L)]         # a tie
    p = float(rng.uniform(0.3, 0.99))
    mask = O.top_p_select(l, p)
    _, w, Z = O.softmax_weights(l)
    size, best = _brute_force_minimal_set(list(w), p)
    assert mask.sum() == size
    assert w[mask].sum() >= p * Z
    assert np.isclose(w[mask].sum(), best, rtol=1e-12)
    assert w[mask].min() >= w[~mask].max() if (~mask).any() else True


def test_top_p_closed_forms_and_ties():
    L = 512
    assert O.top_p_select(np.zeros(L), 0.9).sum() == math.ceil(0.9 * L)              # uniform attention
    assert np.array_equal(np.nonzero(O.top_p_select(np.zeros(L), 0.9))[0], np.arange(461))  # lowest indices win ties
    one_hot = np.full(L, -1e4)
    one_hot[77] = 0.0
    m = O.top_p_select(one_hot, 0.999)
    assert m.sum() == 1 and m[77]
    # geometric weights r^i: prefix mass (1 - r^k)/(1 - r^L) -> k* = ceil(ln(1 - p(1 - r^L)) / ln r)
    r, p = 0.8, 0.95
    l = np.log(r) * np.arange(200)
    k_star = math.ceil(math.log(1 - p * (1 - r ** 200)) / math.log(r))
    got = O.top_p_select(l[::-1].copy(), p)            # reversed: best keys have the highest indices
    assert got.sum() == k_star and np.all(got[-k_star:]) and not got[:-k_star].any()
    assert O.top_p_select(l, 1.0).all()
    # monotone in p
    rng = np.random.default_rng(0)
    l = rng.normal(size=300) * 2
    prev = np.zeros(300, bool)
    for p in (0.1, 0.5, 0.9, 0.95, 0.999):
        cur = O.top_p_select(l, p)
        assert cur.sum() >= 1 and np.all(cur[prev])
        prev = cur
    # tie at the cut: two equal logits, only one is needed -> the lower index
    l = np.array([0.0, 5.0, 1.0, 5.0, -3.0])
    m = O.top_p_select(l, 0.4)
    assert m.tolist() == [False, True, False, False, False]
    m = O.top_p_select(l, 0.6)
    assert m.tolist() == [False, True, False, True, False]


def test_top_k_select():
    l = np.array([0.0, 5.0, 1.0, 5.0, -3.0])
    assert O.top_k_select(l, 1).tolist() == [False, True, False, False, False]
    assert O.top_k_select(l, 3).tolist() == [False, True, True, True, False]
    assert O.top_k_select(l, 9).all()


# ---------------------------------------------------------------- union, count, compaction
def test_union_budget_and_compaction_hand_example():
    S, hq, hkv, L, dk = 2, 4, 2, 6, 3
    rm = np.zeros((S, hq, L), bool)
    rm[0, 0, [0, 2]] = True     # kv 0
    rm[1, 1, [2, 5]] = True     # kv 0
    rm[0, 2, [1]] = True        # kv 1
    rm[1, 3, [1, 4]] = True     # kv 1
    union, budget = O.union_vote(rm, hkv)
    assert union.tolist() == [[True, False, True, False, False, True], [False, True, False, False, True, False]]
    assert budget.tolist() == [3, 2]
    k = np.arange(L * hkv * dk, dtype=np.float32).reshape(L, hkv, dk)
    v = -k
    ko, vo, idx, offs = O.compact(k, v, union)
    assert offs.tolist() == [0, 3, 5] and idx.tolist() == [0, 2, 5, 1, 4]
    assert np.array_equal(ko, np.stack([k[0, 0], k[2, 0], k[5, 0], k[1, 1], k[4, 1]]))
    assert np.array_equal(vo, -ko)
    # union is at least every row set, at most the sum, and at most L
    for s in range(S):
        for h in range(hq):
            assert budget[h // 2] >= rm[s, h].sum()
    assert np.all(budget <= L)


def test_mask_word_packing():
    m = np.zeros((2, 70), bool)
    m[0, [0, 31, 32, 69]] = True
    m[1, 33] = True
    w = O.pack_mask_words(m)
    assert w.dtype == np.uint32 and w.shape == (2, 3)
    assert w[0].tolist() == [0x80000001, 0x1, 0x20] and w[1].tolist() == [0, 2, 0]
    assert np.array_equal(O.unpack_mask_words(w, 70), m)


# ---------------------------------------------------------------- the composed path: invariants
def test_path_invariants_on_tiny_workload():
    import torch
    from synth import workloads as W
    wl = W.config(1)
    it = W.make_item(wl, 0)
    f = lambda x: x.to(torch.float32).numpy()
    kw = dict(n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, d_k=wl.d_k, theta=wl.theta, seed=1,
              stream_id=0, dtype="f32")
    base = O.gvote_item(f(it["hidden"]), f(it["w_q"]), None, f(it["k"]), f(it["v"]), S=4, p=0.5, **kw)
    G = wl.group
    for s in range(4):
        for h in range(wl.n_q_heads):
            assert base["budget"][h // G] >= base["rowmask"][s, h].sum() >= 1
    assert np.all(base["budget"] <= 512)
    more_s = O.gvote_item(f(it["hidden"]), f(it["w_q"]), None, f(it["k"]), f(it["v"]), S=8, p=0.5, **kw)
    assert np.all(more_s["union"][base["union"]])                        # union grows with S
    more_p = O.gvote_item(f(it["hidden"]), f(it["w_q"]), None, f(it["k"]), f(it["v"]), S=4, p=0.8, **kw)
    assert np.all(more_p["union"][base["union"]])                        # and with p
    allp = O.gvote_item(f(it["hidden"]), f(it["w_q"]), None, f(it["k"]), f(it["v"]), S=4, p=1.0, **kw)
    assert allp["union"].all() and np.array_equal(allp["k_out"], f(it["k"]).transpose(1, 0, 2).reshape(-1, wl.d_k))
    one = O.gvote_item(f(it["hidden"]), f(it["w_q"]), None, f(it["k"]), f(it["v"]), S=1, p=0.5,
                       **{**kw, "n_q_heads": wl.n_q_heads})
    # S = 1 with one head per group reduces to the single query's threshold set
    lg = one["logits"]
    assert np.array_equal(one["rowmask"][0, 0], O.top_p_select(lg[0, 0], 0.5))


# ---------------------------------------------------------------- consumer side
def test_decode_attention_closed_forms_and_scipy():
    from scipy.special import softmax, logsumexp
    rng = np.random.default_rng(6)
    hq, hkv, dk = 4, 2, 8
    offs = np.array([0, 5, 12])
    k = rng.normal(size=(12, dk))
    v = rng.normal(size=(12, dk))
    q = rng.normal(size=(hq, dk))
    out, lse = O.decode_attention(q, k, v, offs, hkv)
    for h in range(hq):
        lo, hi = offs[h // 2], offs[h // 2 + 1]
        l = k[lo:hi] @ q[h] / math.sqrt(dk)
        assert np.allclose(out[h], softmax(l) @ v[lo:hi]) and np.isclose(lse[h], logsumexp(l))
    # equal keys -> plain mean of the head's values; a dominant key -> its value row
    out, _ = O.decode_attention(q, np.ones_like(k), v, offs, hkv)
    assert np.allclose(out[0], v[0:5].mean(0)) and np.allclose(out[3], v[5:12].mean(0))
    kd = np.zeros_like(k)
    kd[7] = 100.0 * q[2] / np.linalg.norm(q[2])
    out, _ = O.decode_attention(q, kd, v, offs, hkv)
    assert np.allclose(out[2], v[7], atol=1e-9)


def test_attention_overlap_identities():
    rng = np.random.default_rng(7)
    S, hq, hkv, dk, L = 3, 4, 2, 8, 40
    k = rng.normal(size=(L, hkv, dk))
    q = rng.normal(size=(hq, dk))
    rm = rng.random((S, hq, L)) < 0.3
    ov = O.attention_overlap(q, k, rm)
    assert np.all(ov >= 0) and np.all(ov <= 1 + 1e-12)
    assert np.allclose(ov + O.attention_overlap(q, k, ~rm), 1.0)               # a set and its complement
    assert np.allclose(O.attention_overlap(q, k, np.ones_like(rm)), 1.0)
    # the real query's own top-p set overlaps itself by at least p
    lg = O.scores(q[None], k)[0]
    own = np.stack([O.top_p_select(lg[h], 0.9) for h in range(hq)])[None]
    assert np.all(O.attention_overlap(q, k, own) >= 0.9 - 1e-12)


def test_consumer_side_hand_worked_values():
    """Values worked out by hand (Eq. (1)-(2), Sec. 3.3): with d_k = 4 and q = (2, 0, 0, 0) a key (ln w, 0, 0, 0) has logit
    ln w, i.e. attention weight w / sum(w)."""
    ln = math.log
    # decode attention over a packed cache of two heads with two rows each
    q = np.array([[2.0, 0, 0, 0], [2.0, 0, 0, 0]])
    k_out = np.array([[ln(1), 0, 0, 0], [ln(3), 0, 0, 0], [ln(2), 0, 0, 0], [ln(2), 0, 0, 0]])
    v_out = np.array([[1.0, 0, 0, 0], [0, 1.0, 0, 0], [0, 0, 8.0, 0], [0, 0, 0, 4.0]])
    out, lse = O.decode_attention(q, k_out, v_out, np.array([0, 2, 4]), 2)
    assert np.allclose(out[0], [0.25, 0.75, 0, 0]) and np.allclose(out[1], [0, 0, 4.0, 2.0])
    assert np.allclose(lse, [ln(4), ln(4)])
    # one KV head shared by both query heads: the group map sends both to rows 0..3
    out, lse = O.decode_attention(np.array([[2.0, 0, 0, 0], [4.0, 0, 0, 0]]), k_out, v_out, np.array([0, 4]), 1)
    assert np.allclose(out[0], [1 / 8, 3 / 8, 2.0, 1.0]) and np.allclose(lse[0], ln(8))
    assert np.allclose(out[1], [1 / 18, 9 / 18, 8 * 4 / 18, 4 * 4 / 18]) and np.allclose(lse[1], ln(18))   # weights w^2
    # overlap: weights (1, 2, 3, 4) / 10 for head 0 on KV head 0, (4, 3, 2, 1) / 10 for head 1 on KV head 1
    k = np.zeros((4, 2, 4))
    k[:, 0, 0] = [ln(1), ln(2), ln(3), ln(4)]
    k[:, 1, 0] = [ln(4), ln(3), ln(2), ln(1)]
    rm = np.zeros((2, 2, 4), dtype=bool)
    rm[0, 0, [1, 3]] = True          # sample 0, head 0: keys 1 and 3 -> 0.2 + 0.4
    rm[0, 1, 0] = True               # sample 0, head 1: key 0 -> 0.4
    rm[1, 0, 0] = True               # sample 1, head 0: key 0 -> 0.1
    rm[1, 1, [2, 3]] = True          # sample 1, head 1: keys 2, 3 -> 0.3
    ov = O.attention_overlap(q, k, rm)
    assert np.allclose(ov, [[0.6, 0.4], [0.1, 0.3]])
    # both query heads on one KV head, the second with twice the query: weights w^2 / 30
    ov = O.attention_overlap(np.array([[2.0, 0, 0, 0], [4.0, 0, 0, 0]]), k[:, :1], rm)
    assert np.allclose(ov, [[0.6, 1 / 30], [0.1, (9 + 16) / 30]])


# ---------------------------------------------------------------- test infrastructure itself
def test_band_sets_bracket_the_oracle_selection():
    import sys
    sys.path.insert(0, os.path.dirname(__file__))
    import parity_util as U
    rng = np.random.default_rng(4)
    for _ in range(20):
        l = rng.normal(scale=2.0, size=200)
        p = float(rng.uniform(0.5, 0.99))
        sel = O.top_p_select(l, p)
        must, may = U.band_sets(l, p, 1e-3)
        assert np.all(sel[must]) and np.all(may[sel])
        must0, may0 = U.band_sets(l, p, 0.0)
        # with no tolerance only the key that crosses p is free
        assert (may0 & ~must0).sum() <= 1 and np.all(sel[must0]) and np.all(may0[sel])


def test_mask_checks_reject_planted_mistakes():
    """The mask checks of the GPU parity tests, exercised on mistakes planted into the ORACLE's own
    selection (CPU only): a set short of p by a whole heavy key (which the interval band alone lets pass),
    a set with a superfluous key, a set that skips a heavier key for a lighter one."""
    import sys
    sys.path.insert(0, os.path.dirname(__file__))
    import parity_util as U
    p, tol = 0.95, 2e-3
    w = np.array([0.50, 0.44, 0.02, 0.015, 0.010] + [0.015 / 30] * 30)       # masses; cumulative 0.5, 0.94, 0.96 ...
    l = np.log(w)
    good = O.top_p_select(l, p)
    assert good.sum() == 3
    lg, gm = l[None, None, :], good[None, None, :]
    assert U.check_rowmask_strict(gm, lg, p, tol) == 0 and U.check_rowmask_sandwich(gm, lg, p, tol) == 0
    short = good.copy(); short[2] = False                 # mass 0.94: short of p - tol by the key that straddles p
    must, may = U.band_sets(l, p, tol)
    assert np.all(short[must]) and np.all(may[short])     # the band alone accepts it ...
    for check in (U.check_rowmask_strict, U.check_rowmask_sandwich):
        with pytest.raises(AssertionError):               # ... the validity asserts do not
            check(short[None, None, :], lg, p, tol)
    fat = good.copy(); fat[3] = True                       # one key too many: not minimal
    skip = good.copy(); skip[2] = False; skip[3] = True; skip[4] = True        # lighter keys instead of a heavier one
    for bad in (fat, skip):
        for check in (U.check_rowmask_strict, U.check_rowmask_sandwich):
            with pytest.raises(AssertionError):
                check(bad[None, None, :], lg, p, tol)
    # two nearly tied heavy keys at the boundary may swap end to end (band + validity) but not under the strict check
    w2 = np.array([0.60, 0.30, 0.04, 0.0101, 0.0100] + [0.0399 / 40] * 40)   # cumulative 0.6, 0.9, 0.94, 0.9501
    l2 = np.log(w2)
    sel = O.top_p_select(l2, p)
    assert sel.sum() == 4
    swapped = sel.copy(); swapped[3] = False; swapped[4] = True              # mass 0.95 exactly, still reaches p - tol
    U.check_rowmask_sandwich(swapped[None, None, :], l2[None, None, :], p, tol)
    with pytest.raises(AssertionError):
        U.check_rowmask_strict(swapped[None, None, :], l2[None, None, :], p, tol)
    # ... also when the tied pair is so heavy that the second key's interval starts beyond p + tol (two keys of 1 % each,
    # logits 1e-5 apart: one query element rounding the other way swaps them); a key that is lighter by more than the
    # score tolerance is no substitute
    w3 = np.array([0.60, 0.30, 0.048, 0.0106, 0.0106 * (1 - 1e-5), 0.009] + [0.02180011 / 40] * 40)
    l3 = np.log(w3)
    sel = O.top_p_select(l3, p)
    assert sel.sum() == 4 and sel[3] and not sel[4]
    must, may = U.band_sets(l3, p, tol)
    assert not may[4]                                                        # the band alone would refuse key 4
    twin = sel.copy(); twin[3] = False; twin[4] = True
    U.check_rowmask_sandwich(twin[None, None, :], l3[None, None, :], p, tol)
    with pytest.raises(AssertionError):
        U.check_rowmask_strict(twin[None, None, :], l3[None, None, :], p, tol)
    lighter = sel.copy(); lighter[3] = False; lighter[5] = True             # 0.9 % instead of 1.06 %: logits 0.16 apart
    with pytest.raises(AssertionError):
        U.check_rowmask_sandwich(lighter[None, None, :], l3[None, None, :], p, tol)
    U.check_budgets([100, 4000], [104, 4080])
    with pytest.raises(AssertionError):
        U.check_budgets([100], [120])


def test_workload_generator_is_seeded_and_shaped():
    from synth import workloads as W
    wl = W.scaled(W.config(5), lengths=(200, 90))
    a, b = W.make_items(wl, "cpu"), W.make_items(wl, "cpu")
    for x, y in zip(a, b):
        for k in ("hidden", "w_q", "k", "v"):
            assert x[k].dtype == wl.torch_dtype and bool((x[k] == y[k]).all())
    assert a[0]["hidden"].shape == (200, wl.d) and a[1]["k"].shape == (90, wl.n_kv_heads, wl.d_k)
    assert a[0]["w_q"].data_ptr() == a[1]["w_q"].data_ptr()          # one layer, many requests
    assert [W.config(i).n_items for i in range(1, 6)] == [1, 1, 32, 28, 16]
    assert min(W.config(5).lengths) >= 1024 and max(W.config(5).lengths) <= 16384
