"""Plain fp64 NumPy oracle of GVote's selection path.  TEST INFRASTRUCTURE ONLY.

Every function takes the steps of the paper in the paper's order and notation;
nothing is blocked, fused or reordered.  Floating point is fp64 except at the
two stated rounding points (the sampled hidden state and the synthetic query
are stored in the model dtype, as a model would store them).

What is computed (one "item" = one request x one layer):

  fit_gaussian      Sec. 3.2 Step 2 / Alg. 1 "mean, var of h"; first n_s tokens skipped
  philox4x32_10     counter-based generator (Salmon et al., SC'11) used for the draws
  standard_normals  Box-Muller on the Philox stream
  sample_hidden     Alg. 1 "H~ ~ N(mu, diag sigma^2)"                (Step 3)
  rope_cos_sin      Alg. 1 "AverageCosSin(n_f)"                      (Step 3)
  project_rope      Alg. 1 "Q~ = RoPE(H~ W_q, P)"                    (Step 3)
  scores            Eq. (1) logits / Alg. 1 "L = Q~ K^T / sqrt(d_k)"
  top_p_select      Sec. 3.1: the minimal key set whose softmax mass reaches p
  union_vote        Step 4 / Alg. 1 "K = union of C^(s)", B = |K|
  compact           Alg. 1 "prune (K, V) to the indices in K", Sec. 3.4 (mask, nonzero, gather)
  decode_attention  Eq. (1)-(2) of one decode query per head over the compressed, per-head cache (Sec. 3.4)
  attention_overlap Sec. 3.3 "Attention Overlap": real-query attention mass on a synthetic query's set

Pins (tests/test_oracle_pins.py, CPU only): Philox against the generator's
published known-answer vectors; normals by distribution tests against SciPy's
normal law; moments, RoPE, top-p by closed forms; top-p by brute-force subset
enumeration; projection/scores by hand-built one-hot cases; union/compaction by
set arithmetic on hand-written examples; decode attention against SciPy's softmax,
closed forms (equal keys -> mean of V, a dominant key -> its V) and values worked out
by hand (weights 1:3, the group map, the log-sum-exp); overlap by hand-worked values
(weights 1:2:3:4 per head, shared KV head), its bounds and the full-set / complement identities.  `gvote_item` (the composition, i.e.
end-to-end budgets on synthetic inputs) has no printed value in the paper to
compare with: parity unpinned for its budgets beyond the invariants the tests
state (union >= every row set, monotone in p and S, p -> 1 keeps all).
"""
from __future__ import annotations

import math
import numpy as np

__all__ = [
    "philox4x32_10", "philox_u32_stream", "uniform_from_u32", "standard_normals",
    "round_to_dtype", "fit_gaussian", "sample_hidden", "rope_cos_sin", "project_rope",
    "scores", "softmax_weights", "top_p_select", "top_k_select", "select_rows", "union_vote",
    "compact", "pack_mask_words", "unpack_mask_words", "gvote_item", "decode_attention", "attention_overlap",
]

_M32 = np.uint64(0xFFFFFFFF)


# --------------------------------------------------------------------------
# Random integers: Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11).
# --------------------------------------------------------------------------
def philox4x32_10(ctr: np.ndarray, key: np.ndarray) -> np.ndarray:
    """Ten rounds of Philox-4x32.  ctr: uint32[..., 4], key: uint32[..., 2] -> uint32[..., 4].

    One round maps (c0, c1, c2, c3) with round key (k0, k1) to
    (hi(M1*c2) ^ c1 ^ k0, lo(M1*c2), hi(M0*c0) ^ c3 ^ k1, lo(M0*c0));
    between rounds the key advances by the Weyl constants.
    """
    m0, m1 = np.uint64(0xD2511F53), np.uint64(0xCD9E8D57)
    w0, w1 = np.uint64(0x9E3779B9), np.uint64(0xBB67AE85)
    ctr = np.asarray(ctr, dtype=np.uint32)
    key = np.asarray(key, dtype=np.uint32)
    c0, c1, c2, c3 = (ctr[..., i].astype(np.uint64) for i in range(4))
    k0 = np.broadcast_to(key[..., 0].astype(np.uint64), c0.shape).copy()
    k1 = np.broadcast_to(key[..., 1].astype(np.uint64), c0.shape).copy()
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + w0) & _M32
            k1 = (k1 + w1) & _M32
        p0 = m0 * c0
        p1 = m1 * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & _M32
        hi1, lo1 = p1 >> np.uint64(32), p1 & _M32
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def philox_u32_stream(seed: int, stream_id: int, n: int) -> np.ndarray:
    """The first n 32-bit draws of stream (seed, stream_id).

    Draw e lives in block e >> 2, word e & 3.  The block's counter is
    (block_lo32, block_hi32, stream_lo32, stream_hi32); the key is (seed_lo32, seed_hi32).
    """
    nblk = (n + 3) // 4
    blk = np.arange(nblk, dtype=np.uint64)
    ctr = np.empty((nblk, 4), dtype=np.uint32)
    ctr[:, 0] = (blk & _M32).astype(np.uint32)
    ctr[:, 1] = (blk >> np.uint64(32)).astype(np.uint32)
    ctr[:, 2] = np.uint32(stream_id & 0xFFFFFFFF)
    ctr[:, 3] = np.uint32((stream_id >> 32) & 0xFFFFFFFF)
    key = np.array([seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF], dtype=np.uint32)
    return philox4x32_10(ctr, key).reshape(-1)[:n]


def uniform_from_u32(x: np.ndarray) -> np.ndarray:
    """u = ((x >> 9) + 1/2) * 2^-23: the top 23 bits, strictly inside (0, 1), exact in fp32 too."""
    return ((np.asarray(x, dtype=np.uint32) >> np.uint32(9)).astype(np.float64) + 0.5) * 2.0 ** -23


def standard_normals(seed: int, stream_id: int, S: int, d: int) -> np.ndarray:
    """z[S, d] ~ N(0, 1) by Box-Muller on the stream; element (s, j) is draw s*d + j.

    Within a 4-word block the words pair up as (0, 1) and (2, 3).  A pair (u_a, u_b)
    gives r = sqrt(-2 ln u_a), phi = 2 pi u_b; the even word becomes r cos(phi),
    the odd word r sin(phi).  d must be a multiple of 4 (a block never straddles samples).
    """
    if d % 4:
        raise ValueError("d must be a multiple of 4")
    u = uniform_from_u32(philox_u32_stream(seed, stream_id, S * d)).reshape(-1, 2)
    r = np.sqrt(-2.0 * np.log(u[:, 0]))
    phi = 2.0 * np.pi * u[:, 1]
    z = np.stack([r * np.cos(phi), r * np.sin(phi)], axis=-1)
    return z.reshape(S, d)


# --------------------------------------------------------------------------
# Storage rounding (the only non-fp64 points).
# --------------------------------------------------------------------------
def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp64 values to the storage type ('f32' or 'bf16', nearest-even); result held in fp64."""
    x = np.asarray(x, dtype=np.float64)
    if dtype == "f32":
        return x.astype(np.float32).astype(np.float64)
    if dtype == "bf16":
        # bf16 keeps 8 significant bits: x = m * 2^e with m in [0.5, 1); round m * 2^8 to an integer.
        m, e = np.frexp(x)
        return np.ldexp(np.rint(m * 256.0) / 256.0, e)
    raise ValueError(dtype)


# --------------------------------------------------------------------------
# Step 2: Gaussian fit of the prefill hidden states.
# --------------------------------------------------------------------------
def fit_gaussian(hidden: np.ndarray, n_skip: int, ddof: int = 1):
    """Per-channel mean and variance of hidden[L, d] over tokens n_skip..L-1 (Sec. 3.2 Step 2).

    The first n_skip tokens are left out (attention sinks).  Two-pass fp64; outputs are
    rounded to fp32, the type the statistics are stored in.
    """
    h = np.asarray(hidden, dtype=np.float64)[n_skip:]
    n = h.shape[0]
    mu = h.sum(axis=0) / n
    var = ((h - mu) ** 2).sum(axis=0) / (n - ddof)
    return mu.astype(np.float32), var.astype(np.float32)


# --------------------------------------------------------------------------
# Step 3: sample, project, rotate.
# --------------------------------------------------------------------------
def sample_hidden(mu: np.ndarray, var: np.ndarray, z: np.ndarray, dtype: str) -> np.ndarray:
    """H~[s, j] = mu_j + sqrt(var_j) * z[s, j] (Alg. 1, the Gaussian draw), stored in the model dtype."""
    mu = np.asarray(mu, dtype=np.float64)
    sd = np.sqrt(np.asarray(var, dtype=np.float64))
    return round_to_dtype(mu[None, :] + sd[None, :] * z, dtype)


def rope_cos_sin(theta: float, d_k: int, pos0: int, n_future: int = 1):
    """Alg. 1 "AverageCosSin(n_f)": mean of cos and sin over positions pos0 .. pos0+n_future-1.

    Frequencies omega_i = theta^(-2i/d_k), i = 0 .. d_k/2 - 1.
    """
    i = np.arange(d_k // 2, dtype=np.float64)
    omega = float(theta) ** (-2.0 * i / d_k)
    c = np.zeros(d_k // 2)
    s = np.zeros(d_k // 2)
    for tau in range(pos0, pos0 + n_future):
        c += np.cos(tau * omega)
        s += np.sin(tau * omega)
    return c / n_future, s / n_future


def project_rope(h_tilde, w_q, b_q, cos, sin, n_q_heads: int, d_k: int, dtype: str) -> np.ndarray:
    """Q~ = RoPE(H~ W_q^T + b_q) (Alg. 1), W_q[o, j] maps channel j to output o (linear-layer layout).

    Per head the pair (i, i + d_k/2) is rotated: q'_i = q_i c_i - q_{i+d_k/2} s_i,
    q'_{i+d_k/2} = q_{i+d_k/2} c_i + q_i s_i.  Returns Q~[S, H_q, d_k] rounded to the model dtype.
    """
    h = np.asarray(h_tilde, dtype=np.float64)
    w = np.asarray(w_q, dtype=np.float64)
    q = h @ w.T
    if b_q is not None:
        q = q + np.asarray(b_q, dtype=np.float64)[None, :]
    q = q.reshape(h.shape[0], n_q_heads, d_k)
    half = d_k // 2
    q1, q2 = q[..., :half], q[..., half:]
    out = np.concatenate([q1 * cos - q2 * sin, q2 * cos + q1 * sin], axis=-1)
    return round_to_dtype(out, dtype)


# --------------------------------------------------------------------------
# Eq. (1): logits of every synthetic query against every cached key.
# --------------------------------------------------------------------------
def scores(q_tilde: np.ndarray, k: np.ndarray) -> np.ndarray:
    """logits[s, h, t] = <Q~[s, h, :], K[t, h div G, :]> / sqrt(d_k); K is [L, H_kv, d_k]; no mask."""
    q = np.asarray(q_tilde, dtype=np.float64)
    kk = np.asarray(k, dtype=np.float64)
    S, hq, dk = q.shape
    L, hkv, _ = kk.shape
    G = hq // hkv
    out = np.empty((S, hq, L))
    for h in range(hq):
        out[:, h, :] = q[:, h, :] @ kk[:, h // G, :].T / math.sqrt(dk)
    return out


def softmax_weights(logits_row: np.ndarray):
    """m = max, w_t = exp(l_t - m), Z = sum w (the softmax of Eq. (1), left un-normalised)."""
    l = np.asarray(logits_row, dtype=np.float64)
    m = l.max()
    w = np.exp(l - m)
    return m, w, w.sum()


# --------------------------------------------------------------------------
# Sec. 3.1: required keys of one query = the minimal set with softmax mass >= p.
# --------------------------------------------------------------------------
def top_p_select(logits_row: np.ndarray, p: float) -> np.ndarray:
    """Boolean mask of the smallest key set whose attention mass reaches p.

    Keys are taken in the order (logit descending, index ascending); the set is the
    shortest prefix whose cumulative un-normalised weight is >= p * Z.  p >= 1 keeps all.
    """
    l = np.asarray(logits_row, dtype=np.float64)
    L = l.shape[0]
    if p >= 1.0:
        return np.ones(L, dtype=bool)
    _, w, Z = softmax_weights(l)
    order = np.argsort(-l, kind="stable")          # ties keep ascending index
    cum = np.cumsum(w[order])
    reached = np.nonzero(cum >= p * Z)[0]
    k_star = (reached[0] + 1) if reached.size else L
    mask = np.zeros(L, dtype=bool)
    mask[order[:k_star]] = True
    return mask


def top_k_select(logits_row: np.ndarray, k: int) -> np.ndarray:
    """Alg. 1's row-wise TopK on logits: the k largest, ties to the lower index."""
    l = np.asarray(logits_row, dtype=np.float64)
    order = np.argsort(-l, kind="stable")
    mask = np.zeros(l.shape[0], dtype=bool)
    mask[order[:max(0, min(int(k), l.shape[0]))]] = True
    return mask


def select_rows(logits: np.ndarray, p: float) -> np.ndarray:
    """top_p_select on every (s, h) row of logits[S, H_q, L]."""
    S, hq, L = logits.shape
    out = np.empty((S, hq, L), dtype=bool)
    for s in range(S):
        for h in range(hq):
            out[s, h] = top_p_select(logits[s, h], p)
    return out


# --------------------------------------------------------------------------
# Step 4: vote, count, prune.
# --------------------------------------------------------------------------
def union_vote(rowmask: np.ndarray, n_kv_heads: int):
    """Keep-set per KV head = union over samples and over the query heads of the group; B = its size."""
    S, hq, L = rowmask.shape
    G = hq // n_kv_heads
    union = np.zeros((n_kv_heads, L), dtype=bool)
    for s in range(S):
        for h in range(hq):
            union[h // G] |= rowmask[s, h]
    budget = union.sum(axis=1).astype(np.int32)
    return union, budget


def compact(k: np.ndarray, v: np.ndarray, union: np.ndarray):
    """Gather kept rows of K, V[L, H_kv, d_k] per KV head in ascending position (mask -> nonzero -> index).

    Returns (K_out[sum B, d_k], V_out, idx[sum B], offsets[H_kv + 1]); head h owns rows
    offsets[h] .. offsets[h+1]-1.
    """
    hkv = union.shape[0]
    ks, vs, ids, offs = [], [], [], [0]
    for h in range(hkv):
        idx = np.nonzero(union[h])[0]
        ks.append(k[idx, h, :])
        vs.append(v[idx, h, :])
        ids.append(idx.astype(np.int32))
        offs.append(offs[-1] + idx.size)
    return (np.concatenate(ks, axis=0), np.concatenate(vs, axis=0),
            np.concatenate(ids), np.asarray(offs, dtype=np.int64))


def pack_mask_words(mask: np.ndarray) -> np.ndarray:
    """bool[..., L] -> uint32[..., ceil(L/32)]; key t is bit t % 32 of word t // 32; unused bits 0."""
    L = mask.shape[-1]
    nw = (L + 31) // 32
    padded = np.zeros(mask.shape[:-1] + (nw * 32,), dtype=np.uint64)
    padded[..., :L] = mask
    bits = padded.reshape(mask.shape[:-1] + (nw, 32)) << np.arange(32, dtype=np.uint64)
    return bits.sum(axis=-1).astype(np.uint32)


def unpack_mask_words(words: np.ndarray, L: int) -> np.ndarray:
    """Inverse of pack_mask_words."""
    w = np.asarray(words, dtype=np.uint32)
    bits = (w[..., :, None] >> np.arange(32, dtype=np.uint32)) & np.uint32(1)
    return bits.reshape(w.shape[:-1] + (-1,))[..., :L].astype(bool)


# --------------------------------------------------------------------------
# Consumer side: attention over the compressed cache, and the overlap diagnostic.
# --------------------------------------------------------------------------
def decode_attention(q, k_out, v_out, offsets, n_kv_heads: int):
    """Eq. (1)-(2) on the non-uniform cache of Sec. 3.4: for query head h (KV head h div G) the output is
    softmax(q[h] K_h^T / sqrt(d_k)) V_h over the rows offsets[h div G] .. offsets[h div G + 1] - 1 of the
    packed cache.  q[H_q, d_k]; returns (out[H_q, d_k], lse[H_q]) in fp64, lse = log sum exp of the logits."""
    q = np.asarray(q, dtype=np.float64)
    hq, dk = q.shape
    G = hq // n_kv_heads
    out = np.zeros((hq, dk))
    lse = np.zeros(hq)
    for h in range(hq):
        lo, hi = int(offsets[h // G]), int(offsets[h // G + 1])
        kk = np.asarray(k_out[lo:hi], dtype=np.float64)
        vv = np.asarray(v_out[lo:hi], dtype=np.float64)
        l = kk @ q[h] / math.sqrt(dk)
        m = l.max()
        w = np.exp(l - m)
        out[h] = (w / w.sum()) @ vv
        lse[h] = m + math.log(w.sum())
    return out, lse


def attention_overlap(q_real, k, rowmask):
    """Sec. 3.3: overlap[s, h] = sum over the keys of synthetic row (s, h)'s set of the attention weights
    of the real query head h (softmax over all L keys).  q_real[H_q, d_k], k[L, H_kv, d_k], rowmask[S, H_q, L]."""
    lg = scores(np.asarray(q_real, dtype=np.float64)[None], k)[0]          # [H_q, L]
    S, hq, L = rowmask.shape
    out = np.zeros((S, hq))
    for h in range(hq):
        _, w, Z = softmax_weights(lg[h])
        a = w / Z
        for s in range(S):
            out[s, h] = a[rowmask[s, h]].sum()
    return out


# --------------------------------------------------------------------------
# The whole path for one item (request x layer), Alg. 1 with per-row top-p.
# --------------------------------------------------------------------------
def gvote_item(hidden, w_q, b_q, k, v, *, n_q_heads, n_kv_heads, d_k, theta, S, p, seed, stream_id,
               dtype, n_skip=4, ddof=1, pos0=None, n_future=1):
    """Run Steps 2-4 for one item and return every intermediate in a dict."""
    L, d = hidden.shape
    if pos0 is None:
        pos0 = L
    mu, var = fit_gaussian(hidden, n_skip, ddof)
    z = standard_normals(seed, stream_id, S, d)
    h_tilde = sample_hidden(mu, var, z, dtype)
    c, s = rope_cos_sin(theta, d_k, pos0, n_future)
    q_tilde = project_rope(h_tilde, w_q, b_q, c, s, n_q_heads, d_k, dtype)
    logits = scores(q_tilde, k)
    rowmask = select_rows(logits, p)
    union, budget = union_vote(rowmask, n_kv_heads)
    k_out, v_out, idx, offsets = compact(np.asarray(k), np.asarray(v), union)
    return dict(mu=mu, var=var, z=z, h_tilde=h_tilde, q_tilde=q_tilde, logits=logits, rowmask=rowmask,
                union=union, budget=budget, k_out=k_out, v_out=v_out, idx=idx, offsets=offsets)
