"""GPU parity of the consumer side: attention over the compressed per-head cache (Sec. 3.4, Eq. (1)-(2))
and the attention-overlap diagnostic (Sec. 3.3), against the CPU oracle on the same stored data."""
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


def _real_queries(wl, items):
    """The last token's query of every item (hidden state through W_q, rotated at L - 1), stored in dtype."""
    qs = []
    for it in items:
        L = it["L"]
        c, s = O.rope_cos_sin(float(np.float32(wl.theta)), wl.d_k, L - 1, 1)
        qs.append(O.project_rope(U.f32np(it["hidden"][L - 1:L]), U.f32np(it["w_q"]), None, c, s, wl.n_q_heads, wl.d_k,
                                 wl.dtype)[0])
    return np.stack(qs)          # [n, H_q, d_k]


@pytest.mark.parametrize("cfg", [1, 2, 5])
def test_decode_attention_over_compressed_cache(g, cfg):
    wl = {1: W.config(1), 2: W.config(2),
          5: W.scaled(W.config(5), lengths=(1100, 333, 2049, 64), n_planted=(8, 3, 200, 1))}[cfg]
    items = W.make_items(wl, "cpu")
    b = U.batch_from(g, wl, U.to_device(items, DEV))
    pipe = g.Pipeline(b, wl.S, wl.p, ddof=wl.ddof)
    pipe.run()
    q = _real_queries(wl, items)
    q_dev = torch.tensor(q).to(pipe.q.dtype).to(DEV)
    out = torch.empty_like(q_dev)
    lse = torch.empty(len(items), wl.n_q_heads, device=DEV, dtype=torch.float32)
    g.decode_attention(b, q_dev, pipe.k_out, pipe.v_out, pipe.offsets, out, pipe.ws, lse)
    torch.cuda.synchronize()
    offs = pipe.offsets.cpu().numpy()
    k_out, v_out = U.f32np(pipe.k_out), U.f32np(pipe.v_out)
    tol = U.TOL[wl.dtype]
    for i in range(len(items)):
        o = offs[i * wl.n_kv_heads:(i + 1) * wl.n_kv_heads + 1]
        want, want_lse = O.decode_attention(q[i], k_out, v_out, o, wl.n_kv_heads)
        got = U.f32np(out[i]).astype(np.float64)
        scale = np.sqrt((want ** 2).mean())
        step = 2.0 ** -7 if wl.dtype == "bf16" else 0.0            # one storage rounding of the output
        assert np.all(np.abs(got - want) <= step * np.abs(want) + tol * scale + 1e-6), np.abs(got - want).max()
        assert np.all(np.abs(lse[i].cpu().numpy() - want_lse) <= tol * (1 + np.abs(want_lse)))


def test_attention_overlap_of_synthetic_sets(g):
    wl = W.scaled(W.config(5), lengths=(1100, 333, 2049), n_planted=(8, 3, 200), S=4)
    items = W.make_items(wl, "cpu")
    b = U.batch_from(g, wl, U.to_device(items, DEV))
    pipe = g.Pipeline(b, wl.S, wl.p, ddof=wl.ddof)
    pipe.fit(); pipe.sample(); pipe.select()
    q = _real_queries(wl, items)
    q_dev = torch.tensor(q).to(pipe.q.dtype).to(DEV)
    ov = torch.empty(len(items), wl.S, wl.n_q_heads, device=DEV, dtype=torch.float32)
    g.attention_overlap(b, wl.S, q_dev, pipe.rowmask, ov, pipe.ws)
    torch.cuda.synchronize()
    off = 0
    for i, it in enumerate(items):
        L = it["L"]
        gm = U.unpack_rows(pipe.rowmask[off:off + pipe.mask_words[i]], pipe.rows, L).reshape(wl.S, wl.n_q_heads, L)
        off += pipe.mask_words[i]
        want = O.attention_overlap(q[i], U.f32np(it["k"]), gm)          # on the GPU's own sets
        got = ov[i].cpu().numpy()
        assert np.all(np.abs(got - want) <= 1e-4 + 1e-4 * want), np.abs(got - want).max()
        assert np.all(got >= 0) and np.all(got <= 1 + 1e-5)
