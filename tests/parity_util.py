"""Shared pieces of the parity tests: run the CPU oracle on generated items, compare with the HIP
path.  Tolerances (relative to the paper's fp64 definition, both sides on the same stored inputs):
bf16 storage: 2e-3; fp32 storage: 1e-5 -- on scores / softmax mass; masks may differ only for keys
whose cumulative-mass position lies within that tolerance of the p boundary (sandwich test)."""
from __future__ import annotations

import numpy as np
import torch

import oracle as O

TOL = {"f32": 1e-5, "bf16": 2e-3}
# a single stage fed with the oracle's own (stored) inputs: only the accumulation arithmetic differs
# (fp64 accumulate for fp32 storage, fp32 accumulate of exact bf16 products for bf16 storage)
STAGE_TOL = {"f32": 1e-5, "bf16": 1e-4}


def f32np(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float32).numpy()


def p32(p: float) -> float:
    """The ABI carries p as a C float; the oracle must see that very value."""
    return float(np.float32(p))


def oracle_item(wl, it, *, S=None, p=None, n_skip=None, pos0=None, n_future=1, b_q=None, upto="all"):
    S = wl.S if S is None else S
    p = p32(wl.p if p is None else p)
    hidden, w_q, k, v = f32np(it["hidden"]), f32np(it["w_q"]), f32np(it["k"]), f32np(it["v"])
    L = hidden.shape[0]
    n_skip = wl.n_skip if n_skip is None else n_skip
    pos0 = L if pos0 is None else pos0
    out = {}
    out["mu"], out["var"] = O.fit_gaussian(hidden, n_skip, wl.ddof)
    out["z"] = O.standard_normals(it["seed"], it["stream_id"], S, wl.d)
    out["h_tilde"] = O.sample_hidden(out["mu"], out["var"], out["z"], wl.dtype)
    c, s = O.rope_cos_sin(float(np.float32(wl.theta)), wl.d_k, pos0, n_future)
    out["q_tilde"] = O.project_rope(out["h_tilde"], w_q, None if b_q is None else f32np(b_q), c, s,
                                    wl.n_q_heads, wl.d_k, wl.dtype)
    if upto == "q":
        return out
    out["logits"] = O.scores(out["q_tilde"], k)
    out["rowmask"] = O.select_rows(out["logits"], p)
    out["union"], out["budget"] = O.union_vote(out["rowmask"], wl.n_kv_heads)
    out["k_out"], out["v_out"], out["idx"], out["offsets"] = O.compact(k, v, out["union"])
    return out


def band_sets(logits_row: np.ndarray, p: float, tol: float):
    """Keys a correct selection MUST hold and MAY hold, given that cumulative masses are only trusted to
    `tol`.  In the oracle's order (logit descending, position ascending) key i occupies the cumulative-
    mass interval (c_{i-1}, c_i] / Z.  Keys whose interval ends at or before p - tol must be selected;
    keys whose interval starts at or after p + tol must not be; a key whose interval reaches into
    [p - tol, p + tol] lies within the tolerance of the boundary and may go either way (two nearly tied
    heavy keys may swap places when the logits carry bf16-level differences)."""
    l = np.asarray(logits_row, dtype=np.float64)
    _, w, Z = O.softmax_weights(l)
    order = np.argsort(-l, kind="stable")
    cum = np.cumsum(w[order])
    must = np.zeros(l.shape[0], dtype=bool)
    may = np.zeros(l.shape[0], dtype=bool)
    must[order[cum <= (p - tol) * Z]] = True
    may[order[(cum - w[order]) < (p + tol) * Z]] = True
    if p >= 1.0:
        must[:] = True
        may[:] = True
    return must, may


def check_rowmask_sandwich(gpu_mask: np.ndarray, logits: np.ndarray, p: float, tol: float):
    """gpu_mask bool [S, H_q, L]: must <= gpu <= may for every row.  Returns the number of boundary keys
    (gpu xor the oracle's own selection at p)."""
    S, hq, _ = logits.shape
    boundary = 0
    for s in range(S):
        for h in range(hq):
            must, may = band_sets(logits[s, h], p, tol)
            got = gpu_mask[s, h]
            missing, extra = must & ~got, got & ~may
            assert not missing.any(), f"row ({s},{h}): {missing.sum()} keys entirely before the p - tol band are not selected"
            assert not extra.any(), f"row ({s},{h}): {extra.sum()} selected keys lie entirely beyond the p + tol band"
            assert got.any()
            boundary += int((got ^ O.top_p_select(logits[s, h], p)).sum())
    return boundary


def unpack_rows(words: torch.Tensor, rows: int, L: int) -> np.ndarray:
    w = words.detach().to("cpu").numpy().view(np.uint32).reshape(rows, (L + 31) // 32)
    return O.unpack_mask_words(w, L)


def batch_from(g, wl, items, **kw):
    return g.Batch(items, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=wl.d_k,
                   rope_theta=wl.theta, n_skip=wl.n_skip, **kw)


def to_device(items, dev):
    out = []
    for it in items:
        out.append({k: (v.to(dev) if isinstance(v, torch.Tensor) else v) for k, v in it.items()})
    return out
