"""ctypes binding of the GVote C ABI (include/gvote.h).  Argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import torch

F32, BF16 = 0, 1
SELECT_TOPP, SELECT_TOPK = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))


def lib_path() -> str:
    """The in-tree library; GVOTE_LIB names another build of the same sources (kernel experiments)."""
    return os.environ.get("GVOTE_LIB") or os.path.join(_HERE, "libgvote.so")


class GVoteError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: gvote status {code} ({status_string(code)})")


class Shape(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("dtype", C.c_int32), ("rope_theta", C.c_float)]


class Item(C.Structure):
    _fields_ = [("hidden", C.c_void_p), ("hidden_row_stride", C.c_int64), ("w_q", C.c_void_p),
                ("b_q", C.c_void_p), ("k", C.c_void_p), ("v", C.c_void_p), ("kv_tok_stride", C.c_int64),
                ("kv_head_stride", C.c_int64), ("L", C.c_int32), ("n_skip", C.c_int32), ("pos0", C.c_int32),
                ("n_future", C.c_int32), ("seed", C.c_uint64), ("stream_id", C.c_uint64)]


_lib = None


def lib() -> C.CDLL:
    """Load libgvote.so.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or python paper_2509_03136_amd/build.py).  There is no CPU fallback.")
    L = C.CDLL(path)
    vp, i32, i64, u64, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float, C.c_size_t
    sp, ip = C.POINTER(Shape), C.POINTER(Item)
    L.gvote_status_string.restype = C.c_char_p
    L.gvote_status_string.argtypes = [C.c_int]
    L.gvote_abi_version.restype = i32
    L.gvote_abi_version.argtypes = []
    L.gvote_workspace_bytes.restype = sz
    L.gvote_workspace_bytes.argtypes = [sp, ip, i32, i32]
    L.gvote_fit_gaussian.restype = C.c_int
    L.gvote_fit_gaussian.argtypes = [sp, ip, i32, i32, vp, vp, vp, sz, vp]
    L.gvote_sample_queries.restype = C.c_int
    L.gvote_sample_queries.argtypes = [sp, ip, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    L.gvote_score_select.restype = C.c_int
    L.gvote_score_select.argtypes = [sp, ip, i32, i32, vp, f32, i32, vp, vp, vp, vp, vp, sz, vp]
    L.gvote_union_compact.restype = C.c_int
    L.gvote_union_compact.argtypes = [sp, ip, i32, i32, vp, vp, vp, vp, vp, vp, vp, i64, vp, vp, sz, vp]
    L.gvote_union_compact_static.restype = C.c_int
    L.gvote_union_compact_static.argtypes = [sp, ip, i32, i32, vp, vp, vp, vp, vp, vp, vp, i64, vp, vp]
    L.gvote_count_rows.restype = C.c_int
    L.gvote_count_rows.argtypes = [sp, ip, i32, i32, vp, i32, vp, vp]
    L.gvote_decode_attention.restype = C.c_int
    L.gvote_decode_attention.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.gvote_decode_workspace_bytes.restype = sz
    L.gvote_decode_workspace_bytes.argtypes = [sp, i32]
    L.gvote_attention_overlap.restype = C.c_int
    L.gvote_attention_overlap.argtypes = [sp, ip, i32, i32, vp, vp, vp, vp, sz, vp]
    L.gvote_debug_set_spin_limit.restype = i32
    L.gvote_debug_set_spin_limit.argtypes = [i32]
    L.gvote_philox_u32.restype = C.c_int
    L.gvote_philox_u32.argtypes = [u64, u64, i64, vp, vp]
    _lib = L
    return L


def abi_version() -> int:
    return int(lib().gvote_abi_version())


def status_string(code: int) -> str:
    return lib().gvote_status_string(int(code)).decode()


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _check(code: int, where: str) -> None:
    if code != 0:
        raise GVoteError(code, where)


class Batch:
    """Host-side descriptors (gvote_shape + gvote_item[]) of a batch of (request, layer) items.

    `items` is a list of dicts with torch tensors `hidden` [L, d], `w_q` [H_q*d_k, d], `k`, `v`
    [L, H_kv, d_k] (any strides whose innermost dimension is contiguous), optional `b_q`, and the
    integers L, seed, stream_id, optional n_skip, pos0, n_future.  The tensors are kept alive here.
    """

    def __init__(self, items: Sequence[Dict], *, n_q_heads: int, n_kv_heads: int, head_dim: int,
                 rope_theta: float, n_skip: int = 4):
        first = items[0]
        dt = first["hidden"].dtype
        self.dtype = F32 if dt == torch.float32 else BF16
        self.torch_dtype = dt
        self.d_model = int(first["hidden"].shape[1])
        self.shape = Shape(self.d_model, n_q_heads, n_kv_heads, head_dim, self.dtype, float(rope_theta))
        self.n_items = len(items)
        self.items_py = list(items)
        self.items = (Item * self.n_items)()
        self.lengths: List[int] = []
        for i, it in enumerate(items):
            h, k, v = it["hidden"], it["k"], it["v"]
            L = int(it.get("L", h.shape[0]))
            c = self.items[i]
            c.hidden, c.hidden_row_stride = h.data_ptr(), h.stride(0)
            c.w_q = it["w_q"].data_ptr()
            c.b_q = _ptr(it.get("b_q"))
            c.k, c.v = k.data_ptr(), v.data_ptr()
            c.kv_tok_stride, c.kv_head_stride = k.stride(0), k.stride(1)
            assert v.stride(0) == k.stride(0) and v.stride(1) == k.stride(1), "k and v must share strides"
            c.L, c.n_skip = L, int(it.get("n_skip", n_skip))
            c.pos0, c.n_future = int(it.get("pos0", L)), int(it.get("n_future", 1))
            c.seed, c.stream_id = int(it["seed"]), int(it["stream_id"])
            self.lengths.append(L)
        self.n_q_heads, self.n_kv_heads, self.head_dim = n_q_heads, n_kv_heads, head_dim
        self.device = first["hidden"].device

    @classmethod
    def from_workload(cls, wl, items: Sequence[Dict], **kw) -> "Batch":
        """Descriptors for the items of a synthetic workload (synth.workloads.Workload: geometry fields only)."""
        return cls(items, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=wl.d_k,
                   rope_theta=wl.theta, n_skip=wl.n_skip, **kw)

    def words(self, i: int) -> int:
        return (self.lengths[i] + 31) // 32


def workspace_bytes(b: Batch, S: int) -> int:
    return int(lib().gvote_workspace_bytes(C.byref(b.shape), b.items, b.n_items, S))


def fit_gaussian(b: Batch, ddof: int, mu: torch.Tensor, var: torch.Tensor, ws: torch.Tensor, stream=None) -> None:
    _check(lib().gvote_fit_gaussian(C.byref(b.shape), b.items, b.n_items, ddof, _ptr(mu), _ptr(var), _ptr(ws),
                                    ws.numel() * ws.element_size(), _stream(stream)), "gvote_fit_gaussian")


def sample_queries(b: Batch, S: int, mu: torch.Tensor, var: torch.Tensor, q_out: torch.Tensor,
                   h_tilde_out: Optional[torch.Tensor], ws: torch.Tensor, stream=None) -> None:
    _check(lib().gvote_sample_queries(C.byref(b.shape), b.items, b.n_items, S, _ptr(mu), _ptr(var), _ptr(q_out),
                                      _ptr(h_tilde_out), _ptr(ws), ws.numel() * ws.element_size(),
                                      _stream(stream)), "gvote_sample_queries")


def score_select(b: Batch, S: int, q: torch.Tensor, p: float, rowmask: torch.Tensor, *, mode: int = SELECT_TOPP,
                 k_per_row: Optional[torch.Tensor] = None, row_max: Optional[torch.Tensor] = None,
                 row_sum: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None, stream=None) -> None:
    _check(lib().gvote_score_select(C.byref(b.shape), b.items, b.n_items, S, _ptr(q), float(p), mode,
                                    _ptr(k_per_row), _ptr(rowmask), _ptr(row_max), _ptr(row_sum), _ptr(ws),
                                    0 if ws is None else ws.numel() * ws.element_size(), _stream(stream)),
           "gvote_score_select")


def union_compact(b: Batch, S: int, rowmask: torch.Tensor, union_mask: torch.Tensor, budget: torch.Tensor,
                  offsets: torch.Tensor, k_out: torch.Tensor, v_out: torch.Tensor, idx_out: Optional[torch.Tensor],
                  capacity_tokens: int, overflow_flag: torch.Tensor, ws: torch.Tensor, stream=None) -> None:
    _check(lib().gvote_union_compact(C.byref(b.shape), b.items, b.n_items, S, _ptr(rowmask), _ptr(union_mask),
                                     _ptr(budget), _ptr(offsets), _ptr(k_out), _ptr(v_out), _ptr(idx_out),
                                     int(capacity_tokens), _ptr(overflow_flag), _ptr(ws),
                                     ws.numel() * ws.element_size(), _stream(stream)), "gvote_union_compact")


def union_compact_static(b: Batch, S: int, rowmask: torch.Tensor, union_mask: torch.Tensor, budget: torch.Tensor,
                         offsets: torch.Tensor, k_out: torch.Tensor, v_out: torch.Tensor,
                         idx_out: Optional[torch.Tensor], capacity_tokens: int, overflow_flag: torch.Tensor,
                         stream=None) -> None:
    _check(lib().gvote_union_compact_static(C.byref(b.shape), b.items, b.n_items, S, _ptr(rowmask), _ptr(union_mask),
                                            _ptr(budget), _ptr(offsets), _ptr(k_out), _ptr(v_out), _ptr(idx_out),
                                            int(capacity_tokens), _ptr(overflow_flag), _stream(stream)),
           "gvote_union_compact_static")


def count_rows(b: Batch, S: int, rowmask: torch.Tensor, repeat: int, counts: torch.Tensor, stream=None) -> None:
    _check(lib().gvote_count_rows(C.byref(b.shape), b.items, b.n_items, S, _ptr(rowmask), int(repeat), _ptr(counts),
                                  _stream(stream)), "gvote_count_rows")


def decode_workspace_bytes(b: Batch) -> int:
    return int(lib().gvote_decode_workspace_bytes(C.byref(b.shape), b.n_items))


def decode_attention(b: Batch, q: torch.Tensor, k_out: torch.Tensor, v_out: torch.Tensor, offsets: torch.Tensor,
                     out: torch.Tensor, ws: torch.Tensor, lse: Optional[torch.Tensor] = None, stream=None) -> None:
    _check(lib().gvote_decode_attention(C.byref(b.shape), b.n_items, _ptr(q), _ptr(k_out), _ptr(v_out), _ptr(offsets),
                                        _ptr(out), _ptr(lse), _ptr(ws), ws.numel() * ws.element_size(),
                                        _stream(stream)), "gvote_decode_attention")


def attention_overlap(b: Batch, S: int, q_real: torch.Tensor, rowmask: torch.Tensor, overlap: torch.Tensor,
                      ws: torch.Tensor, stream=None) -> None:
    _check(lib().gvote_attention_overlap(C.byref(b.shape), b.items, b.n_items, S, _ptr(q_real), _ptr(rowmask),
                                         _ptr(overlap), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)),
           "gvote_attention_overlap")


def debug_set_spin_limit(polls: int) -> int:
    return int(lib().gvote_debug_set_spin_limit(int(polls)))


def philox_u32(seed: int, stream_id: int, n: int, out: torch.Tensor, stream=None) -> None:
    _check(lib().gvote_philox_u32(int(seed), int(stream_id), int(n), _ptr(out), _stream(stream)), "gvote_philox_u32")


class Pipeline:
    """Output and workspace buffers of one batch, allocated once with torch, plus `run()` = the four
    ABI calls back to back on the current stream (no host synchronisation in between)."""

    def __init__(self, b: Batch, S: int, p: float, *, ddof: int = 1, capacity_tokens: Optional[int] = None,
                 want_h_tilde: bool = False, want_stats: bool = True):
        dev, n = b.device, b.n_items
        self.b, self.S, self.p, self.ddof = b, S, float(p), ddof
        R = S * b.n_q_heads
        self.rows = R
        self.mask_words = [R * b.words(i) for i in range(n)]
        self.union_words = [b.n_kv_heads * b.words(i) for i in range(n)]
        self.mu = torch.empty(n, b.d_model, device=dev, dtype=torch.float32)
        self.var = torch.empty_like(self.mu)
        self.q = torch.empty(n, S, b.n_q_heads, b.head_dim, device=dev, dtype=b.torch_dtype)
        self.h_tilde = torch.empty(n, S, b.d_model, device=dev, dtype=b.torch_dtype) if want_h_tilde else None
        self.rowmask = torch.empty(sum(self.mask_words), device=dev, dtype=torch.int32)
        self.row_max = torch.empty(n, R, device=dev, dtype=torch.float32) if want_stats else None
        self.row_sum = torch.empty(n, R, device=dev, dtype=torch.float32) if want_stats else None
        self.union_mask = torch.empty(sum(self.union_words), device=dev, dtype=torch.int32)
        self.budget = torch.empty(n, b.n_kv_heads, device=dev, dtype=torch.int32)
        self.offsets = torch.empty(n * b.n_kv_heads + 1, device=dev, dtype=torch.int64)
        self.capacity = int(capacity_tokens) if capacity_tokens is not None else sum(b.lengths) * b.n_kv_heads
        self.k_out = torch.empty(max(1, self.capacity), b.head_dim, device=dev, dtype=b.torch_dtype)
        self.v_out = torch.empty_like(self.k_out)
        self.idx_out = torch.empty(max(1, self.capacity), device=dev, dtype=torch.int32)
        self.overflow = torch.zeros(1, device=dev, dtype=torch.int32)
        nbytes = workspace_bytes(b, S)
        if nbytes == 0:
            raise GVoteError(1, "gvote_workspace_bytes")
        self.ws = torch.empty(nbytes, device=dev, dtype=torch.uint8)

    def fit(self):
        fit_gaussian(self.b, self.ddof, self.mu, self.var, self.ws)

    def sample(self):
        sample_queries(self.b, self.S, self.mu, self.var, self.q, self.h_tilde, self.ws)

    def select(self):
        score_select(self.b, self.S, self.q, self.p, self.rowmask, row_max=self.row_max, row_sum=self.row_sum,
                     ws=self.ws)

    def fallback_rows(self) -> int:
        """Rows of the last select() redone by the exact general selector (matrix-core path only)."""
        return int(self.ws[:4].view(torch.int32).item())

    def fallback_reasons(self):
        """(cut below the histogram window, candidate lists full, too many candidates, first pass gave up) row counts."""
        return [int(x) for x in self.ws[8:24].view(torch.int32).tolist()]

    def refined_rows(self) -> int:
        """Rows of the last select() whose cut lay below their first histogram window and was found in a deeper one."""
        return int(self.ws[24:28].view(torch.int32).item())

    def compact(self):
        union_compact(self.b, self.S, self.rowmask, self.union_mask, self.budget, self.offsets, self.k_out,
                      self.v_out, self.idx_out, self.capacity, self.overflow, self.ws)

    def run(self):
        self.fit()
        self.sample()
        self.select()
        self.compact()
