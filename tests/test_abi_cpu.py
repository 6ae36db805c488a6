"""CPU-only checks of the boundary: the shared library loads, exports every symbol the header
declares, and rejects bad arguments on the host before any launch (no GPU needed, no compute)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def g():
    import paper_2509_03136_amd as g
    if not os.path.exists(g.lib_path()):
        import __graft_entry__
        __graft_entry__.build()
    return g


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "gvote.h")).read()
    return sorted(set(re.findall(r"GVOTE_API[^;(]*?\b(gvote_\w+)\s*\(", text)))


def test_header_symbols_are_exported(g):
    names = declared_symbols()
    assert {"gvote_fit_gaussian", "gvote_sample_queries", "gvote_score_select", "gvote_union_compact",
            "gvote_workspace_bytes", "gvote_status_string", "gvote_abi_version", "gvote_philox_u32",
            "gvote_count_rows", "gvote_decode_attention", "gvote_decode_workspace_bytes", "gvote_attention_overlap",
            "gvote_union_compact_static", "gvote_debug_set_spin_limit"} <= set(names)
    lib = C.CDLL(g.lib_path())
    for n in names:
        assert hasattr(lib, n), n
    assert g.abi_version() == 1001
    for code in range(7):
        assert g.status_string(code)


def test_struct_layout_matches_header(g):
    assert C.sizeof(g.Shape) == 24
    assert C.sizeof(g.Item) == 96
    assert g.Item.L.offset == 64 and g.Item.seed.offset == 80


def _shape(g, **kw):
    base = dict(d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, dtype=g.F32, rope_theta=1e4)
    base.update(kw)
    return g.Shape(**base)


def _items(g, n=1, **kw):
    arr = (g.Item * n)()
    for i in range(n):
        it = arr[i]
        it.hidden, it.hidden_row_stride = 0x1000, 256
        it.w_q, it.b_q, it.k, it.v = 0x2000, None, 0x3000, 0x4000
        it.kv_tok_stride, it.kv_head_stride = 128, 64
        it.L, it.n_skip, it.pos0, it.n_future = 512, 4, 512, 1
        it.seed, it.stream_id = 1, i
        for k, v in kw.items():
            setattr(it, k, v)
    return arr


def test_workspace_size_is_host_logic(g):
    L = g.lib()
    sh, it = _shape(g), _items(g, 3)
    n = L.gvote_workspace_bytes(C.byref(sh), it, 3, 8)
    assert n > 0 and n % 256 == 0
    assert L.gvote_workspace_bytes(C.byref(sh), it, 0, 8) == 0
    assert L.gvote_workspace_bytes(C.byref(sh), it, 3, 0) == 0
    assert L.gvote_workspace_bytes(C.byref(_shape(g, n_q_heads=3)), it, 3, 8) == 0
    assert L.gvote_workspace_bytes(None, it, 3, 8) == 0
    big = _items(g, 3, L=1 << 20)
    assert L.gvote_workspace_bytes(C.byref(sh), big, 3, 8) > n


def test_bad_arguments_are_rejected_before_any_launch(g):
    L = g.lib()
    sh, it = _shape(g), _items(g)
    ws, wsn = 0x10000, 1 << 30
    INVALID, SHAPE, UNSUP, WS, CAP = 1, 2, 3, 4, 5
    fit = L.gvote_fit_gaussian
    assert fit(None, it, 1, 1, 0x100, 0x200, ws, wsn, None) == INVALID
    assert fit(C.byref(sh), None, 1, 1, 0x100, 0x200, ws, wsn, None) == INVALID
    assert fit(C.byref(sh), it, 0, 1, 0x100, 0x200, ws, wsn, None) == INVALID
    assert fit(C.byref(sh), it, 1, 2, 0x100, 0x200, ws, wsn, None) == INVALID
    assert fit(C.byref(sh), it, 1, 1, None, 0x200, ws, wsn, None) == INVALID
    assert fit(C.byref(sh), it, 1, 1, 0x100, 0x200, ws, 16, None) == WS
    assert fit(C.byref(sh), _items(g, L=1), 1, 1, 0x100, 0x200, ws, wsn, None) == INVALID
    assert fit(C.byref(sh), _items(g, n_skip=511), 1, 1, 0x100, 0x200, ws, wsn, None) == INVALID
    assert fit(C.byref(sh), _items(g, hidden=0x1004), 1, 1, 0x100, 0x200, ws, wsn, None) == SHAPE
    assert fit(C.byref(sh), _items(g, hidden_row_stride=250), 1, 1, 0x100, 0x200, ws, wsn, None) == SHAPE
    assert fit(C.byref(_shape(g, dtype=7)), it, 1, 1, 0x100, 0x200, ws, wsn, None) == UNSUP
    assert fit(C.byref(_shape(g, n_q_heads=3)), it, 1, 1, 0x100, 0x200, ws, wsn, None) == SHAPE
    assert fit(C.byref(_shape(g, head_dim=512)), it, 1, 1, 0x100, 0x200, ws, wsn, None) == UNSUP
    smp = L.gvote_sample_queries
    assert smp(C.byref(sh), it, 1, 0, 0x100, 0x200, 0x300, None, ws, wsn, None) == INVALID
    assert smp(C.byref(sh), it, 1, 129, 0x100, 0x200, 0x300, None, ws, wsn, None) == CAP
    assert smp(C.byref(sh), _items(g, w_q=None), 1, 8, 0x100, 0x200, 0x300, None, ws, wsn, None) == INVALID
    assert smp(C.byref(sh), it, 1, 8, 0x100, 0x200, 0x300, None, ws, 8, None) == WS
    sel = L.gvote_score_select
    assert sel(C.byref(sh), it, 1, 8, 0x100, 0.0, 0, None, 0x200, None, None, ws, wsn, None) == INVALID
    assert sel(C.byref(sh), it, 1, 8, 0x100, 1.5, 0, None, 0x200, None, None, ws, wsn, None) == INVALID
    assert sel(C.byref(sh), it, 1, 8, 0x100, 0.9, 1, None, 0x200, None, None, ws, wsn, None) == INVALID
    assert sel(C.byref(sh), it, 1, 8, 0x100, 0.9, 5, None, 0x200, None, None, ws, wsn, None) == INVALID
    assert sel(C.byref(sh), it, 1, 8, None, 0.9, 0, None, 0x200, None, None, ws, wsn, None) == INVALID
    assert sel(C.byref(sh), _items(g, kv_head_stride=60), 1, 8, 0x100, 0.9, 0, None, 0x200, None, None, ws, wsn,
               None) == SHAPE
    uni = L.gvote_union_compact
    assert uni(C.byref(sh), it, 1, 8, 0x100, 0x200, 0x300, 0x400, 0x500, 0x600, None, 10, None, ws, wsn,
               None) == INVALID
    assert uni(C.byref(sh), it, 1, 8, 0x100, 0x200, 0x300, 0x400, 0x500, 0x600, None, -1, 0x700, ws, wsn,
               None) == INVALID
    assert uni(C.byref(sh), it, 1, 8, 0x100, 0x200, 0x300, 0x400, 0x500, 0x600, None, 10, 0x700, ws, 8,
               None) == WS
    assert L.gvote_count_rows(C.byref(sh), it, 1, 1, None, 8, 0x100, None) == INVALID
    assert L.gvote_count_rows(C.byref(sh), it, 1, 1, 0x100, 0, 0x200, None) == INVALID
    dec = L.gvote_decode_attention
    assert dec(C.byref(sh), 1, None, 0x100, 0x200, 0x300, 0x400, None, ws, wsn, None) == INVALID
    assert dec(C.byref(sh), 0, 0x100, 0x100, 0x200, 0x300, 0x400, None, ws, wsn, None) == INVALID
    assert dec(C.byref(sh), 1, 0x100, 0x100, 0x200, 0x300, 0x400, None, None, wsn, None) == INVALID
    assert dec(C.byref(sh), 1, 0x100, 0x100, 0x200, 0x300, 0x400, None, ws, 8, None) == WS
    assert dec(C.byref(_shape(g, head_dim=24)), 1, 0x100, 0x100, 0x200, 0x300, 0x400, None, ws, wsn, None) == UNSUP
    assert L.gvote_decode_workspace_bytes(C.byref(sh), 3) > 0 and L.gvote_decode_workspace_bytes(C.byref(sh), 0) == 0
    # the fit refuses a batch with more row chunks than one launch grid holds, before any launch
    assert fit(C.byref(sh), _items(g, 32, L=(1 << 31) - 8), 32, 1, 0x100, 0x200, ws, 1 << 40, None) == CAP
    # the static-scratch variant of stage 4 refuses calls beyond its array
    assert L.gvote_union_compact_static(C.byref(sh), _items(g, L=1 << 30), 1, 8, 0x100, 0x200, 0x300, 0x400, 0x500, 0x600,
                                        None, 10, 0x700, None) == CAP
    ovl = L.gvote_attention_overlap
    assert ovl(C.byref(sh), it, 1, 8, None, 0x100, 0x200, ws, wsn, None) == INVALID
    assert ovl(C.byref(sh), it, 1, 8, 0x100, 0x200, 0x300, ws, 8, None) == WS
    assert L.gvote_philox_u32(1, 2, -1, None, None) == INVALID
    assert L.gvote_philox_u32(1, 2, 0, None, None) == 0


def test_missing_library_is_a_loud_error(g, monkeypatch, tmp_path):
    import paper_2509_03136_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_HERE", str(tmp_path))
    with pytest.raises(ImportError):
        b.lib()


def test_bench_takes_traffic_only_from_profiles_of_these_kernel_sources(g):
    """bench.py fills roofline.traffic from the committed counter summary of the workload, and only when that summary
    carries the digest of the kernel sources in this tree (a summary of other sources must not be quoted)."""
    import sys
    sys.path.insert(0, ROOT)
    import bench
    from paper_2509_03136_amd.build import sources_digest
    path = os.path.join(ROOT, "profiles", "cfg3_llama8b_stack_32k_hbm_traffic_pmc.txt")
    assert os.path.exists(path)
    stamp = [l.split(":", 1)[1].strip() for l in open(path).read().splitlines() if l.startswith("kernel sources sha256:")]
    assert len(stamp) == 1 and len(stamp[0]) == 16
    got = bench.profiled_traffic("cfg3_llama8b_stack_32k", "moments_partial_kernel")
    step = bench.profiled_traffic("cfg3_llama8b_stack_32k", "whole step")
    if stamp[0] == sources_digest():
        assert 8.5e9 < got < 9.5e9          # the fit reads the hidden states (8.59 GB) once
        assert 12.9e9 < step < 20e9         # a step moves at least its algorithmic bytes
    else:
        assert got is None and step is None
    assert bench.profiled_traffic("no_such_workload", "moments_partial_kernel") is None
