"""MI355X-native GVote KV-cache selection: thin ctypes binding over libgvote.so.

The four stage calls have the names of the C ABI (include/gvote.h).  This layer only marshals
arguments (torch tensors -> device pointers, Python ints -> C ints); every step of the path runs
in the HIP kernels of the library.  PyTorch is used for device memory and streams only.
"""
from .binding import (  # noqa: F401
    GVoteError, Shape, Item, Batch, lib, lib_path, abi_version, status_string, workspace_bytes,
    fit_gaussian, sample_queries, score_select, union_compact, union_compact_static, count_rows, decode_attention, decode_workspace_bytes, attention_overlap,
    philox_u32, debug_set_spin_limit, Pipeline,
    SELECT_TOPP, SELECT_TOPK, F32, BF16,
)
