"""ctypes binding for include/failsafe.h: same names, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

FS_OK, FS_EINVAL, FS_ECAPACITY, FS_EHIP, FS_EUNSUPPORTED = 0, -1, -2, -3, -4
FS_MODE_TP, FS_MODE_DP = 0, 1
FS_KV_BF16, FS_KV_FP8_E4M3 = 0, 1
FS_V_ANY, FS_V_FP16_RANGE = 0, 1

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class FsError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"fs_status {status}: {message}")
        self.status = status


class FsShape(C.Structure):
    _fields_ = [("n_req", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("page_tokens", C.c_int32), ("n_ranks", C.c_int32)]


class FsKvView(C.Structure):
    _fields_ = [("q", C.c_void_p), ("k_pool", C.c_void_p), ("v_pool", C.c_void_p),
                ("k_slot_stride", C.c_int64), ("v_slot_stride", C.c_int64),
                ("k_scale", C.c_void_p), ("v_scale", C.c_void_p),
                ("page_indptr", C.c_void_p), ("page_ids", C.c_void_p),
                ("kv_dtype", C.c_int32), ("sm_scale", C.c_float), ("page_scales", C.c_void_p), ("v_range", C.c_int32)]


ITEM_DTYPE = np.dtype([(n, np.int32) for n in
                       ("req", "kv_head", "tok_begin", "tok_end", "pair", "chunk", "q_row", "part_row")])
PAIR_DTYPE = np.dtype([(n, np.int32) for n in ("req", "kv_head", "ctx_len", "n_chunks")])
RECORD_DTYPE = np.dtype([("first_page", np.int64), ("n_tok", np.int32), ("q_row", np.int32), ("row", np.int32),
                         ("n_chunks", np.int32), ("first_slots", np.int32, (8,)), ("pair", np.int32),
                         ("pair_row", np.int32)])
PREFILL_ENTRY_DTYPE = np.dtype([(n, np.int32) for n in ("req", "rank", "n_done", "n_new")])
PREFILL_ITEM_DTYPE = np.dtype([(n, np.int32) for n in
                               ("pair", "q_begin", "q_end", "n_done", "kv_begin", "kv_end", "q_row", "part_row")])
PREFILL_PAIR_DTYPE = np.dtype([(n, np.int32) for n in ("req", "kv_head", "n_done", "n_new")])


def library_path() -> str:
    """The in-tree library, or the build named by FAILSAFE_LIBRARY (for comparing two builds on one GPU)."""
    return os.environ.get("FAILSAFE_LIBRARY") or os.path.join(_PKG, "libfailsafe.so")


def load_library(path: str | None = None):
    """Load libfailsafe.so (built in-tree by paper_2511_14116_amd/build.py).  No fallback."""
    global _LIB
    if _LIB is not None and path is None:
        return _LIB
    p = path or library_path()
    try:
        # PyTorch ships a HIP runtime of its own.  If this library were loaded first it would bring in the system's,
        # and a process with both finds no device for this library's kernels; loading torch first makes both use one.
        import torch  # noqa: F401
    except ImportError:
        pass
    if not os.path.exists(p):
        raise FileNotFoundError(
            f"{p} is not built; run `python -m paper_2511_14116_amd.build` (needs hipcc) first")
    lib = C.CDLL(p)
    i32p, i64p, u8p = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_uint8)
    lib.fs_build_placement.argtypes = [C.POINTER(FsShape), i32p, u8p, i32p, C.c_int32, i32p, i32p, i64p]
    lib.fs_build_placement.restype = C.c_int
    lib.fs_build_placement_hybrid_heads.argtypes = [C.POINTER(FsShape), i32p, C.c_int32, i32p, i32p, i32p, i64p, i64p]
    lib.fs_build_placement_hybrid_heads.restype = C.c_int
    lib.fs_build_worklist.argtypes = [C.POINTER(FsShape), i32p, i32p, C.c_int32, C.c_int32,
                                      C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                      C.c_void_p, C.c_void_p, i64p, i64p]
    lib.fs_build_worklist.restype = C.c_int
    lib.fs_build_worklist_units.argtypes = [C.POINTER(FsShape), i32p, i32p, C.c_int32, C.c_int32,
                                            C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                            C.c_void_p, C.c_int64, C.c_void_p, i64p, i64p, i64p]
    lib.fs_build_worklist_units.restype = C.c_int
    lib.fs_decode_attention_units.argtypes = [C.POINTER(FsShape), C.POINTER(FsKvView), C.c_void_p, C.c_int64,
                                              C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                              C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.fs_decode_attention_units.restype = C.c_int
    lib.fs_build_launch_records.argtypes = [C.POINTER(FsShape), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                            C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p]
    lib.fs_build_launch_records.restype = C.c_int
    lib.fs_decode_attention_records.argtypes = [C.POINTER(FsShape), C.POINTER(FsKvView), C.c_void_p, C.c_int64,
                                                C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                                C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.fs_decode_attention_records.restype = C.c_int
    lib.fs_choose_chunk_tokens.argtypes = [C.POINTER(FsShape), i32p, i32p, C.c_int32, C.c_int32, C.c_int32, C.c_int64,
                                           i32p, i64p]
    lib.fs_choose_chunk_tokens.restype = C.c_int
    lib.fs_route_request.argtypes = [C.c_int32, i64p, C.c_int64, i32p]
    lib.fs_route_request.restype = C.c_int
    lib.fs_route_requests.argtypes = [C.c_int32, i64p, i64p, C.c_int32, i32p]
    lib.fs_route_requests.restype = C.c_int
    lib.fs_schedule_prefill.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, i64p, i32p, i64p, i32p]
    lib.fs_schedule_prefill.restype = C.c_int
    lib.fs_plan_kv_reload.argtypes = [C.c_int32, C.c_int32, i32p, i32p, i32p, C.c_int32, u8p, i64p, i64p]
    lib.fs_plan_kv_reload.restype = C.c_int
    lib.fs_replace_failed_gpu.argtypes = [C.c_int32, C.c_int32, i32p, i32p, i32p, C.c_int32, u8p, i32p, i32p, i64p]
    lib.fs_replace_failed_gpu.restype = C.c_int
    lib.fs_plan_ffn_reload.argtypes = [C.c_int32, i32p, C.c_int32, u8p, i32p, i32p]
    lib.fs_plan_ffn_reload.restype = C.c_int
    lib.fs_build_prefill_worklist.argtypes = [C.POINTER(FsShape), i32p, i32p, i32p, C.c_int32, C.c_int32, C.c_int32,
                                              C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                              C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, i64p, i64p, i64p]
    lib.fs_build_prefill_worklist.restype = C.c_int
    lib.fs_choose_prefill_chunk.argtypes = [C.POINTER(FsShape), i32p, i32p, i32p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                            C.c_int64, i32p, i64p]
    lib.fs_choose_prefill_chunk.restype = C.c_int
    lib.fs_prefill_tile_tokens.argtypes = [C.c_int32]
    lib.fs_prefill_tile_tokens.restype = C.c_int32
    lib.fs_prefill_attention.argtypes = [C.POINTER(FsShape), C.POINTER(FsKvView), C.c_void_p, C.c_void_p,
                                         C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.fs_prefill_attention.restype = C.c_int
    lib.fs_prefill_attention_fused.argtypes = [C.POINTER(FsShape), C.POINTER(FsKvView), C.c_void_p, C.c_void_p,
                                               C.c_int64, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p,
                                               C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.fs_prefill_attention_fused.restype = C.c_int
    lib.fs_kv_elem_offset.argtypes = [C.c_int32] * 4
    lib.fs_kv_elem_offset.restype = C.c_int32
    lib.fs_decode_attention.argtypes = [C.POINTER(FsShape), C.POINTER(FsKvView), C.c_void_p, C.c_void_p,
                                        C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.fs_decode_attention.restype = C.c_int
    lib.fs_decode_attention_persistent.argtypes = [C.POINTER(FsShape), C.POINTER(FsKvView), C.c_void_p, C.c_void_p,
                                                   C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.fs_decode_attention_persistent.restype = C.c_int
    lib.fs_decode_attention_fused.argtypes = [C.POINTER(FsShape), C.POINTER(FsKvView), C.c_void_p, C.c_void_p,
                                              C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_void_p]
    lib.fs_decode_attention_fused.restype = C.c_int
    lib.fs_decode_attention_fused_static.argtypes = [C.POINTER(FsShape), C.POINTER(FsKvView), C.c_void_p, C.c_void_p,
                                                     C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.fs_decode_attention_fused_static.restype = C.c_int
    lib.fs_merge_lse.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32,
                                 C.c_void_p, C.c_void_p, C.c_void_p]
    lib.fs_merge_lse.restype = C.c_int
    lib.fs_pack_kv_slots.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.c_void_p]
    lib.fs_pack_kv_slots.restype = C.c_int
    lib.fs_stream_read_probe.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
    lib.fs_stream_read_probe.restype = C.c_int
    lib.fs_set_option.argtypes = [C.c_char_p, C.c_int32]
    lib.fs_set_option.restype = C.c_int
    lib.fs_get_option.argtypes = [C.c_char_p]
    lib.fs_get_option.restype = C.c_int32
    lib.fs_last_error.argtypes = []
    lib.fs_last_error.restype = C.c_char_p
    lib.fs_abi_version.argtypes = []
    lib.fs_abi_version.restype = C.c_int32
    if path is None:
        _LIB = lib
    return lib


def fs_last_error() -> str:
    return load_library().fs_last_error().decode()


def fs_abi_version() -> int:
    return load_library().fs_abi_version()


def _check(st: int):
    if st != FS_OK:
        raise FsError(st, fs_last_error())


def _ptr(x):
    """Address of a device tensor / host array / raw int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    raise TypeError(type(x))


def _host(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def fs_build_placement(shape: FsShape, ctx_len, mode, rot=None, layer: int = 0, rank_load=None):
    """-> (owner [B][H_kv] int32, dp_rank [B] int32, rank_load [R] int64)."""
    lib = load_library()
    B, H, R = shape.n_req, shape.n_kv_heads, shape.n_ranks
    ctx = _host(ctx_len, np.int32)
    md = _host(mode, np.uint8)
    if len(ctx) != B or len(md) != B:
        raise ValueError("ctx_len and mode must have n_req entries")
    rt = None if rot is None else _host(rot, np.int32)
    owner = np.empty((max(B, 0), max(H, 0)), dtype=np.int32)
    dp = np.empty(max(B, 0), dtype=np.int32)
    load = np.zeros(max(R, 0), dtype=np.int64) if rank_load is None else np.array(rank_load, dtype=np.int64)
    i32p, i64p, u8p = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_uint8)
    st = lib.fs_build_placement(C.byref(shape), ctx.ctypes.data_as(i32p), md.ctypes.data_as(u8p),
                                None if rt is None else rt.ctypes.data_as(i32p), layer,
                                owner.ctypes.data_as(i32p), dp.ctypes.data_as(i32p), load.ctypes.data_as(i64p))
    _check(st)
    return owner, dp, load


def fs_build_placement_hybrid_heads(shape: FsShape, ctx_len, layer: int = 0, route=None, rank_load=None,
                                    dp_load=None):
    """-> (owner [B][H_kv] int32, dp_rank [B] int32, rank_load [R] int64, dp_load [R] int64)."""
    lib = load_library()
    B, H, R = shape.n_req, shape.n_kv_heads, shape.n_ranks
    ctx = _host(ctx_len, np.int32)
    if len(ctx) != B:
        raise ValueError("ctx_len must have n_req entries")
    rt = None if route is None else _host(route, np.int32)
    owner = np.empty((max(B, 0), max(H, 0)), dtype=np.int32)
    dp = np.empty(max(B, 0), dtype=np.int32)
    load = np.zeros(max(R, 0), dtype=np.int64) if rank_load is None else np.array(rank_load, dtype=np.int64)
    dload = np.zeros(max(R, 0), dtype=np.int64) if dp_load is None else np.array(dp_load, dtype=np.int64)
    i32p, i64p = C.POINTER(C.c_int32), C.POINTER(C.c_int64)
    st = lib.fs_build_placement_hybrid_heads(C.byref(shape), ctx.ctypes.data_as(i32p), layer,
                                             None if rt is None else rt.ctypes.data_as(i32p),
                                             owner.ctypes.data_as(i32p), dp.ctypes.data_as(i32p),
                                             load.ctypes.data_as(i64p), dload.ctypes.data_as(i64p))
    _check(st)
    return owner, dp, load, dload


def fs_build_worklist(shape: FsShape, ctx_len, owner, rank: int, chunk_tokens: int, out=None):
    """-> (items [n] ITEM_DTYPE, pairs [m] PAIR_DTYPE, sched [n] int32, chunk_indptr [m+1] int64).

    ``out`` may hold preallocated host arrays (items, pairs, sched, chunk_indptr), e.g. views
    of pinned memory; they are filled in place and sliced to the counts."""
    lib = load_library()
    ctx = _host(ctx_len, np.int32)
    own = _host(owner, np.int32)
    i32p, i64p = C.POINTER(C.c_int32), C.POINTER(C.c_int64)
    n_items, n_pairs = C.c_int64(0), C.c_int64(0)
    if out is None:
        st = lib.fs_build_worklist(C.byref(shape), ctx.ctypes.data_as(i32p), own.ctypes.data_as(i32p), rank,
                                   chunk_tokens, None, 0, None, 0, None, None, C.byref(n_items), C.byref(n_pairs))
        _check(st)
        items = np.empty(n_items.value, dtype=ITEM_DTYPE)
        pairs = np.empty(n_pairs.value, dtype=PAIR_DTYPE)
        sched = np.empty(n_items.value, dtype=np.int32)
        indptr = np.empty(n_pairs.value + 1, dtype=np.int64)
    else:
        items, pairs, sched, indptr = out
    st = lib.fs_build_worklist(C.byref(shape), ctx.ctypes.data_as(i32p), own.ctypes.data_as(i32p), rank,
                               chunk_tokens, items.ctypes.data, len(items), pairs.ctypes.data, len(pairs),
                               sched.ctypes.data, indptr.ctypes.data, C.byref(n_items), C.byref(n_pairs))
    _check(st)
    n, m = n_items.value, n_pairs.value
    return items[:n], pairs[:m], sched[:n], indptr[:m + 1]


def fs_build_worklist_units(shape: FsShape, ctx_len, owner, rank: int, n_units: int):
    """-> (items [n] ITEM_DTYPE, pairs [m] PAIR_DTYPE, unit_indptr [U+1] int64, chunk_indptr [m+1] int64):
    the rank's share cut into U = min(n_units, pages) equal runs of pages."""
    lib = load_library()
    ctx = _host(ctx_len, np.int32)
    own = _host(owner, np.int32)
    i32p = C.POINTER(C.c_int32)
    n_items, n_pairs, n_u = C.c_int64(0), C.c_int64(0), C.c_int64(0)
    args = (C.byref(shape), ctx.ctypes.data_as(i32p), own.ctypes.data_as(i32p), rank, n_units)
    counts = (C.byref(n_items), C.byref(n_pairs), C.byref(n_u))
    _check(lib.fs_build_worklist_units(*args, None, 0, None, 0, None, 0, None, *counts))
    items = np.empty(n_items.value, dtype=ITEM_DTYPE)
    pairs = np.empty(n_pairs.value, dtype=PAIR_DTYPE)
    unit_indptr = np.empty(n_u.value + 1, dtype=np.int64)
    chunk_indptr = np.empty(n_pairs.value + 1, dtype=np.int64)
    _check(lib.fs_build_worklist_units(*args, items.ctypes.data, len(items), pairs.ctypes.data, len(pairs),
                                       unit_indptr.ctypes.data, n_u.value, chunk_indptr.ctypes.data, *counts))
    return items, pairs, unit_indptr, chunk_indptr


def fs_build_launch_records(shape: FsShape, items, order, chunk_indptr, page_indptr, page_ids, direct_rows: bool = True,
                            out=None):
    """-> records [n_items] RECORD_DTYPE: record k describes item order[k] (order None: item k).  ``out``: a
    preallocated RECORD_DTYPE array (e.g. a view of pinned memory) to fill instead."""
    lib = load_library()
    it = np.ascontiguousarray(items)
    if it.dtype != ITEM_DTYPE:
        raise TypeError("items must be an ITEM_DTYPE array")
    od = None if order is None else _host(order, np.int32)
    ci, pi, ids = _host(chunk_indptr, np.int64), _host(page_indptr, np.int64), _host(page_ids, np.int32)
    if od is not None and len(od) != len(it):
        raise ValueError("order must have one entry per item")
    if len(pi) != len(ci):
        raise ValueError("chunk_indptr and page_indptr must both have n_pairs+1 entries")
    rec = np.zeros(len(it), dtype=RECORD_DTYPE) if out is None else out
    if rec.dtype != RECORD_DTYPE or len(rec) < len(it):
        raise TypeError("out must be a RECORD_DTYPE array with room for every item")
    st = lib.fs_build_launch_records(C.byref(shape), it.ctypes.data, None if od is None else od.ctypes.data, len(it),
                                     ci.ctypes.data, len(ci) - 1, pi.ctypes.data, ids.ctypes.data, len(ids),
                                     int(bool(direct_rows)), rec.ctypes.data)
    _check(st)
    return rec[:len(it)]


def fs_choose_chunk_tokens(shape: FsShape, ctx_len, owner, rank: int, max_chunk: int, min_chunk: int,
                           n_slots: int):
    """-> (chunk_tokens, n_items): the split-K chunk for ``rank``'s share, four thirds of the share of the cached tokens
    that one of ``n_slots`` concurrently running workgroups would get, in whole pages within [min_chunk, max_chunk], and
    the list's length with it."""
    lib = load_library()
    ctx = _host(ctx_len, np.int32)
    own = _host(owner, np.int32)
    i32p = C.POINTER(C.c_int32)
    chunk, n_items = C.c_int32(0), C.c_int64(0)
    _check(lib.fs_choose_chunk_tokens(C.byref(shape), ctx.ctypes.data_as(i32p), own.ctypes.data_as(i32p), rank,
                                      max_chunk, min_chunk, n_slots, C.byref(chunk), C.byref(n_items)))
    return chunk.value, n_items.value


def fs_route_request(pending: np.ndarray, work: int) -> int:
    """Route one request; ``pending`` (int64, one entry per rank) is updated in place.  -> rank."""
    if not isinstance(pending, np.ndarray) or pending.dtype != np.int64 or not pending.flags.c_contiguous:
        raise TypeError("pending must be a contiguous int64 array (it is updated in place)")
    rank = C.c_int32(-1)
    st = load_library().fs_route_request(len(pending), pending.ctypes.data_as(C.POINTER(C.c_int64)), work,
                                         C.byref(rank))
    _check(st)
    return rank.value


def fs_route_requests(pending: np.ndarray, work) -> np.ndarray:
    """Route a queue of requests in arrival order; ``pending`` (int64, one entry per rank) is updated in
    place.  -> ranks [n] int32."""
    if not isinstance(pending, np.ndarray) or pending.dtype != np.int64 or not pending.flags.c_contiguous:
        raise TypeError("pending must be a contiguous int64 array (it is updated in place)")
    work = np.ascontiguousarray(work, dtype=np.int64)
    if work.ndim != 1:
        raise ValueError("work must be one-dimensional")
    rank = np.full(len(work), -1, dtype=np.int32)
    st = load_library().fs_route_requests(len(pending), pending.ctypes.data_as(C.POINTER(C.c_int64)),
                                          work.ctypes.data_as(C.POINTER(C.c_int64)), len(work),
                                          rank.ctypes.data_as(C.POINTER(C.c_int32)))
    _check(st)
    return rank


def fs_schedule_prefill(n_ranks: int, budget: int, min_tokens: int, entries, init_load=None):
    """-> (take [n_entries] int32, load [R] int64, n_tokens).  ``entries``: PREFILL_ENTRY_DTYPE array or
    rows of (req, rank, n_done, n_new)."""
    lib = load_library()
    if isinstance(entries, np.ndarray) and entries.dtype == PREFILL_ENTRY_DTYPE:
        ent = np.ascontiguousarray(entries)
    else:
        ent = np.ascontiguousarray(np.asarray(entries, dtype=np.int32).reshape(-1, 4)).view(PREFILL_ENTRY_DTYPE).reshape(-1)
    n = len(ent)
    take = np.zeros(n, dtype=np.int32)
    load = np.zeros(max(n_ranks, 0), dtype=np.int64)
    init = None if init_load is None else _host(init_load, np.int64)
    if init is not None and len(init) != n_ranks:
        raise ValueError("init_load must have one entry per rank")
    n_tok = C.c_int32(0)
    i32p, i64p = C.POINTER(C.c_int32), C.POINTER(C.c_int64)
    st = lib.fs_schedule_prefill(n_ranks, budget, min_tokens, ent.ctypes.data if n else None, n,
                                 None if init is None else init.ctypes.data_as(i64p),
                                 take.ctypes.data_as(i32p), load.ctypes.data_as(i64p), C.byref(n_tok))
    _check(st)
    return take, load, n_tok.value


def _owner2d(a, B):
    a = np.ascontiguousarray(a, dtype=np.int32)
    if a.ndim != 2 or a.shape[0] != B:
        raise ValueError("owner maps must be [n_req][n_kv_heads]")
    return a


def _alive(alive):
    return np.ascontiguousarray(np.asarray(alive) != 0, dtype=np.uint8)


def fs_plan_kv_reload(ctx_len, old_owner, new_owner, alive):
    """-> (reload [n_gpus] int64, reuse [n_gpus] int64), KV tokens x KV heads per GPU for one layer."""
    ctx = _host(ctx_len, np.int32)
    old, new = _owner2d(old_owner, len(ctx)), _owner2d(new_owner, len(ctx))
    if old.shape != new.shape:
        raise ValueError("owner maps differ in shape")
    al = _alive(alive)
    n_gpus = len(al)
    reload = np.zeros(n_gpus, dtype=np.int64)
    reuse = np.zeros(n_gpus, dtype=np.int64)
    i32p, i64p, u8p = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_uint8)
    st = load_library().fs_plan_kv_reload(len(ctx), old.shape[1], ctx.ctypes.data_as(i32p), old.ctypes.data_as(i32p),
                                          new.ctypes.data_as(i32p), n_gpus, al.ctypes.data_as(u8p),
                                          reload.ctypes.data_as(i64p), reuse.ctypes.data_as(i64p))
    _check(st)
    return reload, reuse


def fs_replace_failed_gpu(ctx_len, old_owner, old_dp_rank, alive, dp_load=None):
    """-> (new_owner [B][H] int32, new_dp_rank [B] int32, dp_load [n_gpus] int64)."""
    ctx = _host(ctx_len, np.int32)
    old = _owner2d(old_owner, len(ctx))
    odp = _host(old_dp_rank, np.int32)
    if len(odp) != len(ctx):
        raise ValueError("old_dp_rank must have n_req entries")
    new = np.empty_like(old)
    ndp = np.empty_like(odp)
    al = _alive(alive)
    n_gpus = len(al)
    load = np.zeros(n_gpus, dtype=np.int64) if dp_load is None else np.array(dp_load, dtype=np.int64)
    if len(load) != n_gpus:
        raise ValueError("dp_load must have one entry per GPU")
    i32p, i64p, u8p = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_uint8)
    st = load_library().fs_replace_failed_gpu(len(ctx), old.shape[1], ctx.ctypes.data_as(i32p),
                                              old.ctypes.data_as(i32p), odp.ctypes.data_as(i32p), n_gpus, al.ctypes.data_as(u8p),
                                              new.ctypes.data_as(i32p), ndp.ctypes.data_as(i32p),
                                              load.ctypes.data_as(i64p))
    _check(st)
    return new, ndp, load


def fs_plan_ffn_reload(shard_owner, alive):
    """-> (new_owner [n_shards] int32, n_load [n_gpus] int32)."""
    own = _host(shard_owner, np.int32)
    new = np.empty_like(own)
    al = _alive(alive)
    n_gpus = len(al)
    n_load = np.zeros(n_gpus, dtype=np.int32)
    i32p, u8p = C.POINTER(C.c_int32), C.POINTER(C.c_uint8)
    st = load_library().fs_plan_ffn_reload(len(own), own.ctypes.data_as(i32p), n_gpus, al.ctypes.data_as(u8p),
                                           new.ctypes.data_as(i32p), n_load.ctypes.data_as(i32p))
    _check(st)
    return new, n_load


def fs_prefill_tile_tokens(group: int) -> int:
    return load_library().fs_prefill_tile_tokens(group)


def fs_build_prefill_worklist(shape: FsShape, n_done, n_new, owner, rank: int, tile_tokens: int,
                              kv_chunk_tokens: int = 0):
    """-> (items [n] PREFILL_ITEM_DTYPE, pairs [m] PREFILL_PAIR_DTYPE, sched [n] int32,
    chunk_indptr [n_tiles+1] int64, out_indptr [m+1] int64)."""
    lib = load_library()
    nd, nn, own = _host(n_done, np.int32), _host(n_new, np.int32), _host(owner, np.int32)
    if len(nd) != shape.n_req or len(nn) != shape.n_req or own.size != shape.n_req * shape.n_kv_heads:
        raise ValueError("n_done, n_new and owner must match the shape")
    i32p = C.POINTER(C.c_int32)
    n_items, n_pairs, n_tiles = C.c_int64(0), C.c_int64(0), C.c_int64(0)
    args = (C.byref(shape), nd.ctypes.data_as(i32p), nn.ctypes.data_as(i32p), own.ctypes.data_as(i32p), rank,
            tile_tokens, kv_chunk_tokens)
    counts = (C.byref(n_items), C.byref(n_pairs), C.byref(n_tiles))
    _check(lib.fs_build_prefill_worklist(*args, None, 0, None, 0, None, None, 0, None, *counts))
    items = np.empty(n_items.value, dtype=PREFILL_ITEM_DTYPE)
    pairs = np.empty(n_pairs.value, dtype=PREFILL_PAIR_DTYPE)
    sched = np.empty(n_items.value, dtype=np.int32)
    chunk_indptr = np.empty(n_tiles.value + 1, dtype=np.int64)
    out_indptr = np.empty(n_pairs.value + 1, dtype=np.int64)
    _check(lib.fs_build_prefill_worklist(*args, items.ctypes.data, len(items), pairs.ctypes.data, len(pairs),
                                         sched.ctypes.data, chunk_indptr.ctypes.data, n_tiles.value,
                                         out_indptr.ctypes.data, *counts))
    return items, pairs, sched, chunk_indptr, out_indptr


def fs_choose_prefill_chunk(shape: FsShape, n_done, n_new, owner, rank: int, tile_tokens: int, max_chunk: int,
                            min_chunk: int, n_slots: int):
    """-> (kv_chunk_tokens, n_items): the split-K chunk for ``rank``'s batch, four thirds of the share of the keys that
    one of ``n_slots`` concurrently running workgroups would get, within [min_chunk, max_chunk], and the list's length
    with it."""
    nd, nn, own = _host(n_done, np.int32), _host(n_new, np.int32), _host(owner, np.int32)
    if len(nd) != shape.n_req or len(nn) != shape.n_req or own.size != shape.n_req * shape.n_kv_heads:
        raise ValueError("n_done, n_new and owner must match the shape")
    i32p = C.POINTER(C.c_int32)
    chunk, n_items = C.c_int32(0), C.c_int64(0)
    _check(load_library().fs_choose_prefill_chunk(C.byref(shape), nd.ctypes.data_as(i32p), nn.ctypes.data_as(i32p),
                                                  own.ctypes.data_as(i32p), rank, tile_tokens, max_chunk, min_chunk,
                                                  n_slots, C.byref(chunk), C.byref(n_items)))
    return chunk.value, n_items.value


def fs_prefill_attention(shape: FsShape, kv: FsKvView, items_dev, sched_dev, n_items: int, tile_tokens: int,
                         part_o, part_lse, stream=None) -> None:
    st = load_library().fs_prefill_attention(C.byref(shape), C.byref(kv), _ptr(items_dev), _ptr(sched_dev),
                                             n_items, tile_tokens, _ptr(part_o), _ptr(part_lse), _ptr(stream))
    _check(st)


def fs_prefill_attention_fused(shape: FsShape, kv: FsKvView, items_dev, sched_dev, n_items: int, tile_tokens: int,
                               chunk_indptr_dev, n_tiles: int, out_indptr_dev, part_o, part_lse, out, lse,
                               stream=None) -> None:
    st = load_library().fs_prefill_attention_fused(C.byref(shape), C.byref(kv), _ptr(items_dev), _ptr(sched_dev),
                                                   n_items, tile_tokens, _ptr(chunk_indptr_dev), n_tiles,
                                                   _ptr(out_indptr_dev), _ptr(part_o), _ptr(part_lse), _ptr(out),
                                                   _ptr(lse), _ptr(stream))
    _check(st)


def fs_kv_elem_offset(kv_dtype: int, is_v: int, tok: int, d: int) -> int:
    return load_library().fs_kv_elem_offset(kv_dtype, is_v, tok, d)


def fs_decode_attention(shape: FsShape, kv: FsKvView, items_dev, sched_dev, n_items: int,
                        part_o, part_lse, stream=None) -> None:
    st = load_library().fs_decode_attention(C.byref(shape), C.byref(kv), _ptr(items_dev), _ptr(sched_dev),
                                            n_items, _ptr(part_o), _ptr(part_lse), _ptr(stream))
    _check(st)


def fs_decode_attention_persistent(shape: FsShape, kv: FsKvView, items_dev, sched_dev, n_items: int, claim_dev,
                                   part_o, part_lse, stream=None) -> None:
    st = load_library().fs_decode_attention_persistent(C.byref(shape), C.byref(kv), _ptr(items_dev), _ptr(sched_dev),
                                                       n_items, _ptr(claim_dev), _ptr(part_o), _ptr(part_lse),
                                                       _ptr(stream))
    _check(st)


def fs_decode_attention_fused(shape: FsShape, kv: FsKvView, items_dev, sched_dev, n_items: int, chunk_indptr_dev,
                              n_pairs: int, part_o, part_lse, claim_dev, out, lse, stream=None) -> None:
    st = load_library().fs_decode_attention_fused(C.byref(shape), C.byref(kv), _ptr(items_dev), _ptr(sched_dev),
                                                  n_items, _ptr(chunk_indptr_dev), n_pairs, _ptr(part_o),
                                                  _ptr(part_lse), _ptr(claim_dev), _ptr(out), _ptr(lse), _ptr(stream))
    _check(st)


def fs_decode_attention_fused_static(shape: FsShape, kv: FsKvView, items_dev, sched_dev, n_items: int,
                                     chunk_indptr_dev, n_pairs: int, out, lse, stream=None) -> None:
    st = load_library().fs_decode_attention_fused_static(C.byref(shape), C.byref(kv), _ptr(items_dev), _ptr(sched_dev),
                                                         n_items, _ptr(chunk_indptr_dev), n_pairs, _ptr(out), _ptr(lse),
                                                         _ptr(stream))
    _check(st)


def fs_decode_attention_units(shape: FsShape, kv: FsKvView, items_dev, n_items: int, unit_indptr_dev, n_units: int,
                              chunk_indptr_dev, n_pairs: int, part_o, part_lse, out, lse, stream=None) -> None:
    st = load_library().fs_decode_attention_units(C.byref(shape), C.byref(kv), _ptr(items_dev), n_items,
                                                  _ptr(unit_indptr_dev), n_units, _ptr(chunk_indptr_dev), n_pairs,
                                                  _ptr(part_o), _ptr(part_lse), _ptr(out), _ptr(lse), _ptr(stream))
    _check(st)


def fs_decode_attention_records(shape: FsShape, kv: FsKvView, records_dev, n_items: int, unit_indptr_dev, n_units: int,
                                chunk_indptr_dev, n_pairs: int, part_o, part_lse, out, lse, pair_counters_dev=None,
                                claim_dev=None, stream=None) -> None:
    st = load_library().fs_decode_attention_records(C.byref(shape), C.byref(kv), _ptr(records_dev), n_items,
                                                    _ptr(unit_indptr_dev), n_units, _ptr(chunk_indptr_dev), n_pairs,
                                                    _ptr(part_o), _ptr(part_lse), _ptr(out), _ptr(lse),
                                                    _ptr(pair_counters_dev), _ptr(claim_dev), _ptr(stream))
    _check(st)


def fs_merge_lse(part_o, part_lse, chunk_indptr_dev, n_pairs: int, group: int, head_dim: int,
                 out, lse, stream=None) -> None:
    st = load_library().fs_merge_lse(_ptr(part_o), _ptr(part_lse), _ptr(chunk_indptr_dev), n_pairs, group,
                                     head_dim, _ptr(out), _ptr(lse), _ptr(stream))
    _check(st)


def fs_pack_kv_slots(src_dev, src_slot_stride: int, dst_dev, dst_slot_stride: int, n_slots: int, kv_dtype: int,
                     is_v: bool, stream=None) -> None:
    _check(load_library().fs_pack_kv_slots(_ptr(src_dev), src_slot_stride, _ptr(dst_dev), dst_slot_stride, n_slots,
                                           kv_dtype, int(bool(is_v)), _ptr(stream)))


def fs_stream_read_probe(buf_dev, nbytes: int, sink_dev, stream=None) -> None:
    _check(load_library().fs_stream_read_probe(_ptr(buf_dev), nbytes, _ptr(sink_dev), _ptr(stream)))


class BoundCall:
    """One library call with its arguments marshalled once.  A serving loop that repeats the
    same call on the same buffers every step pays only the foreign call itself afterwards.
    The arrays the pointers refer to are kept alive by the object."""

    __slots__ = ("_fn", "_args", "_keep", "n_items", "n_pairs", "n_tiles")

    def __init__(self, fn, args, keep, n_items=None, n_pairs=None, n_tiles=None):
        self._fn, self._args, self._keep = fn, args, keep
        self.n_items, self.n_pairs, self.n_tiles = n_items, n_pairs, n_tiles

    def __call__(self) -> None:
        st = self._fn(*self._args)
        if st != FS_OK:
            raise FsError(st, fs_last_error())


def _vp(x):
    p = _ptr(x)
    return C.c_void_p(p) if p is not None else None


def bind_build_placement(shape: FsShape, ctx_len: np.ndarray, mode: np.ndarray, owner: np.ndarray,
                         dp_rank: np.ndarray, rank_load: np.ndarray, rot=None, layer: int = 0) -> BoundCall:
    """fs_build_placement on caller-held arrays (int32 ctx_len/owner/dp_rank, uint8 mode, int64
    rank_load).  rank_load is in/out: zero it before each call for a fresh batch."""
    lib = load_library()
    for a, dt in ((ctx_len, np.int32), (mode, np.uint8), (owner, np.int32), (dp_rank, np.int32), (rank_load, np.int64)):
        if a.dtype != dt or not a.flags.c_contiguous:
            raise TypeError("bind_build_placement needs contiguous arrays of the documented dtypes")
    i32p, i64p, u8p = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_uint8)
    args = (C.byref(shape), ctx_len.ctypes.data_as(i32p), mode.ctypes.data_as(u8p),
            None if rot is None else rot.ctypes.data_as(i32p), C.c_int32(layer),
            owner.ctypes.data_as(i32p), dp_rank.ctypes.data_as(i32p), rank_load.ctypes.data_as(i64p))
    return BoundCall(lib.fs_build_placement, args, (shape, ctx_len, mode, rot, owner, dp_rank, rank_load))


def bind_build_placement_hybrid_heads(shape: FsShape, ctx_len: np.ndarray, owner: np.ndarray, dp_rank: np.ndarray,
                                      rank_load: np.ndarray, dp_load: np.ndarray, layer: int = 0, route=None) -> BoundCall:
    """fs_build_placement_hybrid_heads on caller-held arrays; zero both load arrays for a fresh batch."""
    lib = load_library()
    for a, dt in ((ctx_len, np.int32), (owner, np.int32), (dp_rank, np.int32), (rank_load, np.int64), (dp_load, np.int64)):
        if a.dtype != dt or not a.flags.c_contiguous:
            raise TypeError("bind_build_placement_hybrid_heads needs contiguous arrays of the documented dtypes")
    i32p, i64p = C.POINTER(C.c_int32), C.POINTER(C.c_int64)
    args = (C.byref(shape), ctx_len.ctypes.data_as(i32p), C.c_int32(layer),
            None if route is None else route.ctypes.data_as(i32p),
            owner.ctypes.data_as(i32p), dp_rank.ctypes.data_as(i32p),
            rank_load.ctypes.data_as(i64p), dp_load.ctypes.data_as(i64p))
    return BoundCall(lib.fs_build_placement_hybrid_heads, args, (shape, ctx_len, route, owner, dp_rank, rank_load, dp_load))


def bind_route_requests(pending: np.ndarray, work: np.ndarray, rank_out: np.ndarray) -> BoundCall:
    """fs_route_requests on caller-held arrays: pending int64 [R] (in/out: set it before each call), work int64 [n],
    rank_out int32 [n]."""
    lib = load_library()
    for a, dt in ((pending, np.int64), (work, np.int64), (rank_out, np.int32)):
        if a.dtype != dt or not a.flags.c_contiguous or a.ndim != 1:
            raise TypeError("bind_route_requests needs contiguous one-dimensional arrays of the documented dtypes")
    if len(rank_out) != len(work):
        raise ValueError("rank_out must have one entry per request")
    i32p, i64p = C.POINTER(C.c_int32), C.POINTER(C.c_int64)
    args = (C.c_int32(len(pending)), pending.ctypes.data_as(i64p), work.ctypes.data_as(i64p), C.c_int32(len(work)),
            rank_out.ctypes.data_as(i32p))
    return BoundCall(lib.fs_route_requests, args, (pending, work, rank_out))


def bind_schedule_prefill(n_ranks: int, budget: int, min_tokens: int, entries: np.ndarray, take: np.ndarray,
                          load: np.ndarray, init_load=None) -> BoundCall:
    """fs_schedule_prefill on caller-held arrays: entries PREFILL_ENTRY_DTYPE [n] (read at every call), take int32 [n]
    and load int64 [R] written.  After a call the batch's token count is in .n_items.value."""
    lib = load_library()
    if entries.dtype != PREFILL_ENTRY_DTYPE or not entries.flags.c_contiguous or take.dtype != np.int32 or \
            len(take) != len(entries) or load.dtype != np.int64 or len(load) != n_ranks:
        raise TypeError("bind_schedule_prefill: arrays do not match the documented layouts")
    if init_load is not None and (init_load.dtype != np.int64 or len(init_load) != n_ranks):
        raise TypeError("bind_schedule_prefill: init_load must be int64 [n_ranks]")
    i32p, i64p = C.POINTER(C.c_int32), C.POINTER(C.c_int64)
    n_tok = C.c_int32(0)
    args = (C.c_int32(n_ranks), C.c_int32(budget), C.c_int32(min_tokens), C.c_void_p(entries.ctypes.data),
            C.c_int32(len(entries)), None if init_load is None else init_load.ctypes.data_as(i64p),
            take.ctypes.data_as(i32p), load.ctypes.data_as(i64p), C.byref(n_tok))
    return BoundCall(lib.fs_schedule_prefill, args, (entries, take, load, init_load, n_tok), n_items=n_tok)


def bind_build_worklist(shape: FsShape, ctx_len: np.ndarray, owner: np.ndarray, rank: int, chunk_tokens: int,
                        items: np.ndarray, pairs: np.ndarray, sched: np.ndarray, chunk_indptr: np.ndarray) -> BoundCall:
    """fs_build_worklist into caller-held arrays (e.g. views of pinned memory).  After a call the
    counts are in .n_items.value and .n_pairs.value."""
    lib = load_library()
    i32p, i64p = C.POINTER(C.c_int32), C.POINTER(C.c_int64)
    n_items, n_pairs = C.c_int64(0), C.c_int64(0)
    args = (C.byref(shape), ctx_len.ctypes.data_as(i32p), owner.ctypes.data_as(i32p), C.c_int32(rank),
            C.c_int32(chunk_tokens), C.c_void_p(items.ctypes.data), C.c_int64(len(items)),
            C.c_void_p(pairs.ctypes.data), C.c_int64(len(pairs)), C.c_void_p(sched.ctypes.data),
            C.c_void_p(chunk_indptr.ctypes.data), C.byref(n_items), C.byref(n_pairs))
    return BoundCall(lib.fs_build_worklist, args, (shape, ctx_len, owner, items, pairs, sched, chunk_indptr),
                     n_items, n_pairs)


def bind_build_worklist_units(shape: FsShape, ctx_len: np.ndarray, owner: np.ndarray, rank: int, n_units: int,
                              items: np.ndarray, pairs: np.ndarray, unit_indptr: np.ndarray,
                              chunk_indptr: np.ndarray) -> BoundCall:
    """fs_build_worklist_units into caller-held arrays (e.g. views of pinned memory).  After a call the counts
    are in .n_items.value, .n_pairs.value and .n_tiles.value (the number of units)."""
    lib = load_library()
    i32p = C.POINTER(C.c_int32)
    n_items, n_pairs, n_u = C.c_int64(0), C.c_int64(0), C.c_int64(0)
    args = (C.byref(shape), ctx_len.ctypes.data_as(i32p), owner.ctypes.data_as(i32p), C.c_int32(rank), C.c_int32(n_units),
            C.c_void_p(items.ctypes.data), C.c_int64(len(items)), C.c_void_p(pairs.ctypes.data), C.c_int64(len(pairs)),
            C.c_void_p(unit_indptr.ctypes.data), C.c_int64(len(unit_indptr) - 1), C.c_void_p(chunk_indptr.ctypes.data),
            C.byref(n_items), C.byref(n_pairs), C.byref(n_u))
    return BoundCall(lib.fs_build_worklist_units, args, (shape, ctx_len, owner, items, pairs, unit_indptr, chunk_indptr),
                     n_items, n_pairs, n_u)


def bind_build_prefill_worklist(shape: FsShape, n_done: np.ndarray, n_new: np.ndarray, owner: np.ndarray, rank: int,
                                tile_tokens: int, kv_chunk_tokens: int, items: np.ndarray, pairs: np.ndarray,
                                sched: np.ndarray, chunk_indptr: np.ndarray, out_indptr: np.ndarray) -> BoundCall:
    """fs_build_prefill_worklist into caller-held arrays (e.g. views of pinned memory); the inputs are read
    from the given arrays at every call.  After a call the counts are in .n_items.value, .n_pairs.value
    and .n_tiles.value; a list that outgrows the arrays raises FsError (FS_ECAPACITY)."""
    lib = load_library()
    for a in (n_done, n_new, owner, sched):
        if a.dtype != np.int32 or not a.flags.c_contiguous:
            raise TypeError("bind_build_prefill_worklist needs contiguous int32 n_done, n_new, owner and sched")
    for a in (chunk_indptr, out_indptr):
        if a.dtype != np.int64 or not a.flags.c_contiguous:
            raise TypeError("bind_build_prefill_worklist needs contiguous int64 chunk_indptr and out_indptr")
    if items.dtype != PREFILL_ITEM_DTYPE or pairs.dtype != PREFILL_PAIR_DTYPE or len(sched) != len(items):
        raise TypeError("bind_build_prefill_worklist: items, pairs and sched do not match the documented layouts")
    if len(out_indptr) != len(pairs) + 1 or len(chunk_indptr) < 1:
        raise ValueError("bind_build_prefill_worklist: out_indptr needs len(pairs)+1 entries, chunk_indptr at least one")
    i32p = C.POINTER(C.c_int32)
    n_items, n_pairs, n_tiles = C.c_int64(0), C.c_int64(0), C.c_int64(0)
    args = (C.byref(shape), n_done.ctypes.data_as(i32p), n_new.ctypes.data_as(i32p), owner.ctypes.data_as(i32p),
            C.c_int32(rank), C.c_int32(tile_tokens), C.c_int32(kv_chunk_tokens),
            C.c_void_p(items.ctypes.data), C.c_int64(len(items)), C.c_void_p(pairs.ctypes.data), C.c_int64(len(pairs)),
            C.c_void_p(sched.ctypes.data), C.c_void_p(chunk_indptr.ctypes.data), C.c_int64(len(chunk_indptr) - 1),
            C.c_void_p(out_indptr.ctypes.data), C.byref(n_items), C.byref(n_pairs), C.byref(n_tiles))
    return BoundCall(lib.fs_build_prefill_worklist, args,
                     (shape, n_done, n_new, owner, items, pairs, sched, chunk_indptr, out_indptr), n_items, n_pairs, n_tiles)


def bind_choose_prefill_chunk(shape: FsShape, n_done: np.ndarray, n_new: np.ndarray, owner: np.ndarray, rank: int,
                              tile_tokens: int, max_chunk: int, min_chunk: int, n_slots: int) -> BoundCall:
    """fs_choose_prefill_chunk on caller-held int32 arrays, read at every call.  After a call the chunk is in
    .n_tiles.value and the list's length in .n_items.value."""
    lib = load_library()
    for a in (n_done, n_new, owner):
        if a.dtype != np.int32 or not a.flags.c_contiguous:
            raise TypeError("bind_choose_prefill_chunk needs contiguous int32 n_done, n_new and owner")
    i32p = C.POINTER(C.c_int32)
    chunk, n_items = C.c_int32(0), C.c_int64(0)
    args = (C.byref(shape), n_done.ctypes.data_as(i32p), n_new.ctypes.data_as(i32p), owner.ctypes.data_as(i32p),
            C.c_int32(rank), C.c_int32(tile_tokens), C.c_int32(max_chunk), C.c_int32(min_chunk), C.c_int64(n_slots),
            C.byref(chunk), C.byref(n_items))
    return BoundCall(lib.fs_choose_prefill_chunk, args, (shape, n_done, n_new, owner), n_items, None, chunk)


def bind_decode_attention(shape: FsShape, kv: FsKvView, items_dev, sched_dev, n_items: int,
                          part_o, part_lse, stream=None) -> BoundCall:
    lib = load_library()
    args = (C.byref(shape), C.byref(kv), _vp(items_dev), _vp(sched_dev), C.c_int64(n_items),
            _vp(part_o), _vp(part_lse), _vp(stream))
    return BoundCall(lib.fs_decode_attention, args, (shape, kv, items_dev, sched_dev, part_o, part_lse))


def bind_decode_attention_persistent(shape: FsShape, kv: FsKvView, items_dev, sched_dev, n_items: int, claim_dev,
                                     part_o, part_lse, stream=None) -> BoundCall:
    lib = load_library()
    args = (C.byref(shape), C.byref(kv), _vp(items_dev), _vp(sched_dev), C.c_int64(n_items), _vp(claim_dev),
            _vp(part_o), _vp(part_lse), _vp(stream))
    return BoundCall(lib.fs_decode_attention_persistent, args, (shape, kv, items_dev, sched_dev, claim_dev, part_o, part_lse))


def bind_decode_attention_fused(shape: FsShape, kv: FsKvView, items_dev, sched_dev, n_items: int, chunk_indptr_dev,
                                n_pairs: int, part_o, part_lse, claim_dev, out, lse, stream=None) -> BoundCall:
    lib = load_library()
    args = (C.byref(shape), C.byref(kv), _vp(items_dev), _vp(sched_dev), C.c_int64(n_items), _vp(chunk_indptr_dev),
            C.c_int64(n_pairs), _vp(part_o), _vp(part_lse), _vp(claim_dev), _vp(out), _vp(lse), _vp(stream))
    return BoundCall(lib.fs_decode_attention_fused, args,
                     (shape, kv, items_dev, sched_dev, chunk_indptr_dev, part_o, part_lse, claim_dev, out, lse))


def bind_decode_attention_units(shape: FsShape, kv: FsKvView, items_dev, n_items: int, unit_indptr_dev, n_units: int,
                                chunk_indptr_dev, n_pairs: int, part_o, part_lse, out, lse, stream=None) -> BoundCall:
    lib = load_library()
    args = (C.byref(shape), C.byref(kv), _vp(items_dev), C.c_int64(n_items), _vp(unit_indptr_dev), C.c_int64(n_units),
            _vp(chunk_indptr_dev), C.c_int64(n_pairs), _vp(part_o), _vp(part_lse), _vp(out), _vp(lse), _vp(stream))
    return BoundCall(lib.fs_decode_attention_units, args,
                     (shape, kv, items_dev, unit_indptr_dev, chunk_indptr_dev, part_o, part_lse, out, lse))


def bind_build_launch_records(shape: FsShape, items: np.ndarray, order, chunk_indptr: np.ndarray, n_pairs: int,
                              page_indptr: np.ndarray, page_ids: np.ndarray, records: np.ndarray,
                              direct_rows: bool = True) -> BoundCall:
    """fs_build_launch_records on caller-held arrays (items and records e.g. views of pinned memory); reads all of
    ``items`` (its length is the item count)."""
    lib = load_library()
    if items.dtype != ITEM_DTYPE or records.dtype != RECORD_DTYPE or len(records) < len(items):
        raise TypeError("bind_build_launch_records: items / records do not match the documented layouts")
    args = (C.byref(shape), C.c_void_p(items.ctypes.data), None if order is None else C.c_void_p(order.ctypes.data),
            C.c_int64(len(items)), C.c_void_p(chunk_indptr.ctypes.data), C.c_int64(n_pairs),
            C.c_void_p(page_indptr.ctypes.data), C.c_void_p(page_ids.ctypes.data), C.c_int64(len(page_ids)),
            C.c_int32(int(bool(direct_rows))), C.c_void_p(records.ctypes.data))
    return BoundCall(lib.fs_build_launch_records, args, (shape, items, order, chunk_indptr, page_indptr, page_ids, records))


def bind_decode_attention_records(shape: FsShape, kv: FsKvView, records_dev, n_items: int, unit_indptr_dev, n_units: int,
                                  chunk_indptr_dev, n_pairs: int, part_o, part_lse, out, lse, pair_counters_dev=None,
                                  claim_dev=None, stream=None) -> BoundCall:
    lib = load_library()
    args = (C.byref(shape), C.byref(kv), _vp(records_dev), C.c_int64(n_items), _vp(unit_indptr_dev), C.c_int64(n_units),
            _vp(chunk_indptr_dev), C.c_int64(n_pairs), _vp(part_o), _vp(part_lse), _vp(out), _vp(lse),
            _vp(pair_counters_dev), _vp(claim_dev), _vp(stream))
    return BoundCall(lib.fs_decode_attention_records, args,
                     (shape, kv, records_dev, unit_indptr_dev, chunk_indptr_dev, part_o, part_lse, out, lse, pair_counters_dev,
                      claim_dev))


def bind_merge_lse(part_o, part_lse, chunk_indptr_dev, n_pairs: int, group: int, head_dim: int,
                   out, lse, stream=None) -> BoundCall:
    lib = load_library()
    args = (_vp(part_o), _vp(part_lse), _vp(chunk_indptr_dev), C.c_int64(n_pairs), C.c_int32(group),
            C.c_int32(head_dim), _vp(out), _vp(lse), _vp(stream))
    return BoundCall(lib.fs_merge_lse, args, (part_o, part_lse, chunk_indptr_dev, out, lse))


def fs_set_option(key: str, value: int) -> None:
    _check(load_library().fs_set_option(key.encode(), value))


def fs_get_option(key: str) -> int:
    return load_library().fs_get_option(key.encode())
