"""ctypes binding of include/linr.h -- argument marshalling only.

The functions carry the names of the C entry points (without the `linr_` prefix) and
take torch tensors (device memory) or numpy arrays (host memory); `Index` is a small
convenience wrapper that allocates outputs and workspace with torch.  If the HIP
library has not been built, loading fails loudly: nothing here computes on the CPU.
"""
from __future__ import annotations

import ctypes as C
import os
import numpy as np

F32, BF16, I8, BITS = 0, 1, 2, 3
NO_ID = 0xFFFFFFFF
MAX_K = 8192
MAX_M = 8
NOALLOC_SCRATCH_BYTES = 64 << 20       # fixed scratch of linr_search_filtered_noalloc
SRC_HOST, SRC_DEVICE_COPY, SRC_DEVICE_BORROW = 0, 1, 2
FILTERS_ON_DEVICE, FILTERS_ON_HOST = 0, 1
PLAN_MASKING, PLAN_PREFILTER = 2, 4          # flags of search_filtered: force a strategy
STRATEGY_MASKING, STRATEGY_PREFILTER = 0, 1
MAX_STAGES = 160
STAGE_NAMES = {0: "init", 1: "scan", 2: "merge", 3: "filter"}

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liblinr.so")
_lib = None

#: every symbol include/linr.h declares
EXPORTS = [
    "linr_index_create", "linr_index_load_fp32", "linr_index_load_bf16", "linr_index_load_int8",
    "linr_search_workspace_bytes", "linr_search_filtered", "linr_index_destroy", "linr_index_info",
    "linr_strerror", "linr_last_hip_error", "linr_set_tuning", "linr_search_filtered_timed",
    "linr_events_create", "linr_events_destroy", "linr_events_elapsed_ms",
    "linr_index_build_bits", "linr_index_load_bits", "linr_quantize_queries", "linr_search_bits_workspace_bytes",
    "linr_search_bits", "linr_select_bits_workspace_bytes", "linr_select_bits", "linr_search_two_stage_workspace_bytes", "linr_search_two_stage", "linr_search_bits_timed",
    "linr_index_enable_updates", "linr_index_upsert", "linr_index_delete", "linr_index_sync_updates",
    "linr_index_load_clauses", "linr_search_clauses_workspace_bytes", "linr_search_clauses", "linr_search_clauses_timed",
    "linr_search_clauses_prefilter", "linr_index_upsert_clauses",
    "linr_search_prefilter_workspace_bytes", "linr_search_filtered_prefilter", "linr_search_filtered_noalloc",
    "linr_plan_filtered", "linr_index_build_bits_rep",
]


class LinrError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = strerror(code)
        if code == -8:
            msg += f" (hipError_t {load_library().linr_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{code}]")


class Tuning(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in ("sample_ratio", "min_sample", "blocks_per_cu", "max_levels",
                                          "force_generic", "max_qg", "no_coop", "coop_min_groups",
                                          "no_top_split", "prefilter_phases", "wide_min_batch", "two_stage_rank_max",
                                          "no_dense", "dense_min_batch", "dense_groups", "top_ratios",
                                          "prefilter_table_min", "select_seg_items")]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """dlopen the in-tree HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it first (python paper_2407_13218_amd/build.py "
                          "or __graft_entry__.build()); there is no fallback path")
    lib = C.CDLL(_LIB_PATH)
    vp, u64, u32, i32 = C.c_void_p, C.c_uint64, C.c_uint32, C.c_int
    lib.linr_index_create.restype = i32
    lib.linr_index_create.argtypes = [C.POINTER(vp), u64, u32, i32, i32]
    for name in ("linr_index_load_fp32", "linr_index_load_bf16"):
        f = getattr(lib, name); f.restype = i32; f.argtypes = [vp, vp, vp, vp, u64, i32]
    lib.linr_index_load_int8.restype = i32
    lib.linr_index_load_int8.argtypes = [vp, vp, vp, vp, vp, u64, i32]
    lib.linr_search_workspace_bytes.restype = i32
    lib.linr_search_workspace_bytes.argtypes = [vp, u32, u32, u32, C.POINTER(u64)]
    sargs = [vp, vp, vp, u32, u32, vp, u32, vp, vp, vp, vp, vp, u64, vp, u32]
    lib.linr_search_filtered.restype = i32
    lib.linr_search_filtered.argtypes = sargs
    lib.linr_plan_filtered.restype = i32
    lib.linr_plan_filtered.argtypes = [vp, vp, u32, u32, u32, C.POINTER(C.c_int), C.POINTER(C.c_double)]
    lib.linr_search_prefilter_workspace_bytes.restype = i32
    lib.linr_search_prefilter_workspace_bytes.argtypes = [vp, u32, u32, u32, C.POINTER(u64)]
    lib.linr_search_filtered_prefilter.restype = i32
    lib.linr_search_filtered_prefilter.argtypes = sargs
    lib.linr_search_filtered_noalloc.restype = i32
    lib.linr_search_filtered_noalloc.argtypes = sargs[:11] + sargs[13:]
    lib.linr_search_filtered_timed.restype = i32
    lib.linr_search_filtered_timed.argtypes = sargs + [vp, C.POINTER(u32), vp, vp]
    lib.linr_index_destroy.restype = i32
    lib.linr_index_destroy.argtypes = [vp]
    lib.linr_index_info.restype = i32
    lib.linr_index_info.argtypes = [vp, C.POINTER(u64), C.POINTER(u32), C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
    lib.linr_strerror.restype = C.c_char_p
    lib.linr_strerror.argtypes = [i32]
    lib.linr_last_hip_error.restype = i32
    lib.linr_last_hip_error.argtypes = []
    lib.linr_set_tuning.restype = i32
    lib.linr_set_tuning.argtypes = [vp]
    lib.linr_events_create.restype = i32
    lib.linr_events_create.argtypes = [vp, u32]
    lib.linr_events_destroy.restype = i32
    lib.linr_events_destroy.argtypes = [vp, u32]
    lib.linr_events_elapsed_ms.restype = i32
    lib.linr_events_elapsed_ms.argtypes = [vp, u32, vp]
    lib.linr_index_build_bits.restype = i32
    lib.linr_index_build_bits.argtypes = [vp, vp, vp, u32, i32]
    lib.linr_index_build_bits_rep.restype = i32
    lib.linr_index_build_bits_rep.argtypes = [vp, vp, vp, u32, u32, i32]
    lib.linr_index_load_bits.restype = i32
    lib.linr_index_load_bits.argtypes = [vp, vp, vp, vp, u64, i32]
    lib.linr_quantize_queries.restype = i32
    lib.linr_quantize_queries.argtypes = [vp, vp, u32, vp, vp]
    lib.linr_search_bits_workspace_bytes.restype = i32
    lib.linr_search_bits_workspace_bytes.argtypes = [vp, u32, u32, C.POINTER(u64)]
    lib.linr_search_bits.restype = i32
    lib.linr_search_bits.argtypes = [vp, vp, u32, vp, u32, vp, vp, vp, vp, u64, vp, u32]
    lib.linr_select_bits_workspace_bytes.restype = i32
    lib.linr_select_bits_workspace_bytes.argtypes = [vp, u32, C.POINTER(u64)]
    lib.linr_select_bits.restype = i32
    lib.linr_select_bits.argtypes = [vp, vp, u32, vp, u64, vp, vp, vp, vp, u64, vp, u32]
    lib.linr_index_load_clauses.restype = i32
    lib.linr_index_load_clauses.argtypes = [vp, vp, vp, u32, u32, u32, u64, i32]
    lib.linr_index_upsert_clauses.restype = i32
    lib.linr_index_upsert_clauses.argtypes = [vp, vp, u32, vp, vp, i32, vp]
    lib.linr_search_clauses_workspace_bytes.restype = i32
    lib.linr_search_clauses_workspace_bytes.argtypes = [vp, u32, u32, u32, C.POINTER(u64)]
    lib.linr_search_clauses.restype = i32
    lib.linr_search_clauses.argtypes = [vp, vp, vp, u32, u32, vp, vp, u32, u32, vp, vp, vp, vp, vp, u64, vp]
    lib.linr_search_clauses_prefilter.restype = i32
    lib.linr_search_clauses_prefilter.argtypes = lib.linr_search_clauses.argtypes
    lib.linr_search_clauses_timed.restype = i32
    lib.linr_search_clauses_timed.argtypes = lib.linr_search_clauses.argtypes + [vp, C.POINTER(u32), vp, vp]
    lib.linr_index_enable_updates.restype = i32
    lib.linr_index_enable_updates.argtypes = [vp]
    lib.linr_index_upsert.restype = i32
    lib.linr_index_upsert.argtypes = [vp, vp, u32, vp, vp, vp, vp, i32, vp]
    lib.linr_index_delete.restype = i32
    lib.linr_index_delete.argtypes = [vp, vp, u32, vp]
    lib.linr_index_sync_updates.restype = i32
    lib.linr_index_sync_updates.argtypes = [vp]
    lib.linr_search_bits_timed.restype = i32
    lib.linr_search_bits_timed.argtypes = lib.linr_search_bits.argtypes + [vp, C.POINTER(u32), vp, vp]
    lib.linr_search_two_stage_workspace_bytes.restype = i32
    lib.linr_search_two_stage_workspace_bytes.argtypes = [vp, u32, u32, u32, C.POINTER(u64)]
    lib.linr_search_two_stage.restype = i32
    lib.linr_search_two_stage.argtypes = [vp, vp, u32, vp, u32, u32, vp, vp, vp, vp, u64, vp, u32]
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load_library().linr_strerror(code).decode()


def _ptr(x):
    """address of a torch tensor (device or host), a numpy array, or None"""
    if x is None:
        return None
    if isinstance(x, np.ndarray):
        if not x.flags["C_CONTIGUOUS"]:
            raise ValueError("numpy argument must be C-contiguous")
        return x.ctypes.data
    if hasattr(x, "data_ptr"):
        if not x.is_contiguous():
            raise ValueError("tensor argument must be contiguous")
        return x.data_ptr()
    if isinstance(x, int):
        return x
    raise TypeError(type(x))


def _check(rc: int, where: str):
    if rc != 0:
        raise LinrError(rc, where)


def index_create(capacity: int, d: int, dtype: int, device: int = 0) -> int:
    h = C.c_void_p()
    _check(load_library().linr_index_create(C.byref(h), capacity, d, dtype, device), "linr_index_create")
    return h.value


def index_load_fp32(ix, emb, mask, ts, n, src):
    _check(load_library().linr_index_load_fp32(ix, _ptr(emb), _ptr(mask), _ptr(ts), n, src), "linr_index_load_fp32")


def index_load_bf16(ix, emb, mask, ts, n, src):
    _check(load_library().linr_index_load_bf16(ix, _ptr(emb), _ptr(mask), _ptr(ts), n, src), "linr_index_load_bf16")


def index_load_int8(ix, emb, row_scale, mask, ts, n, src):
    _check(load_library().linr_index_load_int8(ix, _ptr(emb), _ptr(row_scale), _ptr(mask), _ptr(ts), n, src),
           "linr_index_load_int8")


def index_info(ix):
    n, d = C.c_uint64(), C.c_uint32()
    dt, hts, hrs = C.c_int(), C.c_int(), C.c_int()
    _check(load_library().linr_index_info(ix, C.byref(n), C.byref(d), C.byref(dt), C.byref(hts), C.byref(hrs)), "linr_index_info")
    return dict(n=n.value, d=d.value, dtype=dt.value, has_ts=bool(hts.value), has_row_scale=bool(hrs.value))


def index_destroy(ix):
    _check(load_library().linr_index_destroy(ix), "linr_index_destroy")


def search_workspace_bytes(ix, B, m, k) -> int:
    out = C.c_uint64()
    _check(load_library().linr_search_workspace_bytes(ix, B, m, k, C.byref(out)), "linr_search_workspace_bytes")
    return out.value


def search_filtered(ix, Q, q_scale, B, m, filters, k, out_ids, out_scores, out_raw, out_counts,
                    workspace, workspace_bytes, stream=0, flags=FILTERS_ON_DEVICE):
    _check(load_library().linr_search_filtered(ix, _ptr(Q), _ptr(q_scale), B, m, _ptr(filters), k, _ptr(out_ids),
                                               _ptr(out_scores), _ptr(out_raw), _ptr(out_counts), _ptr(workspace),
                                               workspace_bytes, stream, flags), "linr_search_filtered")


def plan_filtered(ix, host_filters, B, m, k):
    """the planner's choice for these (host, numpy) filters: (STRATEGY_*, estimated feasible (item, query) pairs)"""
    strategy = C.c_int()
    pairs = C.c_double()
    _check(load_library().linr_plan_filtered(ix, _ptr(host_filters), B, m, k, C.byref(strategy), C.byref(pairs)), "linr_plan_filtered")
    return strategy.value, pairs.value


def search_filtered_noalloc(ix, Q, q_scale, B, m, filters, k, out_ids, out_scores, out_raw, out_counts, stream=0,
                            flags=FILTERS_ON_DEVICE):
    """linr_search_filtered without a workspace argument: the library's fixed scratch array serves (callers that cannot allocate)"""
    _check(load_library().linr_search_filtered_noalloc(ix, _ptr(Q), _ptr(q_scale), B, m, _ptr(filters), k, _ptr(out_ids),
                                                       _ptr(out_scores), _ptr(out_raw), _ptr(out_counts), stream, flags),
           "linr_search_filtered_noalloc")


def search_prefilter_workspace_bytes(ix, B, m, k) -> int:
    out = C.c_uint64()
    _check(load_library().linr_search_prefilter_workspace_bytes(ix, B, m, k, C.byref(out)), "linr_search_prefilter_workspace_bytes")
    return out.value


def search_filtered_prefilter(ix, Q, q_scale, B, m, filters, k, out_ids, out_scores, out_raw, out_counts,
                              workspace, workspace_bytes, stream=0, flags=FILTERS_ON_DEVICE):
    _check(load_library().linr_search_filtered_prefilter(ix, _ptr(Q), _ptr(q_scale), B, m, _ptr(filters), k, _ptr(out_ids),
                                                         _ptr(out_scores), _ptr(out_raw), _ptr(out_counts), _ptr(workspace),
                                                         workspace_bytes, stream, flags), "linr_search_filtered_prefilter")


def search_filtered_timed(ix, Q, q_scale, B, m, filters, k, out_ids, out_scores, out_raw, out_counts,
                          workspace, workspace_bytes, stream, flags, events):
    """`events`: ctypes array of 2*MAX_STAGES hipEvent_t.  Returns (kinds, items) per stage."""
    ns = C.c_uint32()
    kinds = (C.c_uint32 * MAX_STAGES)()
    items = (C.c_uint64 * MAX_STAGES)()
    _check(load_library().linr_search_filtered_timed(ix, _ptr(Q), _ptr(q_scale), B, m, _ptr(filters), k, _ptr(out_ids),
                                                     _ptr(out_scores), _ptr(out_raw), _ptr(out_counts), _ptr(workspace),
                                                     workspace_bytes, stream, flags, C.addressof(events), C.byref(ns),
                                                     C.addressof(kinds), C.addressof(items)),
           "linr_search_filtered_timed")
    return [kinds[i] for i in range(ns.value)], [items[i] for i in range(ns.value)]


def events_create(n: int):
    """ctypes array of n hipEvent_t"""
    ev = (C.c_void_p * n)()
    _check(load_library().linr_events_create(C.addressof(ev), n), "linr_events_create")
    return ev


def events_destroy(ev):
    _check(load_library().linr_events_destroy(C.addressof(ev), len(ev)), "linr_events_destroy")


def events_elapsed_ms(ev, n_pairs: int):
    ms = (C.c_float * n_pairs)()
    _check(load_library().linr_events_elapsed_ms(C.addressof(ev), n_pairs, C.addressof(ms)), "linr_events_elapsed_ms")
    return [ms[i] for i in range(n_pairs)]


def index_build_bits(ix, perm, signs, k_bits, src, reps=1):
    if reps == 1:
        _check(load_library().linr_index_build_bits(ix, _ptr(perm), _ptr(signs), k_bits, src), "linr_index_build_bits")
    else:
        _check(load_library().linr_index_build_bits_rep(ix, _ptr(perm), _ptr(signs), k_bits, reps, src), "linr_index_build_bits_rep")


def index_load_bits(ix, bits, mask, ts, n, src):
    _check(load_library().linr_index_load_bits(ix, _ptr(bits), _ptr(mask), _ptr(ts), n, src), "linr_index_load_bits")


def quantize_queries(ix, Q, B, qbits, stream=0):
    _check(load_library().linr_quantize_queries(ix, _ptr(Q), B, _ptr(qbits), stream), "linr_quantize_queries")


def search_bits_workspace_bytes(ix, B, T) -> int:
    out = C.c_uint64()
    _check(load_library().linr_search_bits_workspace_bytes(ix, B, T, C.byref(out)), "linr_search_bits_workspace_bytes")
    return out.value


def search_bits(ix, qbits, B, filters, T, out_ids, out_matches, out_counts, workspace, workspace_bytes, stream=0,
                flags=FILTERS_ON_DEVICE):
    _check(load_library().linr_search_bits(ix, _ptr(qbits), B, _ptr(filters), T, _ptr(out_ids), _ptr(out_matches),
                                           _ptr(out_counts), _ptr(workspace), workspace_bytes, stream, flags), "linr_search_bits")


def search_bits_timed(ix, qbits, B, filters, T, out_ids, out_matches, out_counts, workspace, workspace_bytes, stream, flags,
                      events):
    """As search_bits, recording `events` (2*MAX_STAGES hipEvent_t) around each launch.  Returns (kinds, items) per stage."""
    ns = C.c_uint32()
    kinds = (C.c_uint32 * MAX_STAGES)()
    items = (C.c_uint64 * MAX_STAGES)()
    _check(load_library().linr_search_bits_timed(ix, _ptr(qbits), B, _ptr(filters), T, _ptr(out_ids), _ptr(out_matches),
                                                 _ptr(out_counts), _ptr(workspace), workspace_bytes, stream, flags,
                                                 C.addressof(events), C.byref(ns), C.addressof(kinds), C.addressof(items)),
           "linr_search_bits_timed")
    return [kinds[i] for i in range(ns.value)], [items[i] for i in range(ns.value)]


def select_bits_workspace_bytes(ix, B) -> int:
    out = C.c_uint64()
    _check(load_library().linr_select_bits_workspace_bytes(ix, B, C.byref(out)), "linr_select_bits_workspace_bytes")
    return out.value


def select_bits(ix, qbits, B, filters, K, out_ids, out_counts, out_thresholds, workspace, workspace_bytes, stream=0,
                flags=FILTERS_ON_DEVICE):
    _check(load_library().linr_select_bits(ix, _ptr(qbits), B, _ptr(filters), K, _ptr(out_ids), _ptr(out_counts),
                                           _ptr(out_thresholds), _ptr(workspace), workspace_bytes, stream, flags),
           "linr_select_bits")


def search_two_stage_workspace_bytes(ix, B, T, k) -> int:
    out = C.c_uint64()
    _check(load_library().linr_search_two_stage_workspace_bytes(ix, B, T, k, C.byref(out)),
           "linr_search_two_stage_workspace_bytes")
    return out.value


def search_two_stage(ix, Q, B, filters, T, k, out_ids, out_scores, out_counts, workspace, workspace_bytes, stream=0,
                     flags=FILTERS_ON_DEVICE):
    _check(load_library().linr_search_two_stage(ix, _ptr(Q), B, _ptr(filters), T, k, _ptr(out_ids), _ptr(out_scores),
                                                _ptr(out_counts), _ptr(workspace), workspace_bytes, stream, flags),
           "linr_search_two_stage")


def index_load_clauses(ix, values, counts, n_clauses, row_width, reverse, n, src):
    _check(load_library().linr_index_load_clauses(ix, _ptr(values), _ptr(counts), n_clauses, row_width, reverse, n, src),
           "linr_index_load_clauses")


def index_upsert_clauses(ix, slots, values, counts, src, stream=0):
    slots = np.ascontiguousarray(slots, dtype=np.uint32)
    _check(load_library().linr_index_upsert_clauses(ix, _ptr(slots), slots.size, _ptr(values), _ptr(counts), src, stream),
           "linr_index_upsert_clauses")


def search_clauses_workspace_bytes(ix, B, m, k) -> int:
    out = C.c_uint64()
    _check(load_library().linr_search_clauses_workspace_bytes(ix, B, m, k, C.byref(out)), "linr_search_clauses_workspace_bytes")
    return out.value


def search_clauses(ix, Q, q_scale, B, m, q_values, q_counts, q_width, k, out_ids, out_scores, out_raw, out_counts,
                   workspace, workspace_bytes, stream=0):
    _check(load_library().linr_search_clauses(ix, _ptr(Q), _ptr(q_scale), B, m, _ptr(q_values), _ptr(q_counts), q_width, k,
                                              _ptr(out_ids), _ptr(out_scores), _ptr(out_raw), _ptr(out_counts),
                                              _ptr(workspace), workspace_bytes, stream), "linr_search_clauses")


def search_clauses_prefilter(ix, Q, q_scale, B, m, q_values, q_counts, q_width, k, out_ids, out_scores, out_raw, out_counts,
                             workspace, workspace_bytes, stream=0):
    _check(load_library().linr_search_clauses_prefilter(ix, _ptr(Q), _ptr(q_scale), B, m, _ptr(q_values), _ptr(q_counts), q_width,
                                                        k, _ptr(out_ids), _ptr(out_scores), _ptr(out_raw), _ptr(out_counts),
                                                        _ptr(workspace), workspace_bytes, stream), "linr_search_clauses_prefilter")


def search_clauses_timed(ix, Q, q_scale, B, m, q_values, q_counts, q_width, k, out_ids, out_scores, out_raw, out_counts,
                         workspace, workspace_bytes, stream, events):
    """As search_clauses, recording `events` around each launch.  Returns (kinds, items) per stage."""
    ns = C.c_uint32()
    kinds = (C.c_uint32 * MAX_STAGES)()
    items = (C.c_uint64 * MAX_STAGES)()
    _check(load_library().linr_search_clauses_timed(ix, _ptr(Q), _ptr(q_scale), B, m, _ptr(q_values), _ptr(q_counts), q_width,
                                                    k, _ptr(out_ids), _ptr(out_scores), _ptr(out_raw), _ptr(out_counts),
                                                    _ptr(workspace), workspace_bytes, stream, C.addressof(events),
                                                    C.byref(ns), C.addressof(kinds), C.addressof(items)),
           "linr_search_clauses_timed")
    return [kinds[i] for i in range(ns.value)], [items[i] for i in range(ns.value)]


def index_enable_updates(ix):
    _check(load_library().linr_index_enable_updates(ix), "linr_index_enable_updates")


def index_upsert(ix, slots, emb, row_scale, mask, ts, src, stream=0):
    """slots: numpy uint32 (host).  emb / row_scale / mask / ts: numpy (src = SRC_HOST) or device tensors."""
    slots = np.ascontiguousarray(slots, dtype=np.uint32)
    _check(load_library().linr_index_upsert(ix, _ptr(slots), slots.size, _ptr(emb), _ptr(row_scale), _ptr(mask), _ptr(ts),
                                            src, stream), "linr_index_upsert")


def index_delete(ix, slots, stream=0):
    slots = np.ascontiguousarray(slots, dtype=np.uint32)
    _check(load_library().linr_index_delete(ix, _ptr(slots), slots.size, stream), "linr_index_delete")


def index_sync_updates(ix):
    _check(load_library().linr_index_sync_updates(ix), "linr_index_sync_updates")


def set_tuning(**kw):
    """set_tuning() restores the defaults."""
    lib = load_library()
    if not kw:
        _check(lib.linr_set_tuning(None), "linr_set_tuning")
        return
    t = Tuning()
    for key, v in kw.items():
        setattr(t, key, int(v))
    _check(lib.linr_set_tuning(C.addressof(t)), "linr_set_tuning")


class Index:
    """Owns a linr_index handle; torch provides device memory and the stream."""

    def __init__(self, capacity: int, d: int, dtype: int, device: int = 0):
        self.handle = index_create(capacity, d, dtype, device)
        self.dtype, self.d, self.device = dtype, d, device
        self.k_bits = d if dtype == BITS else 0
        self._keep = None

    def load(self, emb, mask, ts=None, row_scale=None, src=None):
        host = isinstance(emb, np.ndarray)
        if src is None:
            src = SRC_HOST if host else SRC_DEVICE_BORROW
        n = emb.shape[0]
        if self.dtype == F32:
            index_load_fp32(self.handle, emb, mask, ts, n, src)
        elif self.dtype == BF16:
            index_load_bf16(self.handle, emb, mask, ts, n, src)
        elif self.dtype == BITS:
            index_load_bits(self.handle, emb, mask, ts, n, src)              # `emb` = codes [n, W] (int64 bit patterns)
        else:
            index_load_int8(self.handle, emb, row_scale, mask, ts, n, src)
        self._keep = (emb, mask, ts, row_scale) if src == SRC_DEVICE_BORROW else None
        self.n = n
        return self

    def workspace_bytes(self, B, m, k):
        return search_workspace_bytes(self.handle, B, m, k)

    def planned_workspace_bytes(self, B, m, k):
        """enough for either strategy of search_filtered (masking or explicit pre-filtering)"""
        return max(search_workspace_bytes(self.handle, B, m, k), search_prefilter_workspace_bytes(self.handle, B, m, k))

    # clause lists ------------------------------------------------------------------------------------------
    def load_clauses(self, values, counts, reverse=0):
        """values [n, row_width] (uint64 / int64 bit patterns), counts [n, n_clauses] uint8; numpy or device tensors"""
        host = isinstance(values, np.ndarray)
        n, width = values.shape
        self.n_clauses = counts.shape[1]
        index_load_clauses(self.handle, values, counts, self.n_clauses, width, reverse, n, SRC_HOST if host else SRC_DEVICE_COPY)
        return self

    def search_clauses(self, Q, q_values, q_counts, k, q_scale=None, want_raw=True, prefilter=False):
        """Q device [B, m, d]; q_values device [B, q_width] int64; q_counts device [B, n_clauses] uint8;
        prefilter=True: the explicit pre-filtering strategy (linr_search_clauses_prefilter)"""
        import torch
        if Q.dim() == 2:
            Q = Q.unsqueeze(1)
        Q = Q.contiguous()
        B, m, dev = Q.shape[0], Q.shape[1], Q.device
        ids = torch.empty((B, k), dtype=torch.int32, device=dev)
        sc = torch.empty((B, k), dtype=torch.float32, device=dev)
        raw = torch.empty((B, k), dtype=torch.int32, device=dev) if want_raw else None
        cnt = torch.empty((B,), dtype=torch.int32, device=dev)
        if B == 0:
            return ids, sc, raw, cnt
        nbytes = search_clauses_workspace_bytes(self.handle, B, m, k)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        fn = search_clauses_prefilter if prefilter else search_clauses
        fn(self.handle, Q, q_scale, B, m, q_values.contiguous(), q_counts.contiguous(), q_values.shape[1], k,
           ids, sc, raw, cnt, ws, nbytes, torch.cuda.current_stream(dev).cuda_stream)
        self._last_workspace = ws
        return ids, sc, raw, cnt

    # live updates ------------------------------------------------------------------------------------------
    def enable_updates(self):
        index_enable_updates(self.handle)
        return self

    def upsert(self, slots, emb, mask, ts=None, row_scale=None, stream=None):
        """slots: host integers; the rest numpy (copied before the call returns) or device tensors"""
        import torch
        host = isinstance(emb, np.ndarray)
        if stream is None:
            stream = torch.cuda.current_stream(self.device).cuda_stream
        index_upsert(self.handle, slots, emb, row_scale, mask, ts, SRC_HOST if host else SRC_DEVICE_COPY, stream)
        if not host:
            self._keep_update = (emb, mask, ts, row_scale)       # device sources are read when the stream gets there

    def upsert_clauses(self, slots, values, counts, stream=None):
        import torch
        host = isinstance(values, np.ndarray)
        if stream is None:
            stream = torch.cuda.current_stream(self.device).cuda_stream
        index_upsert_clauses(self.handle, slots, values, counts, SRC_HOST if host else SRC_DEVICE_COPY, stream)
        if not host:
            self._keep_clause_update = (values, counts)

    def delete(self, slots, stream=None):
        import torch
        if stream is None:
            stream = torch.cuda.current_stream(self.device).cuda_stream
        index_delete(self.handle, slots, stream)

    def sync_updates(self):
        index_sync_updates(self.handle)

    def info(self):
        return index_info(self.handle)

    def search(self, Q, filters, k, q_scale=None, workspace=None, want_raw=True, prefilter=False, strategy="auto"):
        """Q: device tensor [B, m, d] (or [B, d]); filters: numpy records (host) or a device uint8/int32
        tensor of B*40 bytes.  Returns device tensors ids (int32 bits of uint32), scores, raw, counts.
        strategy: "auto" (the library's planner decides where it can: host filters), "masking" or "prefilter"
        (forced through the flags of linr_search_filtered).  prefilter=True: call linr_search_filtered_prefilter itself."""
        import torch
        if Q.dim() == 2:
            Q = Q.unsqueeze(1)
        Q = Q.contiguous()
        B, m, d = Q.shape
        assert d == self.d
        dev = Q.device
        ids = torch.empty((B, k), dtype=torch.int32, device=dev)
        scores = torch.empty((B, k), dtype=torch.float32, device=dev)
        raw = torch.empty((B, k), dtype=torch.int32, device=dev) if (want_raw and self.dtype == I8) else None
        counts = torch.empty((B,), dtype=torch.int32, device=dev)
        if B == 0:
            return ids, scores, raw, counts
        plan_flag = {"auto": 0, "masking": PLAN_MASKING, "prefilter": PLAN_PREFILTER}[strategy]
        if prefilter:
            nbytes = search_prefilter_workspace_bytes(self.handle, B, m, k)
        elif strategy == "masking":
            nbytes = self.workspace_bytes(B, m, k)
        else:
            nbytes = self.planned_workspace_bytes(B, m, k)
        if workspace is None or workspace.numel() < nbytes:
            workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        if isinstance(filters, np.ndarray):
            flags, f = FILTERS_ON_HOST, np.ascontiguousarray(filters)
        else:
            flags, f = FILTERS_ON_DEVICE, filters
        stream = torch.cuda.current_stream(dev).cuda_stream
        if prefilter:
            search_filtered_prefilter(self.handle, Q, q_scale, B, m, f, k, ids, scores, raw, counts, workspace, workspace.numel(), stream, flags)
        else:
            search_filtered(self.handle, Q, q_scale, B, m, f, k, ids, scores, raw, counts, workspace, workspace.numel(), stream,
                            flags | plan_flag)
        self._last_workspace = workspace
        return ids, scores, raw, counts

    # ---- quantised search (Sec. 3.2) ----
    def build_bits(self, perm, signs, k_bits):
        """perm (uint32 [d]) and signs (int8 [d]): numpy (host) or device tensors; [R, d] each for R independent draws
        (codes of k_bits / R bits per draw, concatenated)"""
        src = SRC_HOST if isinstance(perm, np.ndarray) else SRC_DEVICE_COPY
        reps = int(perm.shape[0]) if len(perm.shape) == 2 else 1
        if isinstance(perm, np.ndarray):
            perm, signs = np.ascontiguousarray(perm), np.ascontiguousarray(signs)
        else:
            perm, signs = perm.contiguous(), signs.contiguous()
        index_build_bits(self.handle, perm, signs, k_bits, src, reps)
        self.k_bits = k_bits
        return self

    def _filters(self, filters):
        if isinstance(filters, np.ndarray):
            return FILTERS_ON_HOST, np.ascontiguousarray(filters)
        return FILTERS_ON_DEVICE, filters

    def quantize(self, Q):
        import torch
        Q = Q.reshape(Q.shape[0], -1).contiguous()
        W = (self.k_bits + 63) // 64
        qbits = torch.empty((Q.shape[0], W), dtype=torch.int64, device=Q.device)
        quantize_queries(self.handle, Q, Q.shape[0], qbits, torch.cuda.current_stream(Q.device).cuda_stream)
        return qbits

    def search_bits(self, qbits, filters, T):
        """qbits: device int64 [B, W].  Returns device tensors ids, matches (int32), counts."""
        import torch
        qbits = qbits.contiguous()
        B, dev = qbits.shape[0], qbits.device
        ids = torch.empty((B, T), dtype=torch.int32, device=dev)
        matches = torch.empty((B, T), dtype=torch.int32, device=dev)
        counts = torch.empty((B,), dtype=torch.int32, device=dev)
        if B == 0:
            return ids, matches, counts
        nbytes = search_bits_workspace_bytes(self.handle, B, T)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        flags, f = self._filters(filters)
        search_bits(self.handle, qbits, B, f, T, ids, matches, counts, ws, nbytes, torch.cuda.current_stream(dev).cuda_stream, flags)
        self._last_workspace = ws
        return ids, matches, counts

    def select_bits(self, qbits, filters, K):
        """Large-K selection: qbits device int64 [B, W].  Returns device tensors ids [B, K] (int32; row b holds
        counts[b] ascending ids), counts (int64), thresholds (int32)."""
        import torch
        qbits = qbits.contiguous()
        B, dev = qbits.shape[0], qbits.device
        ids = torch.empty((B, K), dtype=torch.int32, device=dev)
        counts = torch.empty((B,), dtype=torch.int64, device=dev)
        thresholds = torch.empty((B,), dtype=torch.int32, device=dev)
        if B == 0:
            return ids, counts, thresholds
        nbytes = select_bits_workspace_bytes(self.handle, B)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        flags, f = self._filters(filters)
        select_bits(self.handle, qbits, B, f, K, ids, counts, thresholds, ws, nbytes, torch.cuda.current_stream(dev).cuda_stream, flags)
        self._last_workspace = ws
        return ids, counts, thresholds

    def search_two_stage(self, Q, filters, T, k):
        import torch
        Q = Q.reshape(Q.shape[0], -1).contiguous()
        B, dev = Q.shape[0], Q.device
        ids = torch.empty((B, k), dtype=torch.int32, device=dev)
        scores = torch.empty((B, k), dtype=torch.float32, device=dev)
        counts = torch.empty((B,), dtype=torch.int32, device=dev)
        if B == 0:
            return ids, scores, counts
        nbytes = search_two_stage_workspace_bytes(self.handle, B, T, k)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        flags, f = self._filters(filters)
        search_two_stage(self.handle, Q, B, f, T, k, ids, scores, counts, ws, nbytes, torch.cuda.current_stream(dev).cuda_stream, flags)
        self._last_workspace = ws
        return ids, scores, counts

    def close(self):
        if self.handle:
            index_destroy(self.handle)
            self.handle = None
            self._keep = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
