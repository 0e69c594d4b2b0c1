"""ctypes loader for oracle/linr_oracle.c (plain C, built with gcc).

TEST INFRASTRUCTURE: the product path never calls into this module.

Besides the loader, two functions are written here in numpy from their definitions: filter_passes (the Sec. 3.1.1
rule for whole columns) and bits_select (large-K selection by bit matching, Sec. 3.2 / 5.3); both are pinned in
tests/test_oracle_select_pins.py (hand-worked example, brute force with Python integers, the C ranking routine,
characterising properties).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import numpy as np

F32, BF16, I8 = 0, 1, 2
NO_ID = 0xFFFFFFFF

#: the oracle's own statement of the 40-byte filter record read by linr_oracle.c
FILTER_DTYPE = np.dtype([
    ("all_bits", "<u4"), ("none_bits", "<u4"), ("any_bits", "<u4", (4,)),
    ("n_any", "<u4"), ("ts_min", "<u4"), ("ts_max", "<u4"), ("_pad", "<u4"),
])

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "linr_oracle.c")
_SRC_BITS = os.path.join(_HERE, "linr_oracle_bits.c")
_SRC_CLAUSES = os.path.join(_HERE, "linr_oracle_clauses.c")
_LIB = os.path.join(_HERE, "liblinr_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_BITS), os.path.getmtime(_SRC_CLAUSES))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
                               "-o", tmp, _SRC, _SRC_BITS, _SRC_CLAUSES, "-lpthread", "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = C.CDLL(_LIB)
        vp, u64, u32, i32 = C.c_void_p, C.c_uint64, C.c_uint32, C.c_int
        lib.linr_oracle_search.restype = i32
        lib.linr_oracle_search.argtypes = [i32, vp, vp, vp, vp, u64, u32, u64, vp, vp, u32, u32, vp, u32,
                                           vp, vp, vp, vp, i32]
        lib.linr_oracle_pairs.restype = i32
        lib.linr_oracle_pairs.argtypes = [i32, vp, vp, vp, vp, u32, vp, u32, vp, u64, vp, vp, vp, vp, vp]
        lib.linr_oracle_dot_f64.restype = C.c_double
        lib.linr_oracle_dot_f64.argtypes = [i32, vp, vp, u32]
        lib.linr_oracle_pass.restype = i32
        lib.linr_oracle_pass.argtypes = [vp, u32, i32, u32]
        lib.linr_oracle_sign_oporp.restype = i32
        lib.linr_oracle_sign_oporp.argtypes = [vp, u64, u32, vp, vp, u32, vp]
        lib.linr_oracle_sign_oporp_rep.restype = i32
        lib.linr_oracle_sign_oporp_rep.argtypes = [vp, u64, u32, vp, vp, u32, u32, vp]
        lib.linr_oracle_bit_matches.restype = u32
        lib.linr_oracle_bit_matches.argtypes = [vp, vp, u32, u32]
        lib.linr_oracle_bits_search.restype = i32
        lib.linr_oracle_bits_search.argtypes = [vp, u32, u32, vp, vp, u64, u64, vp, u32, vp, u32, vp, vp, vp]
        lib.linr_oracle_clause_feasible.restype = i32
        lib.linr_oracle_clause_feasible.argtypes = [vp, u32, vp, u32, u64, vp, vp, u32, vp]
        _lib = lib
    return _lib


_ELT = {F32: np.float32, BF16: np.uint16, I8: np.int8}


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a, dt):
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype != dt:
        raise TypeError(f"expected {dt}, got {a.dtype}")
    return a


def search(dtype, emb, mask, Q, filters, k, row_scale=None, ts=None, q_scale=None, id_base=0, nthreads=1):
    """Exhaustive filtered top-k on the CPU.  emb [n,d]; Q [B,m,d] (or [B,d]); filters [B] records.
    Returns ids [B,k] u32, scores [B,k] f32, raw [B,k] i32, counts [B] u32."""
    lib = _load()
    emb = _c(emb, _ELT[dtype]); Q = _c(Q, _ELT[dtype])
    if Q.ndim == 2:
        Q = Q[:, None, :]
    n, d = emb.shape
    B, m, d2 = Q.shape
    assert d2 == d
    mask = _c(mask, np.uint32); ts = _c(ts, np.uint32)
    row_scale = _c(row_scale, np.float32); q_scale = _c(q_scale, np.float32)
    filters = _c(filters, FILTER_DTYPE)
    assert mask.shape == (n,) and filters.shape == (B,)
    ids = np.empty((B, k), np.uint32); sc = np.empty((B, k), np.float32)
    raw = np.empty((B, k), np.int32); cnt = np.empty(B, np.uint32)
    rc = lib.linr_oracle_search(dtype, _ptr(emb), _ptr(row_scale), _ptr(mask), _ptr(ts), n, d, id_base,
                                _ptr(Q), _ptr(q_scale), B, m, _ptr(filters), k,
                                _ptr(ids), _ptr(sc), _ptr(raw), _ptr(cnt), nthreads)
    if rc != 0:
        raise RuntimeError(f"linr_oracle_search failed ({rc})")
    return ids, sc, raw, cnt


def pairs(dtype, emb, mask, Q, filters, pb, pi, row_scale=None, ts=None):
    """Ranking value / raw dot / feasibility of listed (query, item) pairs."""
    lib = _load()
    emb = _c(emb, _ELT[dtype]); Q = _c(Q, _ELT[dtype])
    if Q.ndim == 2:
        Q = Q[:, None, :]
    n, d = emb.shape
    B, m, _ = Q.shape
    mask = _c(mask, np.uint32); ts = _c(ts, np.uint32); row_scale = _c(row_scale, np.float32)
    filters = _c(filters, FILTER_DTYPE)
    pb = np.ascontiguousarray(pb, np.uint32); pi = np.ascontiguousarray(pi, np.uint64)
    npairs = pb.shape[0]
    rank = np.empty(npairs, np.float64); raw = np.empty(npairs, np.int32); feas = np.empty(npairs, np.uint8)
    lib.linr_oracle_pairs(dtype, _ptr(emb), _ptr(row_scale), _ptr(mask), _ptr(ts), d, _ptr(Q), m, _ptr(filters),
                          npairs, _ptr(pb), _ptr(pi), _ptr(rank), _ptr(raw), _ptr(feas))
    return rank, raw, feas.astype(bool)


def dot_f64(dtype, q, x):
    lib = _load()
    q = _c(q, _ELT[dtype]); x = _c(x, _ELT[dtype])
    return lib.linr_oracle_dot_f64(dtype, _ptr(q), _ptr(x), q.shape[0])


def passes(filt_record, mask, ts=None):
    lib = _load()
    f = np.ascontiguousarray(np.asarray(filt_record, dtype=FILTER_DTYPE).reshape(1))
    return bool(lib.linr_oracle_pass(_ptr(f), int(mask), 0 if ts is None else 1, 0 if ts is None else int(ts)))


# ---------------------------------------------------------------------------
# quantised search (Sec. 3.2): Sign-OPORP codes, bit matching, two-stage search
# ---------------------------------------------------------------------------
def widen(dtype, a):
    """fp32 array or bf16 bit patterns (uint16) -> float64, exactly."""
    a = np.ascontiguousarray(a)
    if dtype == F32:
        return a.astype(np.float64)
    if dtype == BF16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    raise TypeError("Sign-OPORP codes are built from fp32 or bf16 embeddings")


def sign_oporp(dtype, x, perm, signs, k_bits):
    """x [n, D] (fp32 or bf16 bit patterns) -> codes [n, ceil(k_bits/64)] uint64.  perm / signs of shape [D]: one draw;
    of shape [R, D]: R independent draws, k_bits / R bits each, concatenated in draw order."""
    lib = _load()
    xd = np.ascontiguousarray(widen(dtype, x))
    n, D = xd.shape
    perm = _c(perm, np.uint32); signs = _c(signs, np.int8)
    W = (k_bits + 63) // 64
    out = np.zeros((n, W), np.uint64)
    if perm.ndim == 2:
        reps = perm.shape[0]
        assert perm.shape == (reps, D) and signs.shape == (reps, D)
        if lib.linr_oracle_sign_oporp_rep(_ptr(xd), n, D, _ptr(perm), _ptr(signs), k_bits, reps, _ptr(out)) != 0:
            raise ValueError("k_bits must be a multiple of the draws and D a multiple of the bits per draw")
        return out
    assert perm.shape == (D,) and signs.shape == (D,)
    if lib.linr_oracle_sign_oporp(_ptr(xd), n, D, _ptr(perm), _ptr(signs), k_bits, _ptr(out)) != 0:
        raise ValueError("D must be a positive multiple of k_bits")
    return out


def bit_matches(a, b, k_bits):
    a = _c(a, np.uint64); b = _c(b, np.uint64)
    return int(_load().linr_oracle_bit_matches(_ptr(a), _ptr(b), a.size, k_bits))


def bits_search(bits, k_bits, mask, qbits, filters, T, ts=None, id_base=0):
    """Filtered top-T by number of matching bits (desc), id (asc).  Returns ids [B,T], matches [B,T], counts [B]."""
    lib = _load()
    bits = _c(bits, np.uint64); qbits = _c(qbits, np.uint64)
    n, W = bits.shape
    B = qbits.shape[0]
    mask = _c(mask, np.uint32); ts = _c(ts, np.uint32)
    filters = np.ascontiguousarray(filters)
    assert filters.dtype.itemsize == 40 and filters.shape == (B,)
    ids = np.empty((B, T), np.uint32); mt = np.empty((B, T), np.int32); cnt = np.empty(B, np.uint32)
    rc = lib.linr_oracle_bits_search(_ptr(bits), W, k_bits, _ptr(mask), _ptr(ts), n, id_base, _ptr(qbits), B, _ptr(filters), T,
                                     _ptr(ids), _ptr(mt), _ptr(cnt))
    if rc != 0:
        raise MemoryError
    return ids, mt, cnt


def two_stage(dtype, emb, mask, Q, filters, perm, signs, k_bits, T, k, ts=None):
    """Figure "KNN with Quantized Filtering": top-T by bit matching, then the exact scores of those T items, then
    top-k by (score desc, id asc).  Q [B, d] or [B, 1, d].  Returns ids [B,k], scores [B,k] (float32), counts [B]."""
    Q2 = Q.reshape(Q.shape[0], -1)
    bits = sign_oporp(dtype, emb, perm, signs, k_bits)
    qbits = sign_oporp(dtype, Q2, perm, signs, k_bits)
    ids1, _, cnt1 = bits_search(bits, k_bits, mask, qbits, filters, T, ts=ts)
    B = Q2.shape[0]
    out_ids = np.full((B, k), NO_ID, np.uint32); out_sc = np.full((B, k), -np.inf, np.float32); out_cnt = np.zeros(B, np.uint32)
    for b in range(B):
        c = int(cnt1[b])
        if c == 0:
            continue
        cand = ids1[b, :c].astype(np.uint64)
        rank, _, feas = pairs(dtype, emb, mask, Q, filters, np.full(c, b, np.uint32), cand, ts=ts)
        assert feas.all()
        order = np.lexsort((cand, -rank))[:k]
        kk = len(order)
        out_ids[b, :kk] = cand[order].astype(np.uint32); out_sc[b, :kk] = rank[order].astype(np.float32); out_cnt[b] = kk
    return out_ids, out_sc, out_cnt


def filter_passes(filt_record, mask, ts=None):
    """Sec. 3.1.1 feasibility rule over the bitmask / timestamp attributes for whole columns at once (numpy): every
    required bit present, no excluded bit present, at least one bit of every "any of" group, timestamp inside the
    inclusive window.  Returns a bool array [n]."""
    f = np.asarray(filt_record, dtype=FILTER_DTYPE).reshape(())
    mask = np.asarray(mask, np.uint32)
    ok = (mask & np.uint32(f["all_bits"])) == np.uint32(f["all_bits"])
    ok &= (mask & np.uint32(f["none_bits"])) == 0
    for g in range(min(int(f["n_any"]), 4)):
        ok &= (mask & np.uint32(f["any_bits"][g])) != 0
    if ts is not None:
        ts = np.asarray(ts, np.uint32)
        ok &= (ts >= np.uint32(f["ts_min"])) & (ts <= np.uint32(f["ts_max"]))
    return ok


def bits_select(bits, k_bits, mask, qbits, filters, K, ts=None, id_base=0):
    """Large-K selection by bit matching (Sec. 3.2, the quantised module used on its own "when K is large"; the
    notification use case of Sec. 5.3: the top 50 million of a billion members): per query the K feasible items with
    the most matching bits, ties to the lower id -- i.e. the first K of the ranking by (matches desc, id asc) -- reported
    as a set, in ascending id order.  Written as that definition: a stable sort by descending match count.
    Returns (ids: list of B uint32 arrays, thresholds int32 [B] = fewest matching bits among the selected (-1: none),
    counts uint64 [B] = min(K, #feasible))."""
    bits = np.ascontiguousarray(bits, np.uint64); qbits = np.ascontiguousarray(qbits, np.uint64)
    n, W = bits.shape
    B = qbits.shape[0]
    filters = np.ascontiguousarray(filters)
    assert filters.shape == (B,) and K >= 1 and k_bits <= 64 * W
    out, thr, cnt = [], np.full(B, -1, np.int32), np.zeros(B, np.uint64)
    for b in range(B):
        differing = np.zeros(n, np.uint16)
        for w in range(W):
            differing += np.bitwise_count(bits[:, w] ^ qbits[b, w]).astype(np.uint16)
        feasible = np.flatnonzero(filter_passes(filters[b], mask, ts))
        order = np.argsort(differing[feasible], kind="stable")          # fewest differing bits first, equal ones by id
        chosen = feasible[order[:K]]
        cnt[b] = chosen.size
        if chosen.size:
            thr[b] = k_bits - int(differing[chosen[-1]])
        out.append((np.sort(chosen) + id_base).astype(np.uint32))
    return out, thr, cnt


# ---------------------------------------------------------------------------
# attribute matching over clause lists (Sec. 3.1.1; the benchmark's representation, Sec. 5.3)
# ---------------------------------------------------------------------------
def clause_feasible(values, counts, q_values_row, q_counts_row, reverse):
    """0/1 vector over the n items for ONE query.  values [n, row_width] u64, counts [n, C] u8 (lists back to back,
    clause 0 first); the query's lists in the same layout; bit c of `reverse` marks clause c as a reverse clause."""
    lib = _load()
    values = _c(values, np.uint64); counts = _c(counts, np.uint8)
    qv = _c(np.atleast_1d(q_values_row), np.uint64); qc = _c(q_counts_row, np.uint8)
    n, row_width = values.shape
    C = counts.shape[1]
    assert counts.shape == (n, C) and qc.shape == (C,) and int(qc.sum()) <= qv.size
    out = np.empty(n, np.uint8)
    if lib.linr_oracle_clause_feasible(_ptr(values), row_width, _ptr(counts), C, n, _ptr(qv), _ptr(qc), int(reverse), _ptr(out)) != 0:
        raise ValueError("an item's counts exceed the row width")
    return out


def clause_search(dtype, emb, values, counts, Q, q_values, q_counts, reverse, k, row_scale=None, q_scale=None, nthreads=1):
    """Exhaustive top-k among the items that satisfy every clause of the query: for each query the feasibility vector
    above, then the exhaustive oracle restricted to the feasible items (feasibility handed over as a one-bit mask)."""
    if Q.ndim == 2:
        Q = Q[:, None, :]
    B = Q.shape[0]
    ids = np.empty((B, k), np.uint32); sc = np.empty((B, k), np.float32)
    raw = np.empty((B, k), np.int32); cnt = np.empty(B, np.uint32)
    f = np.zeros(1, FILTER_DTYPE)
    f["all_bits"] = 1
    f["ts_max"] = 0xFFFFFFFF
    for b in range(B):
        feas = clause_feasible(values, counts, q_values[b], q_counts[b], reverse).astype(np.uint32)
        i1, s1, r1, c1 = search(dtype, emb, feas, Q[b:b + 1], f, k, row_scale=row_scale,
                                q_scale=None if q_scale is None else q_scale[b:b + 1], nthreads=nthreads)
        ids[b], sc[b], raw[b], cnt[b] = i1[0], s1[0], r1[0], c1[0]
    return ids, sc, raw, cnt
