"""Pins of the CPU oracle against things other than itself: a hand-worked example,
numpy matmul + stable sort, a set-based restatement of the clause rule, brute
force on tiny inputs and invariants of exact top-k.  CPU only."""
import itertools
import json
import os
import numpy as np
import pytest

import synth_inputs as S

HERE = os.path.dirname(os.path.abspath(__file__))


def filt(B=1, **kw):
    f = S.make_filters(B)
    for key, v in kw.items():
        if key == "any_bits":
            for b in range(B):
                for g, x in enumerate(v):
                    f["any_bits"][b][g] = x
                f["n_any"][b] = len(v)
        else:
            f[key] = v
    return f


def bf16_bits(a):
    a = np.asarray(a, np.float32)
    u = a.view(np.uint32)
    assert np.all((u & 0xFFFF) == 0), "value not exactly representable in bf16"
    return (u >> 16).astype(np.uint16)


def as_dtype(dtype, a):
    a = np.asarray(a)
    if dtype == S.F32:
        return a.astype(np.float32)
    if dtype == S.BF16:
        return bf16_bits(a)
    return a.astype(np.int8)


# ---------------------------------------------------------------------------
# 1. hand-worked example (tests/golden/hand_example.json)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [S.F32, S.BF16, S.I8])
def test_hand_example(oracle_mod, dtype):
    g = json.load(open(os.path.join(HERE, "golden", "hand_example.json")))
    emb = as_dtype(dtype, g["items"]); Q = as_dtype(dtype, [g["query"]])
    mask = np.array(g["masks"], np.uint32)
    for c in g["cases"]:
        f = filt(all_bits=c["all_bits"], none_bits=c["none_bits"], any_bits=c["any_bits"])
        ids, sc, raw, cnt = oracle_mod.search(dtype, emb, mask, Q, f, c["k"])
        n = c["count"]
        assert cnt[0] == n, c["name"]
        assert ids[0, :n].tolist() == c["ids"], c["name"]
        assert sc[0, :n].tolist() == [float(x) for x in c["scores"]], c["name"]
        assert np.all(ids[0, n:] == S.NO_ID) and np.all(np.isneginf(sc[0, n:])), c["name"]
        if dtype == S.I8:
            assert raw[0, :n].tolist() == c["scores"] and np.all(raw[0, n:] == np.iinfo(np.int32).min)


def test_hand_example_scaled_int8(oracle_mod):
    g = json.load(open(os.path.join(HERE, "golden", "hand_example.json")))
    c = g["scaled_int8_case"]
    emb = as_dtype(S.I8, g["items"]); Q = as_dtype(S.I8, [g["query"]])
    mask = np.array(g["masks"], np.uint32)
    rs = np.array(g["row_scales_for_scaled_case"], np.float32)
    ids, sc, raw, cnt = oracle_mod.search(S.I8, emb, mask, Q, filt(all_bits=c["all_bits"]), c["k"], row_scale=rs,
                                          q_scale=np.array([0.5], np.float32))
    assert ids[0].tolist() == c["ids"] and raw[0].tolist() == c["raw"]
    assert sc[0].tolist() == [0.5 * x for x in c["rank"]]


def test_liquidity_case(oracle_mod):
    """The unfiltered top-1 is infeasible; post-filtering a top-1 would return nothing,
    pre-filtering must still return a full list (Sec. 1 'liquidity', Sec. 6 'Pre-filtering')."""
    g = json.load(open(os.path.join(HERE, "golden", "hand_example.json")))
    emb = as_dtype(S.F32, g["items"]); Q = as_dtype(S.F32, [g["query"]]); mask = np.array(g["masks"], np.uint32)
    ids, _, _, _ = oracle_mod.search(S.F32, emb, mask, Q, filt(), 1)
    assert ids[0, 0] == 5 and not (mask[5] & 3) == 3
    ids, _, _, cnt = oracle_mod.search(S.F32, emb, mask, Q, filt(all_bits=3), 1)
    assert cnt[0] == 1 and ids[0, 0] == 0


# ---------------------------------------------------------------------------
# 2. clause rule restated over attribute *sets* (Sec. 3.1.1), exhaustive
# ---------------------------------------------------------------------------
def feasible_by_sets(item_attrs, clauses):
    """clauses: list of (attribute set, reverse flag).  Every clause must hold;
    a forward clause holds if it shares an attribute with the item, a reverse one if it shares none."""
    for attrs, reverse in clauses:
        hit = len(item_attrs & attrs) > 0
        if hit == reverse:
            return False
    return True


def test_predicate_truth_table(oracle_mod):
    universe = range(4)
    subsets = [frozenset(c) for r in range(5) for c in itertools.combinations(universe, r)]
    nonempty = [s for s in subsets if s]
    bits = lambda s: sum(1 << a for a in s)
    checked = 0
    for single in itertools.product([None, 0, 1], repeat=2):               # up to two single-attribute clauses
        for multi in [(), (frozenset({1, 2}),), (frozenset({0, 3}), frozenset({2, 3}))]:
            for rev in [frozenset(), frozenset({2}), frozenset({0, 1})]:
                clauses = [(frozenset({a}), False) for a in single if a is not None]
                clauses += [(mset, False) for mset in multi]
                clauses += [(frozenset({a}), True) for a in rev]            # each reverse attribute is its own clause
                f = filt(all_bits=bits({a for a in single if a is not None}), none_bits=bits(rev),
                         any_bits=[bits(mset) for mset in multi])[0]
                for item in subsets:
                    assert oracle_mod.passes(f, bits(item)) == feasible_by_sets(item, clauses), (clauses, item)
                    checked += 1
    assert checked > 1000 and len(nonempty) == 15


def test_timestamp_window_inclusive(oracle_mod):
    f = filt(ts_min=100, ts_max=200)[0]
    got = [oracle_mod.passes(f, 0, ts) for ts in (99, 100, 150, 200, 201, 0, 0xFFFFFFFF)]
    assert got == [False, True, True, True, False, False, False]
    assert oracle_mod.passes(f, 0, None)          # no timestamp column: window not evaluated
    f = filt(ts_min=0x80000001, ts_max=0xFFFFFFFF)[0]   # unsigned comparison
    assert oracle_mod.passes(f, 0, 0x80000001) and not oracle_mod.passes(f, 0, 5)


# ---------------------------------------------------------------------------
# 3. numpy as an independent witness (matmul + stable sort; naive "V2" slicing)
# ---------------------------------------------------------------------------
def numpy_topk(scores_row, feasible, k):
    idx = np.nonzero(feasible)[0]
    order = np.lexsort((idx, -scores_row[idx]))      # primary: score descending, secondary: id ascending
    return idx[order][:k]


def np_feasible(mask, ts, f):
    ok = (mask & f["all_bits"]) == f["all_bits"]
    ok &= (mask & f["none_bits"]) == 0
    for g in range(int(f["n_any"])):
        ok &= (mask & f["any_bits"][g]) != 0
    if ts is not None:
        ok &= (ts >= f["ts_min"]) & (ts <= f["ts_max"])
    return ok


def random_filters(rng, B, with_ts):
    f = S.make_filters(B)
    for b in range(B):
        kind = b % 5
        if kind == 0:
            pass                                          # pass-all
        elif kind == 1:
            f["all_bits"][b] = 1 << rng.integers(0, 32)
        elif kind == 2:
            f["all_bits"][b] = (1 << rng.integers(0, 16)) | (1 << rng.integers(16, 32))
            f["none_bits"][b] = 1 << rng.integers(0, 32)
        elif kind == 3:
            f["any_bits"][b][0] = rng.integers(1, 2 ** 32, dtype=np.uint64) & 0x0F0F00FF
            f["any_bits"][b][1] = 1 << rng.integers(0, 32)
            f["n_any"][b] = 2
        else:
            f["all_bits"][b] = 0xFFFFFFFF                 # (almost surely) pass-none
        if with_ts and b % 2 == 0:
            f["ts_min"][b] = 300; f["ts_max"][b] = 700
    return f


@pytest.mark.parametrize("seed,n,d,B,m,k", [(1, 777, 24, 7, 1, 50), (2, 333, 16, 5, 3, 400), (3, 50, 8, 11, 2, 10)])
def test_int8_matches_numpy_int64(oracle_mod, seed, n, d, B, m, k):
    rng = np.random.default_rng(seed)
    emb = rng.integers(-127, 128, (n, d), dtype=np.int8); Q = rng.integers(-127, 128, (B, m, d), dtype=np.int8)
    emb[n // 2] = emb[n // 3]                              # a duplicate row: tie broken by id
    mask = rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32)
    ts = rng.integers(0, 1000, n).astype(np.uint32)
    f = random_filters(rng, B, True)
    rs = rng.uniform(0.5, 2.0, n).astype(np.float32); qs = rng.uniform(0.5, 2.0, B).astype(np.float32)
    raw_all = np.einsum("bmd,nd->bmn", Q.astype(np.int64), emb.astype(np.int64)).max(axis=1)     # [B, n]
    for scaled in (False, True):
        ids, sc, raw, cnt = oracle_mod.search(S.I8, emb, mask, Q, f, k, row_scale=rs if scaled else None, ts=ts, q_scale=qs)
        for b in range(B):
            feas = np_feasible(mask, ts, f[b])
            rank = raw_all[b].astype(np.float32) * rs if scaled else raw_all[b].astype(np.float64)
            want = numpy_topk(rank.astype(np.float64), feas, k)
            c = min(k, int(feas.sum()))
            assert cnt[b] == c
            assert ids[b, :c].tolist() == want.tolist()
            assert raw[b, :c].tolist() == raw_all[b][want].tolist()
            exp_sc = (rank[want].astype(np.float32) * qs[b]) if scaled else (raw_all[b][want].astype(np.float32) * qs[b])
            assert sc[b, :c].tobytes() == exp_sc.astype(np.float32).tobytes()
            assert np.all(ids[b, c:] == S.NO_ID)


@pytest.mark.parametrize("dtype", [S.F32, S.BF16])
@pytest.mark.parametrize("seed,n,d,B,m,k", [(4, 600, 32, 6, 1, 64), (5, 257, 48, 4, 3, 300)])
def test_float_matches_numpy_float64_within_band(oracle_mod, dtype, seed, n, d, B, m, k):
    rng = np.random.default_rng(seed)
    e32 = rng.standard_normal((n, d)).astype(np.float32); q32 = rng.standard_normal((B, m, d)).astype(np.float32)
    if dtype == S.BF16:
        e32 = (e32.view(np.uint32) & 0xFFFF0000).view(np.float32); q32 = (q32.view(np.uint32) & 0xFFFF0000).view(np.float32)
        emb, Q = (e32.view(np.uint32) >> 16).astype(np.uint16), (q32.view(np.uint32) >> 16).astype(np.uint16)
    else:
        emb, Q = e32, q32
    mask = rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32)
    f = random_filters(rng, B, False)
    exact = np.einsum("bmd,nd->bmn", q32.astype(np.float64), e32.astype(np.float64)).max(axis=1)
    ids, sc, _, cnt = oracle_mod.search(dtype, emb, mask, Q, f, k)
    for b in range(B):
        feas = np_feasible(mask, None, f[b]); c = min(k, int(feas.sum()))
        assert cnt[b] == c
        got = ids[b, :c].astype(np.int64)
        assert np.all(feas[got]) and len(set(got.tolist())) == c
        assert np.allclose(sc[b, :c], exact[b][got], rtol=1e-5, atol=1e-5)       # fp32 accumulation error only
        assert np.all(np.diff(sc[b, :c]) <= 0)
        if c:                                                                   # nothing clearly better was left out
            kth = exact[b][got].min()
            better = feas & (exact[b] > kth + 1e-4)
            assert set(np.nonzero(better)[0].tolist()) <= set(got.tolist())


def test_operand_order_is_not_transposed(oracle_mod):
    """Q[b][e][j] pairs with emb[i][j]: a one-hot query picks out one embedding column."""
    n, d = 9, 5
    emb = np.arange(n * d, dtype=np.float32).reshape(n, d) * np.array([1, -1, 2, -2, 3], np.float32)
    for j in range(d):
        Q = np.zeros((1, 1, d), np.float32); Q[0, 0, j] = 1
        ids, sc, _, _ = oracle_mod.search(S.F32, emb, np.zeros(n, np.uint32), Q, filt(), n)
        col = emb[:, j]
        assert sc[0].tolist() == sorted(col.tolist(), reverse=True)
        assert ids[0].tolist() == np.lexsort((np.arange(n), -col)).tolist()


def test_fp32_accumulation_is_far_inside_tolerance(oracle_mod):
    w = S.config1(n=2000, B=4, k=10)
    h = S.to_numpy(w)
    ids, sc, _, _ = oracle_mod.search(S.F32, h["emb"], h["mask"], h["Q"], h["filters"], 10)
    for b in range(4):
        for j in range(10):
            ref = oracle_mod.dot_f64(S.F32, h["Q"][b, 0], h["emb"][ids[b, j]])
            assert abs(sc[b, j] - ref) <= 1e-6 * max(1.0, abs(ref))


# ---------------------------------------------------------------------------
# 4. invariants of exact filtered top-k
# ---------------------------------------------------------------------------
def small_int8(rng, n=500, d=16, B=6, with_ts=True):
    emb = rng.integers(-20, 21, (n, d), dtype=np.int8); Q = rng.integers(-20, 21, (B, 1, d), dtype=np.int8)
    mask = rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32)
    ts = rng.integers(0, 1000, n).astype(np.uint32) if with_ts else None
    return emb, Q, mask, ts, random_filters(rng, B, with_ts)


def test_prefix_counts_order_unique(oracle_mod):
    rng = np.random.default_rng(10)
    emb, Q, mask, ts, f = small_int8(rng)
    big = oracle_mod.search(S.I8, emb, mask, Q, f, 400, ts=ts)
    small = oracle_mod.search(S.I8, emb, mask, Q, f, 37, ts=ts)
    for b in range(Q.shape[0]):
        feas = np_feasible(mask, ts, f[b]); P = int(feas.sum())
        assert big[3][b] == min(400, P) and small[3][b] == min(37, P)
        c = int(small[3][b])
        assert small[0][b, :c].tolist() == big[0][b, :c].tolist()                 # top-k' is a prefix of top-k
        got = big[0][b, :big[3][b]]
        assert np.all(feas[got]) and len(set(got.tolist())) == len(got)
        r = big[2][b, :big[3][b]]
        assert np.all(np.diff(r) <= 0)
        same = np.diff(r) == 0
        assert np.all(np.diff(got.astype(np.int64))[same] > 0)                  # equal scores: ascending id


def test_split_and_merge_equals_whole(oracle_mod):
    rng = np.random.default_rng(11)
    emb, Q, mask, ts, f = small_int8(rng, n=640)
    k = 50
    whole = oracle_mod.search(S.I8, emb, mask, Q, f, k, ts=ts)
    cut = 250
    a = oracle_mod.search(S.I8, emb[:cut], mask[:cut], Q, f, k, ts=ts[:cut])
    b = oracle_mod.search(S.I8, emb[cut:], mask[cut:], Q, f, k, ts=ts[cut:], id_base=cut)
    for q in range(Q.shape[0]):
        ids = np.concatenate([a[0][q, :a[3][q]], b[0][q, :b[3][q]]]).astype(np.int64)
        raw = np.concatenate([a[2][q, :a[3][q]], b[2][q, :b[3][q]]]).astype(np.int64)
        order = np.lexsort((ids, -raw))[:k]
        c = int(whole[3][q])
        assert ids[order].tolist() == whole[0][q, :c].tolist()


def test_item_permutation_and_batch_permutation(oracle_mod):
    rng = np.random.default_rng(12)
    emb, Q, mask, ts, f = small_int8(rng, n=300)
    k = 40
    base = oracle_mod.search(S.I8, emb, mask, Q, f, k, ts=ts)
    perm = rng.permutation(emb.shape[0])
    p = oracle_mod.search(S.I8, emb[perm], mask[perm], Q, f, k, ts=ts[perm])
    for b in range(Q.shape[0]):
        c = int(base[3][b]); assert p[3][b] == c
        assert p[2][b, :c].tolist() == base[2][b, :c].tolist()                   # same score list
    bp = rng.permutation(Q.shape[0])
    q = oracle_mod.search(S.I8, emb, mask, Q[bp], f[bp], k, ts=ts)
    assert np.array_equal(q[0], base[0][bp]) and np.array_equal(q[3], base[3][bp])


def test_identical_rows_return_lowest_feasible_ids(oracle_mod):
    n, d = 200, 8
    emb = np.tile(np.arange(1, d + 1, dtype=np.int8), (n, 1)); Q = np.ones((1, 1, d), np.int8)
    mask = (np.arange(n) % 3 == 0).astype(np.uint32)
    ids, _, _, cnt = oracle_mod.search(S.I8, emb, mask, Q, filt(all_bits=1), 25)
    assert cnt[0] == 25 and ids[0].tolist() == list(range(0, 75, 3))


def test_signed_zero_scores_tie_on_id(oracle_mod):
    emb = np.array([[-1.0, 0.0], [1.0, 0.0], [0.0, 0.0]], np.float32); Q = np.array([[[0.0, 1.0]]], np.float32)
    emb[0, 1] = -0.0        # scores: -0.0 (+0*-0...), 0.0, 0.0 -> all compare equal
    ids, sc, _, _ = oracle_mod.search(S.F32, emb, np.zeros(3, np.uint32), Q, filt(), 3)
    assert ids[0].tolist() == [0, 1, 2] and np.all(sc[0] == 0.0)


def test_pairs_agree_with_search(oracle_mod):
    rng = np.random.default_rng(13)
    emb, Q, mask, ts, f = small_int8(rng, n=200)
    rs = rng.uniform(0.5, 2, 200).astype(np.float32)
    ids, sc, raw, cnt = oracle_mod.search(S.I8, emb, mask, Q, f, 20, row_scale=rs, ts=ts)
    for b in range(Q.shape[0]):
        c = int(cnt[b])
        if not c:
            continue
        rank, r, feas = oracle_mod.pairs(S.I8, emb, mask, Q, f, np.full(c, b), ids[b, :c], row_scale=rs, ts=ts)
        assert feas.all() and r.tolist() == raw[b, :c].tolist()
        assert rank.astype(np.float32).tobytes() == sc[b, :c].tobytes()        # q_scale absent -> score == rank


# ---------------------------------------------------------------------------
# 5. closed forms of the input recipe
# ---------------------------------------------------------------------------
def test_generator_pass_rates_and_quantiser_bound():
    w = S.to_numpy(S.config1(n=200_000, B=8))
    for b in range(8):
        frac = np_feasible(w["mask"], None, w["filters"][b]).mean()
        assert abs(frac - 0.125) < 5 * np.sqrt(0.125 * 0.875 / 200_000)
    assert np.allclose(np.linalg.norm(w["emb"], axis=1), 1.0, atol=1e-5)
    w3 = S.config3(n=100_000, B=4, chunk=50_000); h3 = S.to_numpy(w3)
    frac = np.mean([np_feasible(h3["mask"], h3["ts"], h3["filters"][b]).mean() for b in range(4)])
    assert abs(frac - 0.3 * 7 / 30) < 0.01
    assert h3["emb"].dtype == np.int8 and np.abs(h3["emb"].astype(int)).max() == 127 and np.all(h3["scale"] > 0)
    # |x - scale*code| <= scale/2 for the symmetric quantiser
    import torch
    x = S.clustered_rows(1000, S.unit_centres(10, 64, "cpu", 1), 0.3, "cpu", 2)
    c, s = S.quantize_rows(x)
    assert torch.all((x - c.float() * s[:, None]).abs() <= s[:, None] / 2 + 1e-7)
    w5 = S.to_numpy(S.config5(n=200_000, B=4, chunk=100_000, selectivity="5%"))
    frac = np.mean([np_feasible(w5["mask"], None, w5["filters"][b]).mean() for b in range(4)])
    assert abs(frac - 0.05) < 0.005


def test_scaled_rank_is_one_fp32_product(oracle_mod):
    """(float)raw * row_scale is rounded to fp32 before ranking: 3 * fl(1/3) rounds to exactly 1.0
    and therefore ties with 1 * 1.0, so the lower id wins although the unrounded product is larger."""
    third = np.float32(1.0) / np.float32(3.0)
    assert np.float32(3.0) * third == np.float32(1.0) and float(third) * 3.0 > 1.0
    emb = np.array([[1], [3]], np.int8); Q = np.array([[[1]]], np.int8)
    rs = np.array([1.0, third], np.float32)
    ids, sc, raw, _ = oracle_mod.search(S.I8, emb, np.zeros(2, np.uint32), Q, filt(), 2, row_scale=rs)
    assert ids[0].tolist() == [0, 1] and raw[0].tolist() == [1, 3] and sc[0].tolist() == [1.0, 1.0]
