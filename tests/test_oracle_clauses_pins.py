"""Pins of the clause-list feasibility rule and the search over it (oracle.clause_feasible / clause_search; LiNR
Sec. 3.1.1) against things other than themselves: a hand-worked example in the shape of the paper's figure, Python
sets, the already pinned bitmask oracle on inputs where both representations say the same, and invariants."""
import json
import os
import numpy as np
import pytest

import synth_inputs as S

HERE = os.path.dirname(os.path.abspath(__file__))


def pack(lists, C, width=None):
    """lists[i][c] = list of attributes -> (values [n, width] u64, counts [n, C] u8), lists back to back"""
    n = len(lists)
    width = width or max(1, max(sum(len(l) for l in item) for item in lists))
    v = np.zeros((n, width), np.uint64); c = np.zeros((n, C), np.uint8)
    for i, item in enumerate(lists):
        flat = [a for l in item for a in l]
        v[i, :len(flat)] = flat
        c[i] = [len(l) for l in item]
    return v, c


def test_hand_example(oracle_mod):
    g = json.load(open(os.path.join(HERE, "golden", "clause_lists_example.json")))
    v, c = pack(g["item_lists"], 2)
    qv, qc = pack([g["query_lists"]], 2)
    feas = oracle_mod.clause_feasible(v, c, qv[0], qc[0], g["reverse"])
    assert feas.tolist() == g["feasible"]
    emb = np.array(g["emb"], np.float32); Q = np.array([g["query"]], np.float32)
    for k, key in ((1, "top1"), (3, "top3")):
        ids, sc, _, cnt = oracle_mod.clause_search(oracle_mod.F32, emb, v, c, Q, qv, qc, g["reverse"], k)
        assert ids[0].tolist() == g[key]["ids"] and sc[0].tolist() == g[key]["scores"] and cnt[0] == k
    ids, sc, _, cnt = oracle_mod.clause_search(oracle_mod.F32, emb, v, c, Q, qv, qc, g["reverse"], 5)
    assert cnt[0] == g["top5_count"] and np.all(ids[0, 3:] == oracle_mod.NO_ID)
    none = np.zeros((1, 2), np.uint8)
    ids, sc, _, _ = oracle_mod.clause_search(oracle_mod.F32, emb, v, c, Q, qv, none, g["reverse"], 1)
    assert ids[0].tolist() == g["no_clauses_top1"]["ids"] and sc[0].tolist() == g["no_clauses_top1"]["scores"]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_feasibility_against_python_sets(oracle_mod, seed):
    rng = np.random.default_rng(seed)
    n, C = 300, 3
    items = [[rng.integers(0, 6, rng.integers(0, 4)).tolist() for _ in range(C)] for _ in range(n)]
    v, c = pack(items, C, width=12)
    for trial in range(20):
        q = [rng.integers(0, 6, rng.integers(0, 3)).tolist() for _ in range(C)]
        reverse = int(rng.integers(0, 8))
        qv, qc = pack([q], C, width=8)
        got = oracle_mod.clause_feasible(v, c, qv[0], qc[0], reverse)
        for i in range(n):
            ok = True
            for cl in range(C):
                if not q[cl]:
                    continue
                hit = bool(set(items[i][cl]) & set(q[cl]))
                ok &= (not hit) if (reverse >> cl) & 1 else hit
            assert got[i] == ok, (i, items[i], q, reverse)


def test_same_answers_as_the_bitmask_oracle_where_both_apply(oracle_mod):
    """attributes 0..31, one per item and clause: clause 0 "attribute in S" is the any-of group with bits S over the
    mask 1 << attribute; reverse clause 1 "attribute not in R" is none_bits = R over a second bit field"""
    rng = np.random.default_rng(7)
    n, d, B, k = 4000, 16, 6, 30
    emb = rng.standard_normal((n, d)).astype(np.float32)
    Q = rng.standard_normal((B, d)).astype(np.float32)
    a0 = rng.integers(0, 16, n); a1 = rng.integers(16, 32, n)
    v = np.stack([a0, a1], 1).astype(np.uint64); c = np.ones((n, 2), np.uint8)
    mask = ((1 << a0) | (1 << a1)).astype(np.uint32)
    f = S.make_filters(B)
    qlists = []
    for b in range(B):
        Sset = rng.choice(16, rng.integers(1, 5), replace=False).tolist()
        R = rng.choice(np.arange(16, 32), rng.integers(0, 4), replace=False).tolist()
        f["any_bits"][b][0] = sum(1 << s for s in Sset); f["n_any"][b] = 1
        f["none_bits"][b] = sum(1 << r for r in R)
        qlists.append([Sset, R])
    qv, qc = pack(qlists, 2, width=8)
    want = oracle_mod.search(oracle_mod.F32, emb, mask, Q, f, k)
    got = oracle_mod.clause_search(oracle_mod.F32, emb, v, c, Q, qv, qc, 0b10, k)
    for w, g in zip(want, got):
        assert np.array_equal(w, g)


def test_invariants(oracle_mod):
    rng = np.random.default_rng(3)
    n, C = 200, 2
    items = [[rng.integers(0, 5, rng.integers(1, 4)).tolist() for _ in range(C)] for _ in range(n)]
    q = [[1, 3], [2]]
    v, c = pack(items, C, width=8)
    qv, qc = pack([q], C, width=4)
    base = oracle_mod.clause_feasible(v, c, qv[0], qc[0], 0b10)
    # the order of the attributes inside a list and repeated attributes do not matter
    shuffled = [[list(reversed(l)) + l[:1] for l in item] for item in items]
    v2, c2 = pack(shuffled, C, width=10)
    assert np.array_equal(oracle_mod.clause_feasible(v2, c2, qv[0], qc[0], 0b10), base)
    qv2, qc2 = pack([[[3, 1, 3], [2, 2]]], C, width=6)
    assert np.array_equal(oracle_mod.clause_feasible(v, c, qv2[0], qc2[0], 0b10), base)
    # a reverse clause is the complement of the same clause taken forward (for a non-empty query list)
    fwd = oracle_mod.clause_feasible(v, c, np.array([2, 0, 0, 0], np.uint64), np.array([0, 1], np.uint8), 0)
    rev = oracle_mod.clause_feasible(v, c, np.array([2, 0, 0, 0], np.uint64), np.array([0, 1], np.uint8), 0b10)
    assert np.array_equal(fwd ^ 1, rev)
    # all clauses must hold: the joint answer is the AND of the single-clause answers
    only0 = oracle_mod.clause_feasible(v, c, np.array([1, 3, 0, 0], np.uint64), np.array([2, 0], np.uint8), 0b10)
    assert np.array_equal(base, only0 & rev)
    # a clause without query attributes constrains nothing, reverse or not
    every = oracle_mod.clause_feasible(v, c, np.zeros(4, np.uint64), np.zeros(2, np.uint8), 0b11)
    assert every.all()
    # counts that overrun the row are refused
    bad = c.copy(); bad[5] = [5, 5]
    with pytest.raises(ValueError):
        oracle_mod.clause_feasible(v, bad, qv[0], qc[0], 0)
