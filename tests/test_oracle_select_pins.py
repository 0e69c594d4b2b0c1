"""Pins of the large-K selection oracle (oracle.bits_select, oracle.filter_passes) against things other than itself:
a hand-worked example, brute force with Python integers, the separately written and separately pinned ranking
routine in C (oracle.bits_search) and item-by-item filter rule (oracle.passes), and the properties that
characterise the result (threshold rule, lowest ids among the ties, count)."""
import json
import os

import numpy as np
import pytest

import synth_inputs as S

HERE = os.path.dirname(os.path.abspath(__file__))


def rand_case(seed, n, W, k_bits, B, with_ts=False, narrow=False):
    rng = np.random.default_rng(seed)
    bits = rng.integers(0, 2 ** 63, (n, W), dtype=np.uint64) * np.uint64(2) + rng.integers(0, 2, (n, W), dtype=np.uint64)
    q = rng.integers(0, 2 ** 63, (B, W), dtype=np.uint64) * np.uint64(2) + rng.integers(0, 2, (B, W), dtype=np.uint64)
    if narrow:                                   # few distinct match counts: long runs of ties
        bits &= np.uint64(0xFF); q &= np.uint64(0xFF)
    if k_bits % 64:
        keep = np.uint64((1 << (k_bits % 64)) - 1)
        bits[:, -1] &= keep; q[:, -1] &= keep
    mask = rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32)
    ts = rng.integers(0, 1000, n).astype(np.uint32) if with_ts else None
    f = S.make_filters(B)
    for b in range(B):
        if b % 3 == 1:
            f["all_bits"][b] = 1 << int(rng.integers(0, 32))
        if b % 3 == 2:
            f["none_bits"][b] = 3 << int(rng.integers(0, 30)); f["any_bits"][b][0] = 0xF0F0; f["n_any"][b] = 1
        if with_ts and b % 2 == 0:
            f["ts_min"][b] = 100; f["ts_max"][b] = 700
    return bits, q, mask, ts, f


def test_hand_example(oracle_mod):
    g = json.load(open(os.path.join(HERE, "golden", "bits_select_example.json")))
    bits = np.array(g["codes"], np.uint64).reshape(-1, 1)
    q = np.array([[g["query"]]], np.uint64)
    mask = np.array(g["mask"], np.uint32)
    f = S.make_filters(1); f["all_bits"][0] = g["all_bits"]
    for i, want in enumerate(g["matches"]):
        assert oracle_mod.bit_matches(bits[i], q[0], g["k_bits"]) == want
    for c in g["cases"]:
        ids, thr, cnt = oracle_mod.bits_select(bits, g["k_bits"], mask, q, f, c["K"])
        assert ids[0].tolist() == c["ids"] and int(thr[0]) == c["threshold"] and int(cnt[0]) == c["count"], c


@pytest.mark.parametrize("seed,n,W,k_bits,K", [(1, 50, 1, 64, 7), (2, 200, 2, 100, 60), (3, 64, 1, 8, 30), (4, 300, 4, 256, 299)])
def test_brute_force_python_integers(oracle_mod, seed, n, W, k_bits, K):
    bits, q, mask, ts, f = rand_case(seed, n, W, k_bits, 3, with_ts=True, narrow=(k_bits == 8))
    ids, thr, cnt = oracle_mod.bits_select(bits, k_bits, mask, q, f, K, ts=ts)
    for b in range(3):
        rows = []
        for i in range(n):
            if not oracle_mod.passes(f[b], mask[i], ts[i]):
                continue
            diff = sum(bin(int(bits[i, w]) ^ int(q[b, w])).count("1") for w in range(W))
            rows.append((-(k_bits - diff), i))
        rows.sort()
        top = rows[:K]
        assert ids[b].tolist() == sorted(i for _, i in top)
        assert int(cnt[b]) == len(top)
        assert int(thr[b]) == (-top[-1][0] if top else -1)


@pytest.mark.parametrize("W,k_bits,with_ts", [(1, 64, False), (2, 128, True), (4, 200, False)])
def test_agrees_with_the_ranking_routine(oracle_mod, W, k_bits, with_ts):
    n, B = 20_000, 4
    bits, q, mask, ts, f = rand_case(10 + W, n, W, k_bits, B, with_ts=with_ts)
    for K in (1, 999, 5000, n):
        ids, thr, cnt = oracle_mod.bits_select(bits, k_bits, mask, q, f, K, ts=ts)
        rid, rmt, rcnt = oracle_mod.bits_search(bits, k_bits, mask, q, f, K, ts=ts)
        for b in range(B):
            c = int(rcnt[b])
            assert int(cnt[b]) == c
            assert np.array_equal(ids[b], np.sort(rid[b, :c]))
            assert int(thr[b]) == (int(rmt[b, c - 1]) if c else -1)


def test_characterising_properties_with_long_ties(oracle_mod):
    n, k_bits = 100_000, 64
    bits, q, mask, ts, f = rand_case(77, n, 1, k_bits, 3, narrow=True)
    for K in (10, 12_345, 60_000):
        ids, thr, cnt = oracle_mod.bits_select(bits, k_bits, mask, q, f, K)
        for b in range(3):
            m = np.array([k_bits - bin(int(x) ^ int(q[b, 0])).count("1") for x in bits[:, 0]])
            feas = np.array([oracle_mod.passes(f[b], mask[i]) for i in range(n)])
            sel = np.zeros(n, bool); sel[ids[b]] = True
            assert int(cnt[b]) == min(K, int(feas.sum())) == ids[b].size
            assert np.all(np.diff(ids[b].astype(np.int64)) > 0)
            assert feas[sel].all()
            t = int(thr[b])
            assert m[sel].min() == t
            assert not np.any(feas & ~sel & (m > t))                    # nothing better was left out
            ties = np.flatnonzero(feas & (m == t))
            taken = int(sel[ties].sum())
            assert np.array_equal(np.flatnonzero(sel & (m == t)), ties[:taken])      # the lowest ids among the ties


def test_filter_rule_for_whole_columns(oracle_mod):
    rng = np.random.default_rng(5)
    n = 3000
    mask = rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32)
    ts = rng.integers(0, 50, n).astype(np.uint32)
    f = S.make_filters(6)
    f["all_bits"][1] = 0x11; f["none_bits"][2] = 0x300
    f["any_bits"][3][0] = 0xF; f["any_bits"][3][1] = 0xF000; f["n_any"][3] = 2
    f["ts_min"][4] = 10; f["ts_max"][4] = 20
    f["all_bits"][5] = 4; f["none_bits"][5] = 4                  # contradictory: nothing passes
    for b in range(6):
        for use_ts in (False, True):
            got = oracle_mod.filter_passes(f[b], mask, ts if use_ts else None)
            want = [oracle_mod.passes(f[b], mask[i], ts[i] if use_ts else None) for i in range(n)]
            assert got.tolist() == want
    assert not oracle_mod.filter_passes(f[5], mask).any()


def test_k_beyond_feasible_and_id_base(oracle_mod):
    bits, q, mask, ts, f = rand_case(9, 500, 1, 64, 2)
    f["all_bits"][1] = 0xFFFF                                     # almost nothing passes
    ids, thr, cnt = oracle_mod.bits_select(bits, 64, mask, q, f, 10_000, id_base=1000)
    assert int(cnt[0]) == 500 and ids[0].tolist() == list(range(1000, 1500))
    feas1 = [i for i in range(500) if (int(mask[i]) & 0xFFFF) == 0xFFFF]
    assert ids[1].tolist() == [1000 + i for i in feas1] and int(cnt[1]) == len(feas1)
    if not feas1:
        assert int(thr[1]) == -1
