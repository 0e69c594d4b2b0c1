"""Pins of the quantised-search oracle (oracle/linr_oracle_bits.c) against things other than itself:
the hand-worked example, the projection-matrix form of the sketch in numpy, closed forms, the angle law of sign
projections (statistically), brute force with Python integers, and the tie / filter / count rules."""
import json
import math
import os

import numpy as np
import pytest

import synth_inputs as S

HERE = os.path.dirname(os.path.abspath(__file__))


def draw(seed, D):
    rng = np.random.default_rng(seed)
    return rng.permutation(D).astype(np.uint32), rng.choice(np.array([-1, 1], np.int8), D)


def unpack(codes, k_bits):
    """[n, W] uint64 -> [n, k_bits] 0/1, bit j = position j%64 of word j/64"""
    n, W = codes.shape
    out = np.zeros((n, k_bits), np.uint8)
    for j in range(k_bits):
        out[:, j] = (codes[:, j // 64] >> np.uint64(j % 64)) & np.uint64(1)
    return out


def test_hand_example(oracle_mod):
    g = json.load(open(os.path.join(HERE, "golden", "sign_oporp_example.json")))
    x = np.array(g["x"], np.float32)
    codes = oracle_mod.sign_oporp(S.F32, x, np.array(g["perm"], np.uint32), np.array(g["signs"], np.int8), g["k_bits"])
    assert codes.shape == (4, 1) and codes[:, 0].tolist() == g["codes"]
    for key, want in g["matches"].items():
        a, b = map(int, key.split(","))
        assert oracle_mod.bit_matches(codes[a], codes[b], g["k_bits"]) == want


def test_hand_example_two_draws(oracle_mod):
    g = json.load(open(os.path.join(HERE, "golden", "sign_oporp_two_draws_example.json")))
    x = np.array(g["x"], np.float32)
    codes = oracle_mod.sign_oporp(S.F32, x, np.array(g["perm"], np.uint32), np.array(g["signs"], np.int8), g["k_bits"])
    assert codes.shape == (4, 1) and codes[:, 0].tolist() == g["codes"]
    for key, want in g["matches"].items():
        a, b = map(int, key.split(","))
        assert oracle_mod.bit_matches(codes[a], codes[b], g["k_bits"]) == want


@pytest.mark.parametrize("D,k_bits,reps", [(128, 512, 4), (128, 256, 2), (64, 384, 6), (128, 192, 3), (96, 64, 2)])
def test_projection_matrix_form_with_repetitions(oracle_mod, D, k_bits, reps):
    """R draws = one projection matrix of R stacked blocks, block r built from (perm_r, signs_r): sketch = P x"""
    rng = np.random.default_rng(D + k_bits + reps)
    perm = np.stack([rng.permutation(D) for _ in range(reps)]).astype(np.uint32)
    signs = rng.choice(np.array([-1, 1], np.int8), (reps, D))
    x = rng.standard_normal((200, D)).astype(np.float32)
    k1 = k_bits // reps
    L = D // k1
    P = np.zeros((k_bits, D))
    for r in range(reps):
        for j in range(k1):
            for t in range(L):
                P[r * k1 + j, perm[r, j * L + t]] = signs[r, j * L + t]
    sk = x.astype(np.float64) @ P.T
    safe = np.abs(sk) > 1e-9
    got = unpack(oracle_mod.sign_oporp(S.F32, x, perm, signs, k_bits), k_bits)
    assert np.array_equal(got[safe], (sk > 0)[safe].astype(np.uint8))
    assert safe.mean() > 0.999
    # every coordinate enters each draw exactly once
    assert np.all(np.abs(P).reshape(reps, k1, D).sum(axis=1) == 1)
    with pytest.raises(ValueError):
        oracle_mod.sign_oporp(S.F32, x, perm, signs, k_bits + reps * 7)      # bits per draw must divide D


def test_angle_law_holds_for_repeated_draws(oracle_mod):
    """each draw obeys 1 - angle/pi, so does their concatenation; independent draws make the estimate tighter than one
    draw of the same bins would (the reason for repeating): the spread of the match fraction over pairs shrinks"""
    D, reps, k1, pairs_n = 1024, 4, 32, 1200
    rng = np.random.default_rng(77)
    perm = np.stack([rng.permutation(D) for _ in range(reps)]).astype(np.uint32)
    signs = rng.choice(np.array([-1, 1], np.int8), (reps, D))
    rho = 0.6
    a = rng.standard_normal((pairs_n, D))
    b = rho * a + math.sqrt(1 - rho * rho) * rng.standard_normal((pairs_n, D))
    want = 1.0 - math.acos(rho) / math.pi
    kb = reps * k1
    ca = oracle_mod.sign_oporp(S.F32, a.astype(np.float32), perm, signs, kb)
    cb = oracle_mod.sign_oporp(S.F32, b.astype(np.float32), perm, signs, kb)
    fr = np.array([oracle_mod.bit_matches(ca[i], cb[i], kb) for i in range(pairs_n)]) / kb
    assert abs(fr.mean() - want) < 4.0 * 0.5 / math.sqrt(pairs_n * kb) + 3e-3
    c1a = oracle_mod.sign_oporp(S.F32, a.astype(np.float32), perm[0], signs[0], k1)
    c1b = oracle_mod.sign_oporp(S.F32, b.astype(np.float32), perm[0], signs[0], k1)
    fr1 = np.array([oracle_mod.bit_matches(c1a[i], c1b[i], k1) for i in range(pairs_n)]) / k1
    assert fr.std() < 0.62 * fr1.std()                       # 4 x the bits: about half the spread


@pytest.mark.parametrize("D,k_bits", [(64, 64), (128, 64), (256, 128), (96, 32), (64, 16), (512, 256)])
def test_projection_matrix_form(oracle_mod, D, k_bits):
    """sketch = P x with P[j, perm[jL+t]] = signs[jL+t]: "one random projection" written as a matrix"""
    perm, signs = draw(D + k_bits, D)
    rng = np.random.default_rng(1)
    x = rng.standard_normal((300, D)).astype(np.float32)
    L = D // k_bits
    P = np.zeros((k_bits, D))
    for j in range(k_bits):
        for t in range(L):
            P[j, perm[j * L + t]] = signs[j * L + t]
    sk = x.astype(np.float64) @ P.T
    safe = np.abs(sk) > 1e-9                                 # away from rounding-order effects of the matrix product
    got = unpack(oracle_mod.sign_oporp(S.F32, x, perm, signs, k_bits), k_bits)
    assert np.array_equal(got[safe], (sk > 0)[safe].astype(np.uint8))
    assert safe.mean() > 0.999


def test_plain_sign_quantisation_is_the_special_case(oracle_mod):
    """bins of one, identity permutation, all signs +1: bit j = [x_j > 0]"""
    D = 64
    rng = np.random.default_rng(2)
    x = rng.standard_normal((50, D)).astype(np.float32)
    x[3, 5] = 0.0
    x[4] = -0.0
    got = unpack(oracle_mod.sign_oporp(S.F32, x, np.arange(D, dtype=np.uint32), np.ones(D, np.int8), D), D)
    assert np.array_equal(got, (x > 0).astype(np.uint8))


def test_closed_forms(oracle_mod):
    D, k_bits = 128, 64
    perm, signs = draw(7, D)
    rng = np.random.default_rng(3)
    x = rng.standard_normal((20, D)).astype(np.float32)
    c = oracle_mod.sign_oporp(S.F32, x, perm, signs, k_bits)
    cneg = oracle_mod.sign_oporp(S.F32, -x, perm, signs, k_bits)
    cscaled = oracle_mod.sign_oporp(S.F32, (x * np.float32(4.0)), perm, signs, k_bits)
    for i in range(20):
        assert oracle_mod.bit_matches(c[i], c[i], k_bits) == k_bits            # identical vectors
        assert oracle_mod.bit_matches(c[i], cneg[i], k_bits) == 0              # opposite vectors (no zero bin sum here)
        assert np.array_equal(c[i], cscaled[i])                                # positive scaling (exact: power of two)
    # flipping every sign of the random vector complements every code
    cflip = oracle_mod.sign_oporp(S.F32, x, perm, (-signs).astype(np.int8), k_bits)
    assert np.array_equal(cflip, ~c)
    # matches are symmetric and agree with counting equal unpacked bits
    u = unpack(c, k_bits)
    for a, b in [(0, 1), (2, 9), (5, 5), (7, 19)]:
        m = oracle_mod.bit_matches(c[a], c[b], k_bits)
        assert m == oracle_mod.bit_matches(c[b], c[a], k_bits) == int((u[a] == u[b]).sum())


def test_bf16_inputs_are_widened_exactly(oracle_mod):
    D, k_bits = 64, 64
    perm, signs = draw(11, D)
    rng = np.random.default_rng(4)
    xf = rng.standard_normal((40, D)).astype(np.float32)
    hb = (xf.view(np.uint32) >> 16).astype(np.uint16)                          # truncated bf16 patterns
    back = (hb.astype(np.uint32) << 16).view(np.float32)
    assert np.array_equal(oracle_mod.sign_oporp(S.BF16, hb, perm, signs, k_bits),
                          oracle_mod.sign_oporp(S.F32, back, perm, signs, k_bits))


def test_angle_law_of_sign_projections(oracle_mod):
    """For long bins the bin sums of two vectors are jointly close to Gaussian with the vectors' correlation, so the
    expected fraction of equal signs is 1 - angle/pi (the relation that makes bit matching estimate the cosine)."""
    D, k_bits, pairs_n = 2048, 64, 1500
    perm, signs = draw(21, D)
    rng = np.random.default_rng(5)
    for rho in (0.0, 0.5, 0.9, -0.7):
        a = rng.standard_normal((pairs_n, D))
        b = rho * a + math.sqrt(1 - rho * rho) * rng.standard_normal((pairs_n, D))
        ca = oracle_mod.sign_oporp(S.F32, a.astype(np.float32), perm, signs, k_bits)
        cb = oracle_mod.sign_oporp(S.F32, b.astype(np.float32), perm, signs, k_bits)
        frac = np.mean([oracle_mod.bit_matches(ca[i], cb[i], k_bits) for i in range(pairs_n)]) / k_bits
        want = 1.0 - math.acos(rho) / math.pi
        assert abs(frac - want) < 4.0 * 0.5 / math.sqrt(pairs_n * k_bits) + 2e-3, (rho, frac, want)


def py_bits_search(bits, k_bits, mask, ts, qbits, filt, T, passes):
    out = []
    for b in range(qbits.shape[0]):
        cand = []
        for i in range(bits.shape[0]):
            if not passes(filt[b], int(mask[i]), None if ts is None else int(ts[i])):
                continue
            diff = sum(bin(int(bits[i, w]) ^ int(qbits[b, w])).count("1") for w in range(bits.shape[1]))
            cand.append((-(k_bits - diff), i))
        cand.sort()
        out.append([(i, -m) for m, i in cand[:T]])
    return out


@pytest.mark.parametrize("k_bits,with_ts", [(64, False), (128, True), (32, False)])
def test_bits_search_against_python_integers(oracle_mod, k_bits, with_ts):
    rng = np.random.default_rng(k_bits)
    n, B, T = 400, 7, 25
    W = (k_bits + 63) // 64
    bits = rng.integers(0, 2 ** 63, (n, W), dtype=np.uint64) * np.uint64(2) + rng.integers(0, 2, (n, W), dtype=np.uint64)
    qbits = rng.integers(0, 2 ** 63, (B, W), dtype=np.uint64)
    if k_bits < 64:
        bits &= np.uint64((1 << k_bits) - 1); qbits &= np.uint64((1 << k_bits) - 1)
    bits[17] = qbits[0]; bits[5] = qbits[0]; bits[300] = qbits[0]               # three-way tie at the top for query 0
    mask = rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32)
    ts = rng.integers(0, 1000, n).astype(np.uint32) if with_ts else None
    f = S.make_filters(B)
    f["all_bits"][1] = 1; f["none_bits"][2] = 6; f["any_bits"][3][0] = 0xF0; f["n_any"][3] = 1
    f["all_bits"][4] = 0xFFFFFFFF                                              # nothing passes
    f["all_bits"][5] = 0x3F                                                    # fewer than T pass
    if with_ts:
        f["ts_min"][6] = 100; f["ts_max"][6] = 500
    ids, mt, cnt = oracle_mod.bits_search(bits, k_bits, mask, qbits, f, T, ts=ts)
    want = py_bits_search(bits, k_bits, mask, ts, qbits, f, T, oracle_mod.passes)
    for b in range(B):
        assert cnt[b] == len(want[b])
        assert [(int(i), int(m)) for i, m in zip(ids[b, :cnt[b]], mt[b, :cnt[b]])] == want[b]
        assert np.all(ids[b, cnt[b]:] == 0xFFFFFFFF) and np.all(mt[b, cnt[b]:] == np.iinfo(np.int32).min)
    assert ids[0, :3].tolist() == [5, 17, 300] and mt[0, 0] == k_bits           # ties by ascending id
    assert cnt[4] == 0 and 0 < cnt[5] < T


def test_two_stage_reduces_to_the_exact_search_when_T_covers_everything(oracle_mod):
    """with T >= number of feasible items the first stage removes nothing: the result is the exact filtered top-k"""
    w = S.config1(n=3000, B=5, k=20)
    h = S.to_numpy(w)
    D = 64
    perm, signs = draw(31, D)
    ids, sc, cnt = oracle_mod.two_stage(S.F32, h["emb"], h["mask"], h["Q"], h["filters"], perm, signs, 64, 3000, 20)
    oi, os_, _, oc = oracle_mod.search(S.F32, h["emb"], h["mask"], h["Q"], h["filters"], 20)
    assert np.array_equal(ids, oi) and np.array_equal(cnt, oc) and sc.tobytes() == os_.tobytes()


def test_two_stage_is_a_subset_rescored(oracle_mod):
    """every returned id is one of the first stage's T candidates, ordered by its exact score"""
    w = S.config1(n=5000, B=4, k=10)
    h = S.to_numpy(w)
    perm, signs = draw(32, 64)
    T = 200
    ids, sc, cnt = oracle_mod.two_stage(S.F32, h["emb"], h["mask"], h["Q"], h["filters"], perm, signs, 64, T, 10)
    bits = oracle_mod.sign_oporp(S.F32, h["emb"], perm, signs, 64)
    qb = oracle_mod.sign_oporp(S.F32, h["Q"].reshape(4, 64), perm, signs, 64)
    ids1, _, c1 = oracle_mod.bits_search(bits, 64, h["mask"], qb, h["filters"], T)
    for b in range(4):
        assert set(ids[b, :cnt[b]].tolist()) <= set(ids1[b, :c1[b]].tolist())
        exact = (h["emb"][ids[b, :cnt[b]]].astype(np.float64) @ h["Q"][b, 0].astype(np.float64))
        assert np.allclose(exact, sc[b, :cnt[b]], rtol=1e-5, atol=1e-6)
        assert np.all(np.diff(sc[b, :cnt[b]]) <= 0)
