"""GPU parity of the quantised search (Sign-OPORP codes, bit matching, two-stage search) against the oracle.
Codes, match counts, ids and counts are integers: bit-exact.  The second stage's fp32 scores follow the 1e-3 rule."""
import time

import numpy as np
import pytest

import synth_inputs as S

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[{time.strftime('%H:%M:%S')}] {msg}", flush=True)


def mixed_filters(B, rng, with_ts):
    f = S.make_filters(B)
    for b in range(B):
        kind = b % 6
        if kind == 1:
            f["all_bits"][b] = 1 << rng.integers(0, 32)
        elif kind == 2:
            f["all_bits"][b] = (1 << rng.integers(0, 16)) | (1 << rng.integers(16, 32)); f["none_bits"][b] = 1 << rng.integers(0, 32)
        elif kind == 3:
            f["any_bits"][b][0] = 0x0000F00F; f["any_bits"][b][1] = 1 << rng.integers(0, 32); f["n_any"][b] = 2
        elif kind == 4:
            f["all_bits"][b] = 0xFFFFFFFF
        elif kind == 5:
            f["all_bits"][b] = sum(1 << int(x) for x in rng.choice(32, 6, replace=False))
        if with_ts and b % 2 == 1:
            f["ts_min"][b] = 200; f["ts_max"][b] = 800
    return f


def float_items(dtype, n, d, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n, d)).astype(np.float32)
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    if dtype == S.BF16:
        return S.to_bf16_bits_np(x) if hasattr(S, "to_bf16_bits_np") else (x.view(np.uint32) >> 16).astype(np.uint16)
    return x


@pytest.mark.parametrize("dtype,d,k_bits,reps", [(S.F32, 64, 64, 1), (S.F32, 128, 64, 1), (S.BF16, 256, 128, 1), (S.BF16, 64, 16, 1),
                                                 (S.F32, 512 // 4, 128, 1), (S.BF16, 192, 192, 1),
                                                 # codes longer than the embedding: independent draws, concatenated
                                                 (S.F32, 128, 512, 4), (S.BF16, 128, 512, 8), (S.BF16, 128, 384, 3), (S.F32, 64, 192, 3),
                                                 (S.BF16, 128, 256, 2), (S.F32, 64, 64, 2)])
def test_codes_match_the_oracle(oracle_mod, dtype, d, k_bits, reps):
    import torch
    import paper_2407_13218_amd as L
    say(f"codes dtype={dtype} d={d} k_bits={k_bits} draws={reps}")
    n = 3001
    x = float_items(dtype, n, d, d + k_bits)
    x[7] = 0                                                                   # a zero row: all bin sums zero
    perm, signs = S.oporp_draw(d, k_bits) if reps == 1 else S.oporp_draws(d, reps, k_bits)
    xt = torch.from_numpy(x.view(np.int16) if dtype == S.BF16 else x).cuda()
    mask = torch.zeros(n, dtype=torch.int32, device="cuda")
    ix = L.Index(n, d, dtype, 0)
    ix.load(xt, mask)
    ix.build_bits(perm, signs, k_bits)
    got = ix.quantize(xt).cpu().numpy().view(np.uint64)
    want = oracle_mod.sign_oporp(dtype, x, perm, signs, k_bits)
    assert np.array_equal(got, want)
    ix.close()


def run_bits_case(oracle_mod, codes, k_bits, mask, ts, qbits, filt, T, label, host_filters=True):
    import torch
    import paper_2407_13218_amd as L
    n = codes.shape[0]
    ix = L.Index(n, k_bits, S.BITS, 0)
    ix.load(torch.from_numpy(codes.view(np.int64)).cuda(), torch.from_numpy(mask.view(np.int32)).cuda(),
            ts=None if ts is None else torch.from_numpy(ts.view(np.int32)).cuda())
    f = filt if host_filters else torch.from_numpy(np.ascontiguousarray(filt).view(np.uint8).copy()).cuda()
    ids, mt, cnt = ix.search_bits(torch.from_numpy(qbits.view(np.int64)).cuda(), f, T)
    torch.cuda.synchronize()
    ids = ids.cpu().numpy().view(np.uint32); mt = mt.cpu().numpy(); cnt = cnt.cpu().numpy().view(np.uint32)
    oi, om, oc = oracle_mod.bits_search(codes, k_bits, mask, qbits, filt, T, ts=ts)
    assert np.array_equal(cnt, oc), f"{label}: counts {cnt} vs {oc}"
    assert np.array_equal(ids, oi), f"{label}: ids differ"
    assert np.array_equal(mt, om), f"{label}: match counts differ"
    ix.close()


@pytest.mark.parametrize("n,k_bits,B,T,with_ts", [(1, 64, 1, 1, False), (255, 64, 3, 10, False), (100_003, 64, 17, 1000, True),
                                                  (60_000, 128, 70, 500, False), (30_000, 256, 5, 2048, True),
                                                  (50_000, 32, 9, 100, False), (20_000, 192, 130, 64, False),
                                                  (400_000, 64, 3, 8192, False),
                                                  (40_000, 512, 9, 300, True), (30_000, 384, 70, 100, False), (25_000, 500, 3, 1000, False)])
def test_bits_search_exact(oracle_mod, n, k_bits, B, T, with_ts):
    say(f"bits search n={n} k_bits={k_bits} B={B} T={T} ts={with_ts}")
    rng = np.random.default_rng(n + B)
    codes = S.random_codes(n, k_bits, seed=n)
    qbits = S.random_codes(B, k_bits, seed=n + 1)
    if n > 100:
        codes[11] = qbits[0]; codes[3] = qbits[0]; codes[n - 1] = qbits[0]     # ties at the very top of query 0
    mask = rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32)
    ts = rng.integers(0, 1000, n).astype(np.uint32) if with_ts else None
    run_bits_case(oracle_mod, codes, k_bits, mask, ts, qbits, mixed_filters(B, rng, with_ts), T, f"n={n} k_bits={k_bits} B={B}")


@pytest.mark.parametrize("kernel", ["popcount", "matrix"])
@pytest.mark.parametrize("n,k_bits,B,T,with_ts", [(300, 64, 2, 20, False), (70_001, 64, 37, 700, True), (40_000, 128, 129, 300, False),
                                                  (25_000, 100, 16, 2500, True), (33_000, 17, 50, 90, False)])
def test_both_bit_matching_kernels(oracle_mod, kernel, n, k_bits, B, T, with_ts):
    """the same searches forced through the popcount kernel (vector ALU) and the matrix-core kernel (codes expanded to
    0 / 1 bytes, queries to +-1 bytes, accumulators started at the query's zero count); ragged code widths included"""
    import paper_2407_13218_amd as L
    say(f"bits search via the {kernel} kernel: n={n} k_bits={k_bits} B={B} T={T}")
    rng = np.random.default_rng(n + B + 1)
    codes = S.random_codes(n, k_bits, seed=n + 7)
    qbits = S.random_codes(B, k_bits, seed=n + 8)
    codes[n // 2] = qbits[0]; codes[n - 1] = qbits[0]; codes[0] = ~qbits[B - 1] & codes.dtype.type((1 << min(64, k_bits)) - 1 if k_bits <= 64 else 0xFFFFFFFFFFFFFFFF)
    if k_bits > 64 and k_bits % 64:
        codes[0, -1] &= np.uint64((1 << (k_bits % 64)) - 1)
    mask = rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32)
    ts = rng.integers(0, 1000, n).astype(np.uint32) if with_ts else None
    L.set_tuning(**({"no_coop": 1} if kernel == "popcount" else {"force_generic": 1}))
    try:
        run_bits_case(oracle_mod, codes, k_bits, mask, ts, qbits, mixed_filters(B, rng, with_ts), T, f"{kernel} n={n} k_bits={k_bits} B={B}")
    finally:
        L.set_tuning()


def test_bits_search_few_levels_many_ties(oracle_mod):
    """16-bit codes: only 17 distinct match counts, so the T-th place is decided by ids among thousands of ties"""
    say("bits search with 16-bit codes (massive ties), device filters, plan variants")
    import paper_2407_13218_amd as L
    rng = np.random.default_rng(3)
    n, B, T = 80_000, 6, 300
    codes = S.random_codes(n, 16, seed=5); qbits = S.random_codes(B, 16, seed=6)
    mask = rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32)
    f = mixed_filters(B, rng, False)
    run_bits_case(oracle_mod, codes, 16, mask, None, qbits, f, T, "16-bit codes", host_filters=False)
    for tuning in (dict(max_levels=1, blocks_per_cu=1), dict(sample_ratio=2, min_sample=64)):
        L.set_tuning(**tuning)
        try:
            run_bits_case(oracle_mod, codes, 16, mask, None, qbits, f, T, f"16-bit codes {tuning}")
        finally:
            L.set_tuning()


def verify_second_stage(oracle_mod, dtype, x, mask, q, f, oi1, oc1, k, ids, sc, cnt):
    """ids / sc / cnt of a two-stage search against the oracle's candidates (oi1 [B, T], oc1 [B]): the 1e-3 rule among
    the candidates, order, uniqueness, padding"""
    B = q.shape[0]
    # second stage: 1e-3 rule among the candidates
    rtol, atol = 1e-3, 1e-6
    for b in range(B):
        c = int(oc1[b]); kk = min(k, c)
        assert cnt[b] == kk, f"q{b}: count {cnt[b]} vs {kk}"
        assert np.all(ids[b, kk:] == S.NO_ID) and np.all(np.isneginf(sc[b, kk:]))
        if kk == 0:
            continue
        cand = oi1[b, :c].astype(np.uint64)
        rank, _, feas = oracle_mod.pairs(dtype, x, mask, q[:, None, :], f, np.full(c, b, np.uint32), cand)
        assert feas.all()
        exact = dict(zip(cand.tolist(), rank.tolist()))
        got = ids[b, :kk].tolist()
        assert len(set(got)) == kk and set(got) <= set(cand.tolist()), f"q{b}: ids outside the candidate set"
        err = np.abs(sc[b, :kk].astype(np.float64) - np.array([exact[i] for i in got]))
        assert np.all(err <= rtol * np.abs(sc[b, :kk]) + atol), f"q{b}: score error {err.max()}"
        assert np.all(np.diff(sc[b, :kk]) <= 0)
        same = np.diff(sc[b, :kk]) == 0
        assert np.all(np.diff(np.array(got, np.int64))[same] > 0)
        order = np.lexsort((cand, -rank))
        tau = rank[order][kk - 1]; band = rtol * abs(tau) + atol
        must = set(cand[order][rank[order] > tau + band].tolist())
        assert must <= set(got), f"q{b}: clearly better candidates missing"
        assert all(exact[i] >= tau - band for i in got), f"q{b}: returned a candidate below the band"


@pytest.mark.parametrize("dtype,d,k_bits,T,k,B", [(S.F32, 64, 64, 400, 50, 9), (S.BF16, 128, 64, 1000, 100, 9),
                                                  (S.F32, 64, 64, 2048, 2048, 9), (S.BF16, 64, 64, 8192, 3000, 9),
                                                  # more candidates than a ranking holds: selection + candidate scoring
                                                  (S.F32, 64, 64, 8193, 100, 9), (S.BF16, 128, 64, 30_000, 2000, 9),
                                                  (S.F32, 64, 64, 40_000, 500, 9), (S.BF16, 256, 128, 20_000, 8192, 9),
                                                  # more queries than one group of the selection path serves
                                                  (S.F32, 64, 64, 3000, 60, 41),
                                                  # 512-bit codes of 128-dimensional embeddings (four draws), both paths
                                                  (S.BF16, 128, 512, 600, 100, 9), (S.BF16, 128, 512, 12_000, 1000, 9),
                                                  (S.F32, 64, 384, 2000, 200, 5)])
@pytest.mark.parametrize("rank_max", [0, 8192])
def test_two_stage_against_the_oracle(oracle_mod, dtype, d, k_bits, T, k, B, rank_max):
    """rank_max = 8192 forces the ranking path (candidates ranked by linr_search_bits, re-scoring kernel) for every
    T it can serve; the default takes the selection path from T = 1000 on"""
    import torch
    import paper_2407_13218_amd as L
    if rank_max and T > L.MAX_K:
        pytest.skip("only the selection path serves this T")
    say(f"two-stage dtype={dtype} d={d} k_bits={k_bits} T={T} k={k} rank_max={rank_max}")
    n = 40_000
    rng = np.random.default_rng(T + k)
    x = float_items(dtype, n, d, 77)
    q = float_items(dtype, B, d, 78)
    mask = rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32)
    f = mixed_filters(B, rng, False)
    perm, signs = S.oporp_draw(d, 1) if k_bits <= d else S.oporp_draws(d, k_bits // min(d, 128), 1)
    as_t = (lambda a: torch.from_numpy(a.view(np.int16)).cuda()) if dtype == S.BF16 else (lambda a: torch.from_numpy(a).cuda())
    ix = L.Index(n, d, dtype, 0)
    ix.load(as_t(x), torch.from_numpy(mask.view(np.int32)).cuda())
    ix.build_bits(perm, signs, k_bits)
    L.set_tuning(two_stage_rank_max=rank_max)
    try:
        ids, sc, cnt = ix.search_two_stage(as_t(q), f, T, k)
        torch.cuda.synchronize()
    finally:
        L.set_tuning()
    ids = ids.cpu().numpy().view(np.uint32); sc = sc.cpu().numpy(); cnt = cnt.cpu().numpy().view(np.uint32)
    # first stage, exactly: the candidate sets must be the oracle's
    qb = ix.quantize(as_t(q))
    bits = oracle_mod.sign_oporp(dtype, x, perm, signs, k_bits); qbo = oracle_mod.sign_oporp(dtype, q, perm, signs, k_bits)
    oi1, om1, oc1 = oracle_mod.bits_search(bits, k_bits, mask, qbo, f, T)
    if T <= L.MAX_K:
        i1, m1, c1 = ix.search_bits(qb, f, T)
        torch.cuda.synchronize()
        assert np.array_equal(i1.cpu().numpy().view(np.uint32), oi1) and np.array_equal(m1.cpu().numpy(), om1)
        assert np.array_equal(c1.cpu().numpy().view(np.uint32), oc1)
    else:
        i1, c1, _ = ix.select_bits(qb, f, T)
        torch.cuda.synchronize()
        i1 = i1.cpu().numpy().view(np.uint32); c1 = c1.cpu().numpy()
        for b in range(B):
            assert int(c1[b]) == int(oc1[b])
            assert np.array_equal(i1[b, :int(c1[b])], np.sort(oi1[b, :int(oc1[b])]))
    verify_second_stage(oracle_mod, dtype, x, mask, q, f, oi1, oc1, k, ids, sc, cnt)
    ix.close()


def test_quantised_argument_errors():
    import torch
    import paper_2407_13218_amd as L
    say("argument errors of the quantised calls")
    n, d = 1000, 64
    perm, signs = S.oporp_draw(d, 0)
    emb8 = torch.zeros((n, d), dtype=torch.int8, device="cuda"); mask = torch.zeros(n, dtype=torch.int32, device="cuda")
    ix8 = L.Index(n, d, S.I8, 0); ix8.load(emb8, mask)
    with pytest.raises(L.LinrError) as e:
        ix8.build_bits(perm, signs, 64)
    assert e.value.code == -3                                                  # element type mismatch
    ixf = L.Index(n, d, S.F32, 0); ixf.load(torch.zeros((n, d), device="cuda"), mask)
    with pytest.raises(L.LinrError) as e:
        ixf.build_bits(perm, signs, 48)                                        # 64 % 48 != 0
    assert e.value.code == -2
    p4, s4 = S.oporp_draws(d, 5, 0)
    with pytest.raises(L.LinrError) as e:
        ixf.build_bits(p4, s4, 320)                                            # 5 words: no kernel for that length
    assert e.value.code == -2
    with pytest.raises(L.LinrError) as e:
        ixf.build_bits(p4, s4, 128)                                            # 128 bits do not split into 5 draws
    assert e.value.code == -2
    ixf.k_bits = 64
    with pytest.raises(L.LinrError) as e:
        ixf.search_bits(torch.zeros((1, 1), dtype=torch.int64, device="cuda"), S.make_filters(1), 10)
    assert e.value.code == -6                                                  # no codes built yet
    ixf.build_bits(perm, signs, 64)
    with pytest.raises(L.LinrError) as e:
        ixf.search_two_stage(torch.zeros((1, d), device="cuda"), S.make_filters(1), 10, 20)   # k > T
    assert e.value.code == -4
    ix8.close(); ixf.close()
