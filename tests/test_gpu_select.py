"""GPU parity of the large-K selection by bit matching (linr_select_bits; LiNR Sec. 3.2 / the notification use case of
Sec. 5.3) against the oracle's stable sort, through the C ABI.  Everything is integer work: ids, counts and thresholds
are compared bit for bit (the selected set is unique: ties go to the lower id)."""
import time

import numpy as np
import pytest

import synth_inputs as S
from test_gpu_bits import mixed_filters

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[{time.strftime('%H:%M:%S')}] {msg}", flush=True)


def run_case(oracle_mod, codes, k_bits, mask, ts, qbits, filt, K, label, host_filters=True):
    import torch
    import paper_2407_13218_amd as L
    n, B = codes.shape[0], qbits.shape[0]
    ix = L.Index(n, k_bits, S.BITS, 0)
    ix.load(torch.from_numpy(codes.view(np.int64)).cuda(), torch.from_numpy(mask.view(np.int32)).cuda(),
            ts=None if ts is None else torch.from_numpy(ts.view(np.int32)).cuda())
    f = filt if host_filters else torch.from_numpy(np.ascontiguousarray(filt).view(np.uint8).copy()).cuda()
    ids, cnt, thr = ix.select_bits(torch.from_numpy(qbits.view(np.int64)).cuda(), f, K)
    torch.cuda.synchronize()
    ids = ids.cpu().numpy().view(np.uint32); cnt = cnt.cpu().numpy(); thr = thr.cpu().numpy()
    ix.close()
    want_ids, want_thr, want_cnt = oracle_mod.bits_select(codes, k_bits, mask, qbits, filt, K, ts=ts)
    assert np.array_equal(cnt.astype(np.uint64), want_cnt), f"{label}: counts {cnt[:8]} vs {want_cnt[:8]}"
    assert np.array_equal(thr, want_thr), f"{label}: thresholds {thr[:8]} vs {want_thr[:8]}"
    for b in range(B):
        assert np.array_equal(ids[b, :int(cnt[b])], want_ids[b]), f"{label}: ids of query {b} differ"


@pytest.mark.parametrize("n,k_bits,B,K,with_ts", [
    (1, 64, 1, 1, False), (5, 64, 2, 3, True),
    # one pass-all query: the mask column is skipped
    (100_000, 64, 1, 33_333, False), (100_001, 128, 1, 5, True),
    (1000, 64, 7, 100, False), (4099, 16, 3, 2000, True),
    (65_536, 64, 2, 30_000, False), (65_537, 64, 2, 65_537, False), (200_003, 128, 5, 77_777, True),
    (300_000, 256, 3, 150_000, False), (131_072, 200, 2, 1000, False), (1_000_000, 64, 13, 50_000, True),
    # three, six and eight words per code
    (120_000, 192, 2, 5000, False), (100_000, 384, 2, 999, True), (150_000, 512, 3, 40_000, False), (70_000, 450, 9, 35_000, True),
    # long codes whose cut lies beyond what the kept byte per item resolves (255 differing bits or more)
    (60_000, 512, 2, 55_000, False), (80_000, 384, 3, 79_000, True)])
def test_selection_matches_the_stable_sort(oracle_mod, n, k_bits, B, K, with_ts):
    say(f"select n={n} k_bits={k_bits} B={B} K={K} ts={with_ts}")
    rng = np.random.default_rng(n % 1000 + k_bits + B)
    codes = S.random_codes(n, k_bits, seed=n % 97)
    q = S.random_codes(B, k_bits, seed=1000 + B)
    mask = rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32)
    ts = rng.integers(0, 1000, n).astype(np.uint32) if with_ts else None
    run_case(oracle_mod, codes, k_bits, mask, ts, q, mixed_filters(B, rng, with_ts), K, f"n={n} k_bits={k_bits} K={K}",
             host_filters=(B % 2 == 1))


def test_long_runs_of_ties_across_segments(oracle_mod):
    """codes that differ from the query in a handful of bits only: the cut falls inside a run of several hundred
    thousand equal match counts that spans many 65536-item segments"""
    n, k_bits, B = 700_000, 64, 3
    rng = np.random.default_rng(3)
    q = S.random_codes(B, k_bits, seed=5)
    flips = rng.integers(0, 4, n)                                 # 0..3 differing bits from query 0
    codes = np.repeat(q[:1], n, axis=0).copy()
    for j in range(3):
        bit = rng.integers(0, 64, n).astype(np.uint64)
        codes[:, 0] ^= np.where(flips > j, np.uint64(1) << bit, np.uint64(0))
    mask = rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32)
    f = S.make_filters(B); f["all_bits"][1] = 1; f["none_bits"][2] = 6
    for K in (1, 170_000, 350_001, 699_999, 2_000_000):
        run_case(oracle_mod, codes, k_bits, mask, None, q, f, K, f"ties K={K}")


@pytest.mark.parametrize("k_bits", [64, 254, 255, 256])
def test_every_count_of_differing_bits(oracle_mod, k_bits):
    """items that differ from the query in exactly 0, 1, ..., k_bits bits (the full range, up to the complement of the
    query): 254 bits is the widest code whose counts are kept as bytes between the passes, 255 and 256 recompute them"""
    W = (k_bits + 63) // 64
    n = 3 * (k_bits + 1) + 2
    q = S.random_codes(1, k_bits, seed=k_bits)
    codes = np.repeat(q, n, axis=0).copy()
    for i in range(n):
        j = i % (k_bits + 1)                                      # flip the lowest j bits
        for w in range(W):
            nb = min(64, max(0, j - 64 * w))
            if nb:
                codes[i, w] ^= np.uint64((1 << nb) - 1)
    mask = np.ones(n, np.uint32)
    f = S.make_filters(1); f["all_bits"][0] = 1
    for K in (1, 4, n // 2, n - 1, n, n + 10):
        run_case(oracle_mod, codes, k_bits, mask, None, q, f, K, f"full range k_bits={k_bits} K={K}")


def test_nothing_feasible_and_everything_selected(oracle_mod):
    n, k_bits = 70_000, 64
    codes = S.random_codes(n, k_bits, seed=1); q = S.random_codes(2, k_bits, seed=2)
    mask = np.full(n, 2, np.uint32)
    f = S.make_filters(2); f["all_bits"][0] = 1                  # query 0: no item has bit 0; query 1: pass-all
    run_case(oracle_mod, codes, k_bits, mask, None, q, f, n + 5, "none / all")


def test_codes_of_a_float_index_and_live_updates(oracle_mod):
    """the selection over codes built by the library, with deleted and freshly added items"""
    import torch
    import paper_2407_13218_amd as L
    rng = np.random.default_rng(12)
    n, cap, d, k_bits, B, K = 90_000, 100_000, 128, 64, 3, 20_000
    x = rng.standard_normal((cap, d)).astype(np.float32)
    Q = rng.standard_normal((B, d)).astype(np.float32)
    mask = rng.integers(0, 1 << 31, cap, dtype=np.uint32)
    perm, signs = S.oporp_draw(d, k_bits)
    ix = L.Index(cap, d, S.F32, 0)
    ix.load(torch.from_numpy(x[:n]).cuda(), torch.from_numpy(mask[:n].view(np.int32)).cuda(), src=L.SRC_DEVICE_COPY)
    ix.build_bits(perm, signs, k_bits)
    ix.enable_updates()
    gone = rng.choice(n, 30_000, replace=False).astype(np.uint32)
    fresh = np.arange(n, n + 5_000, dtype=np.uint32)
    ix.delete(gone); ix.upsert(fresh, x[fresh], mask[fresh])
    ix.sync_updates()
    f = S.make_filters(B); f["all_bits"][1] = 4
    qb = ix.quantize(torch.from_numpy(Q).cuda())
    ids, cnt, thr = ix.select_bits(qb, f, K)
    torch.cuda.synchronize()
    live = np.ones(n + 5_000, bool); live[gone] = False
    codes = oracle_mod.sign_oporp(S.F32, x[:n + 5_000], perm, signs, k_bits)
    qcodes = oracle_mod.sign_oporp(S.F32, Q, perm, signs, k_bits)
    assert np.array_equal(qb.cpu().numpy().view(np.uint64), qcodes)
    dead_mask = np.where(live, mask[:n + 5_000], np.uint32(0x80000000) | mask[:n + 5_000])
    fo = f.copy(); fo["none_bits"] |= np.uint32(0x80000000)       # the oracle's way of saying "deleted items match nothing"
    want_ids, want_thr, want_cnt = oracle_mod.bits_select(codes, k_bits, dead_mask, qcodes, fo, K)
    assert np.array_equal(cnt.cpu().numpy().astype(np.uint64), want_cnt)
    assert np.array_equal(thr.cpu().numpy(), want_thr)
    got = ids.cpu().numpy().view(np.uint32)
    for b in range(B):
        assert np.array_equal(got[b, :int(want_cnt[b])], want_ids[b])
    ix.close()


def test_errors():
    import torch
    import paper_2407_13218_amd as L
    codes = S.random_codes(100, 64, seed=1)
    ix = L.Index(100, 64, S.BITS, 0)
    ix.load(torch.from_numpy(codes.view(np.int64)).cuda(), torch.zeros(100, dtype=torch.int32, device="cuda"))
    q = torch.from_numpy(S.random_codes(1, 64, seed=2).view(np.int64)).cuda()
    with pytest.raises(L.LinrError):
        ix.select_bits(q, S.make_filters(1), 0)
    nb = L.select_bits_workspace_bytes(ix.handle, 1)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    out = torch.empty((1, 10), dtype=torch.int32, device="cuda"); c = torch.empty(1, dtype=torch.int64, device="cuda")
    t = torch.empty(1, dtype=torch.int32, device="cuda")
    with pytest.raises(L.LinrError):                              # workspace too small
        L.select_bits(ix.handle, q, 1, S.make_filters(1), 10, out, c, t, ws, nb - 256, 0, L.FILTERS_ON_HOST)
    ix.close()
    fx = L.Index(10, 64, S.F32, 0)                                # no codes built
    fx.load(torch.zeros((10, 64), device="cuda"), torch.zeros(10, dtype=torch.int32, device="cuda"))
    with pytest.raises(L.LinrError):
        fx.select_bits(q, S.make_filters(1), 5)
    fx.close()


def test_empty_ts_window_without_a_ts_column_is_no_constraint(oracle_mod):
    """device filters are not validated: ts_min > ts_max matches nothing where the index has timestamps, and is not
    looked at where it has none -- as in the searches"""
    say("select: empty window without a ts column")
    n, k_bits, B = 50_000, 64, 4
    rng = np.random.default_rng(3)
    codes = S.random_codes(n, k_bits, seed=3)
    q = S.random_codes(B, k_bits, seed=4)
    mask = rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32)
    f = mixed_filters(B, rng, False)
    f["ts_min"][:] = 900
    f["ts_max"][:] = 100
    run_case(oracle_mod, codes, k_bits, mask, None, q, f, 5000, "empty window, no ts", host_filters=False)
