"""GPU parity of the explicit pre-filtering strategy for bitmask / timestamp filters (linr_search_filtered_prefilter,
LiNR Sec. 3.1.2) against the oracle, through the C ABI: the same acceptance rules as for the masking strategy (int8
bit-exact, fp32 / bf16 within the tolerance rule), host and device filters, several groups of 32 queries, m > 1,
live updates, and agreement with linr_search_filtered on the same inputs."""
import time

import numpy as np
import pytest

import synth_inputs as S
from gpu_util import run_gpu, run_oracle, assert_exact, assert_float_rule, to_cuda, rand_int8_workload

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[{time.strftime('%H:%M:%S')}] {msg}", flush=True)


@pytest.mark.parametrize("scaled", [True, False])
@pytest.mark.parametrize("n,B,k,host_filters", [(1, 1, 1, True), (1000, 17, 100, False), (100_003, 40, 1000, True),
                                                (300_000, 3, 5000, False), (50_000, 70, 64, True)])
def test_int8_exact_by_prefiltering(oracle_mod, scaled, n, B, k, host_filters):
    say(f"pre-filtering int8 scaled={scaled} n={n} B={B} k={k}")
    w = rand_int8_workload(300 + n % 89 + B, n, 64, B, scaled=scaled, with_ts=(B % 2 == 1))
    gpu = run_gpu(to_cuda(w), k=k, prefilter=True, host_filters=host_filters)
    assert_exact(gpu, run_oracle(oracle_mod, w, k), f"pre-filtering int8 n={n} B={B} k={k}")


@pytest.mark.parametrize("phases", [2, 3])
@pytest.mark.parametrize("n,B,k", [(700_001, 5, 300), (2_000_000, 33, 1000), (513, 2, 10)])
def test_phase_plans(oracle_mod, phases, n, B, k):
    """the two- and the three-phase plan (the latter is the default only for very large indexes) on the same inputs"""
    import paper_2407_13218_amd as L
    say(f"pre-filtering in {phases} phases n={n} B={B} k={k}")
    w = rand_int8_workload(40 + B, n, 64, B, scaled=True, with_ts=(B == 5))
    L.set_tuning(prefilter_phases=phases)
    try:
        gpu = run_gpu(to_cuda(w), k=k, prefilter=True)
    finally:
        L.set_tuning()
    assert_exact(gpu, run_oracle(oracle_mod, w, k), f"pre-filtering, {phases} phases, n={n} B={B} k={k}")


@pytest.mark.parametrize("table_min", [1, 64])
@pytest.mark.parametrize("n,B,k,with_ts", [(200_003, 1, 100, True), (150_000, 7, 300, False), (90_001, 32, 1000, True),
                                           (60_000, 45, 64, False), (511, 33, 20, True)])
def test_clause_table_and_query_loop(oracle_mod, table_min, n, B, k, with_ts):
    """the all / none clauses of a group looked up in the byte table (forced from one query on) and tested query by query
    (table switched off): mixed filters incl. any-of groups, impossible ones and pass-all, timestamp windows, a ragged
    last group"""
    import paper_2407_13218_amd as L
    say(f"pre-filtering table_min={table_min} n={n} B={B} k={k} ts={with_ts}")
    w = rand_int8_workload(70 + B, n, 64, B, scaled=True, with_ts=with_ts)
    L.set_tuning(prefilter_table_min=table_min)
    try:
        gpu = run_gpu(to_cuda(w), k=k, prefilter=True)
    finally:
        L.set_tuning()
    assert_exact(gpu, run_oracle(oracle_mod, w, k), f"pre-filtering table_min={table_min} n={n} B={B}")


def test_borrowed_columns_must_be_aligned():
    """columns used in place (LINR_SRC_DEVICE_BORROW) have to be 16-byte aligned: the loader says so"""
    import torch
    import paper_2407_13218_amd as L
    w = rand_int8_workload(77, 4_000, 64, 2, scaled=True)
    g = to_cuda(w)
    big = torch.empty(g["mask"].numel() + 3, dtype=g["mask"].dtype, device="cuda")
    big[3:] = g["mask"]
    ix = L.Index(4_000, 64, S.I8, 0)
    with pytest.raises(L.LinrError):
        ix.load(g["emb"], big[3:], row_scale=g["scale"])
    ix.close()


def test_int8_multi_embedding_by_prefiltering(oracle_mod):
    w = rand_int8_workload(5, 30_000, 64, 9, m=3, scaled=True)
    gpu = run_gpu(to_cuda(w), k=200, prefilter=True)
    assert_exact(gpu, run_oracle(oracle_mod, w, 200), "pre-filtering m = 3")


def test_config1_fp32_by_prefiltering(oracle_mod):
    w = S.config1()
    gpu = run_gpu(to_cuda(w), prefilter=True)
    assert_float_rule(oracle_mod, w, gpu, w["k"], label="cfg1 pre-filtering")


def test_config2_shape_bf16_by_prefiltering(oracle_mod):
    w = S.config2(n=200_000, B=40, k=1000, p=0.3, chunk=100_000)           # 9 % of the items feasible
    gpu = run_gpu(to_cuda(w), prefilter=True)
    assert_float_rule(oracle_mod, w, gpu, w["k"], label="cfg2 pre-filtering")


def test_config3_shape_by_prefiltering(oracle_mod):
    w = S.config3(n=300_000, B=16, k=1000, chunk=100_000)                   # bit + timestamp window: 7 % feasible
    gpu = run_gpu(to_cuda(w), prefilter=True)
    assert_exact(gpu, run_oracle(oracle_mod, w), "cfg3 pre-filtering")


def test_with_live_updates_by_prefiltering(oracle_mod):
    """deleted slots are infeasible for this strategy too"""
    import torch
    import paper_2407_13218_amd as L
    rng = np.random.default_rng(8)
    n, cap, d, B, k = 20_000, 21_000, 64, 6, 150
    emb = rng.integers(-127, 128, (cap, d), dtype=np.int8)
    sc = rng.uniform(0.001, 0.02, cap).astype(np.float32)
    mask = rng.integers(0, 1 << 31, cap, dtype=np.uint32)
    Q = rng.integers(-127, 128, (B, 1, d), dtype=np.int8); qs = np.ones(B, np.float32)
    f = S.make_filters(B)
    f["all_bits"][1] = 5; f["none_bits"][2] = 8
    li = oracle_mod.LiveIndex(S.I8, d, cap, has_scale=True)
    li.load(emb[:n], mask[:n], scale=sc[:n])
    ix = L.Index(cap, d, S.I8, 0)
    ix.load(emb[:n], mask[:n], row_scale=sc[:n])
    ix.enable_updates()
    gone = rng.choice(n, 9000, replace=False).astype(np.uint32)
    fresh = np.arange(n, n + 700, dtype=np.uint32)
    li.delete(gone); ix.delete(gone)
    li.upsert(fresh, emb[fresh], mask[fresh], scale=sc[fresh]); ix.upsert(fresh, emb[fresh], mask[fresh], row_scale=sc[fresh])
    want = li.search(Q, f, k, q_scale=qs)
    for prefilter in (True, False):
        ids, scr, raw, cnt = ix.search(torch.from_numpy(Q).cuda(), f, k, q_scale=torch.from_numpy(qs).cuda(), prefilter=prefilter, strategy="masking")
        torch.cuda.synchronize()
        assert np.array_equal(cnt.cpu().numpy().view(np.uint32), want[3])
        assert np.array_equal(ids.cpu().numpy().view(np.uint32), want[0])
        assert scr.cpu().numpy().tobytes() == want[1].tobytes() and np.array_equal(raw.cpu().numpy(), want[2])
    ix.close()


def test_prefilter_argument_errors():
    import paper_2407_13218_amd as L
    w = to_cuda(rand_int8_workload(1, 500, 64, 3))
    ix = L.Index(500, 64, S.I8, 0)
    with pytest.raises(L.LinrError) as e:
        ix.search(w["Q"], w["filters"], 5, prefilter=True)
    assert e.value.code == -6
    ix.load(w["emb"], w["mask"], row_scale=w["scale"])
    with pytest.raises(L.LinrError) as e:
        ix.search(w["Q"], w["filters"], 0, prefilter=True)
    assert e.value.code == -4
    bad = w["filters"].copy(); bad["n_any"][1] = 9
    with pytest.raises(L.LinrError) as e:
        ix.search(w["Q"], bad, 5, prefilter=True)
    assert e.value.code == -9
    ix.close()
