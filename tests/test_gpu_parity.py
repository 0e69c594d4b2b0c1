"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element."""
import json
import os
import numpy as np
import pytest

import synth_inputs as S
from gpu_util import run_gpu, run_oracle, assert_exact, assert_float_rule, to_cuda, rand_int8_workload

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


def say(msg):
    print(msg, flush=True)


def hand_workload(dtype, scaled=False):
    import torch
    g = json.load(open(os.path.join(HERE, "golden", "hand_example.json")))
    d = {S.F32: 4, S.BF16: 8, S.I8: 16}[dtype]                 # zero-padded so that a row is 16 bytes
    items = np.zeros((6, d), np.float32); items[:, :2] = g["items"]
    q = np.zeros((1, 1, d), np.float32); q[0, 0, :2] = g["query"]
    if dtype == S.I8:
        emb, Q = torch.from_numpy(items.astype(np.int8)), torch.from_numpy(q.astype(np.int8))
    elif dtype == S.BF16:
        emb, Q = S.to_bf16_bits(torch.from_numpy(items)), S.to_bf16_bits(torch.from_numpy(q))
    else:
        emb, Q = torch.from_numpy(items), torch.from_numpy(q)
    mask = torch.from_numpy(np.array(g["masks"], np.uint32).view(np.int32))
    scale = torch.tensor(g["row_scales_for_scaled_case"], dtype=torch.float32) if scaled else None
    return g, dict(dtype=dtype, d=d, m=1, k=3, emb=emb, scale=scale, mask=mask, ts=None, Q=Q, q_scale=None,
                   filters=S.make_filters(1))


@pytest.mark.parametrize("dtype", [S.I8, S.BF16, S.F32])
def test_hand_example_on_gpu(dtype):
    g, w = hand_workload(dtype)
    w = to_cuda(w)
    for c in g["cases"]:
        say(f"hand example dtype={dtype} case={c['name']}")
        f = S.make_filters(1)
        f["all_bits"] = c["all_bits"]; f["none_bits"] = c["none_bits"]
        for i, x in enumerate(c["any_bits"]):
            f["any_bits"][0][i] = x
        f["n_any"] = len(c["any_bits"])
        w["filters"] = f
        ids, sc, raw, cnt = run_gpu(w, k=c["k"])
        n = c["count"]
        assert cnt[0] == n and ids[0, :n].tolist() == c["ids"] and sc[0, :n].tolist() == [float(x) for x in c["scores"]]
        assert np.all(ids[0, n:] == S.NO_ID) and np.all(np.isneginf(sc[0, n:]))
    if dtype == S.I8:
        g, w = hand_workload(S.I8, scaled=True)
        w = to_cuda(w); c = g["scaled_int8_case"]
        w["filters"]["all_bits"] = c["all_bits"]
        ids, sc, raw, cnt = run_gpu(w, k=c["k"])
        assert ids[0].tolist() == c["ids"] and raw[0].tolist() == c["raw"] and sc[0].tolist() == [float(x) for x in c["rank"]]


@pytest.mark.parametrize("scaled", [True, False])
@pytest.mark.parametrize("n,B,k", [(1, 1, 1), (63, 3, 2), (1000, 17, 100), (100_003, 16, 1000), (50_000, 40, 2048),
                                   (300_000, 1, 1000), (20_000, 130, 500), (200_000, 4, 5000), (1_000_000, 2, 8192),
                                   (6_000, 33, 8192)])
def test_int8_exact(oracle_mod, scaled, n, B, k):
    say(f"int8 exact scaled={scaled} n={n} B={B} k={k}")
    w = rand_int8_workload(100 + n % 97 + B, n, 64, B, scaled=scaled, with_ts=(B % 2 == 1))
    gpu = run_gpu(to_cuda(w), k=k)
    assert_exact(gpu, run_oracle(oracle_mod, w, k), f"int8 n={n} B={B} k={k}")


def test_int8_small_range_many_ties(oracle_mod):
    say("int8 ties")
    w = rand_int8_workload(7, 40_000, 64, 20, scaled=False, lo=-1, hi=1)      # scores in a tiny range: ties everywhere
    gpu = run_gpu(to_cuda(w), k=700)
    assert_exact(gpu, run_oracle(oracle_mod, w, 700), "ties")


def test_config1_fp32(oracle_mod):
    say("config 1 (fp32, N=100k, B=16, k=100)")
    w = S.config1()
    gpu = run_gpu(to_cuda(w))
    assert_float_rule(oracle_mod, w, gpu, w["k"], label="cfg1")


def test_config2_shape_bf16(oracle_mod):
    say("config 2 shape (bf16 d=128), N=200k, B=40, k=1000")
    w = S.config2(n=200_000, B=40, k=1000, p=0.5, chunk=100_000)
    gpu = run_gpu(to_cuda(w))
    assert_float_rule(oracle_mod, w, gpu, w["k"], label="cfg2")


def test_config2_shape_bf16_large_k(oracle_mod):
    say("config 2 shape (bf16 d=128), N=300k, B=6, k=7000")
    w = S.config2(n=300_000, B=6, k=7000, p=0.9, chunk=100_000)
    gpu = run_gpu(to_cuda(w))
    assert_float_rule(oracle_mod, w, gpu, w["k"], label="cfg2 k=7000")


def test_config3_shape_int8_ts(oracle_mod):
    say("config 3 shape (int8 + ts window), N=300k, B=64, k=1000")
    w = S.config3(n=300_000, B=64, k=1000, chunk=100_000)
    gpu = run_gpu(to_cuda(w))
    assert_exact(gpu, run_oracle(oracle_mod, w), "cfg3")


def test_config4_shape_multi_embedding(oracle_mod):
    say("config 4 shape (bf16 d=64, m=8), N=100k, B=20, k=500")
    w = S.config4(n=100_000, B=20, k=500, chunk=50_000)
    gpu = run_gpu(to_cuda(w))
    assert_float_rule(oracle_mod, w, gpu, w["k"], label="cfg4")


def test_config5_shape_int8_all_selectivities(oracle_mod):
    import torch
    idx = None
    for sel in ("50%", "5%", "0.1%"):
        for B in (1, 32, 256):
            say(f"config 5 shape N=400k sel={sel} B={B}")
            w = S.config5(n=400_000, B=B, k=1000, selectivity=sel, C=100, chunk=200_000, index=idx)
            idx = (w["emb"], w["scale"], w["mask"])
            gpu = run_gpu(to_cuda(w))
            assert_exact(gpu, run_oracle(oracle_mod, w), f"cfg5 {sel} B={B}")


@pytest.mark.parametrize("tuning", [dict(max_levels=1), dict(sample_ratio=2, min_sample=64), dict(sample_ratio=4, min_sample=256, blocks_per_cu=1),
                                    dict(sample_ratio=64, min_sample=1)])
def test_sweep_plans_give_identical_results(oracle_mod, tuning):
    say(f"plan variants {tuning}")
    w = rand_int8_workload(11, 150_000, 64, 24, scaled=True)
    gpu = run_gpu(to_cuda(w), k=300, tuning=tuning)
    assert_exact(gpu, run_oracle(oracle_mod, w, 300), f"tuning {tuning}")


def test_adversarial_order_forces_segment_compaction(oracle_mod):
    """Scores increase with the item id, one full sweep, one workgroup per CU: every wave keeps meeting better
    items, so its candidate segments fill up and are compacted in flight."""
    import torch
    say("adversarial ascending order")
    n, d, B, k = 400_000, 64, 5, 100
    rng = np.random.default_rng(5)
    base = rng.integers(1, 4, (1, d), dtype=np.int8)
    level = (np.arange(n) * 120 // n).astype(np.int8)[:, None]                      # slowly growing rows
    emb = torch.from_numpy((base * 0 + level + rng.integers(0, 2, (n, d), dtype=np.int8)).astype(np.int8))
    Q = torch.from_numpy(np.ones((B, 1, d), np.int8))
    mask = torch.from_numpy(rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32).view(np.int32))
    f = S.make_filters(B); f["all_bits"][1] = 1; f["all_bits"][2] = 3; f["none_bits"][3] = 4
    w = dict(dtype=S.I8, d=d, m=1, k=k, emb=emb, scale=None, mask=mask, ts=None, Q=Q, q_scale=None, filters=f)
    gpu = run_gpu(to_cuda(w), k=k, tuning=dict(max_levels=1, blocks_per_cu=1))
    assert_exact(gpu, run_oracle(oracle_mod, w, k), "adversarial")
    w["scale"] = torch.from_numpy(rng.uniform(0.9, 1.1, n).astype(np.float32))
    gpu = run_gpu(to_cuda(w), k=k, tuning=dict(max_levels=1, blocks_per_cu=1))
    assert_exact(gpu, run_oracle(oracle_mod, w, k), "adversarial scaled")


def test_identical_rows_and_duplicates(oracle_mod):
    import torch
    say("identical rows")
    n, d = 70_000, 64
    emb = torch.from_numpy(np.tile(np.arange(-32, 32, dtype=np.int8), (n, 1)))
    mask = torch.from_numpy((np.arange(n) % 3 == 0).astype(np.uint32).view(np.int32))
    f = S.make_filters(2); f["all_bits"][0] = 1
    w = dict(dtype=S.I8, d=d, m=1, k=50, emb=emb, scale=None, mask=mask, ts=None,
             Q=torch.from_numpy(np.ones((2, 1, d), np.int8)), q_scale=None, filters=f)
    gpu = run_gpu(to_cuda(w), k=50)
    assert gpu[0][0].tolist() == list(range(0, 150, 3)) and gpu[0][1].tolist() == list(range(50))
    assert_exact(gpu, run_oracle(oracle_mod, w, 50), "identical")


def test_device_filters_and_repeatability(oracle_mod):
    say("device-resident filters, repeated calls")
    w = rand_int8_workload(21, 120_000, 64, 33, scaled=True, with_ts=True)
    wc = to_cuda(w)
    first = run_gpu(wc, k=256, host_filters=False)
    assert_exact(first, run_oracle(oracle_mod, w, 256), "device filters")
    for _ in range(4):
        again = run_gpu(wc, k=256, host_filters=False)
        for a, b in zip(first, again):
            assert np.array_equal(a, b)


@pytest.mark.parametrize("n,d,B,m,k,scaled", [(30_000, 64, 5, 2, 100, True), (9_000, 128, 20, 3, 64, False), (5_000, 16, 7, 8, 2048, True),
                                              (2_000, 512, 3, 1, 10, True), (40_000, 48, 50, 1, 300, True)])
def test_int8_shapes_served_by_the_lds_kernel(oracle_mod, n, d, B, m, k, scaled):
    """shapes without a register-resident kernel (m > 1, d != 64) stream their queries from LDS"""
    say(f"int8 lds kernel n={n} d={d} B={B} m={m} k={k} scaled={scaled}")
    w = rand_int8_workload(31 + d + m, n, d, B, m=m, scaled=scaled, with_ts=(m == 2), lo=-20, hi=20)
    gpu = run_gpu(to_cuda(w), k=k)
    assert_exact(gpu, run_oracle(oracle_mod, w, k), f"lds int8 d={d} m={m}")


def test_forced_lds_kernel_equals_register_kernel(oracle_mod):
    say("forced lds kernel vs register kernel")
    w = rand_int8_workload(77, 90_000, 64, 70, scaled=True, with_ts=True)
    wc = to_cuda(w)
    a = run_gpu(wc, k=500)
    b = run_gpu(wc, k=500, tuning=dict(force_generic=1))
    ora = run_oracle(oracle_mod, w, 500)
    assert_exact(a, ora, "register kernel"); assert_exact(b, ora, "lds kernel")


@pytest.mark.parametrize("dtype,d,m", [(S.F32, 16, 1), (S.F32, 128, 2), (S.BF16, 32, 1), (S.BF16, 256, 1), (S.BF16, 64, 3)])
def test_float_shapes_served_by_the_lds_kernel(oracle_mod, dtype, d, m):
    import torch
    say(f"float lds kernel dtype={dtype} d={d} m={m}")
    n, B, k = 25_000, 9, 200
    g = torch.Generator().manual_seed(d * 10 + m)
    emb = S.l2_normalise(torch.randn(n, d, generator=g)); Q = S.l2_normalise(torch.randn(B, m, d, generator=g))
    if dtype == S.BF16:
        emb, Q = S.to_bf16_bits(emb), S.to_bf16_bits(Q)
    mask = S.bernoulli_masks(n, [0.5] * 32, "cpu", 5)
    w = dict(dtype=dtype, d=d, m=m, k=k, emb=emb, scale=None, mask=mask, ts=None, Q=Q, q_scale=None,
             filters=S.required_bit_filters(B, 2, 0, 32, 3))
    gpu = run_gpu(to_cuda(w), k=k)
    assert_float_rule(oracle_mod, w, gpu, k, label=f"lds float d={d} m={m}")


@pytest.mark.parametrize("tuning", [dict(wide_min_batch=65), dict(coop_min_groups=2), dict(no_coop=1, max_qg=4), dict(no_coop=1, max_qg=16)])
def test_kernel_families_agree_on_a_large_batch(oracle_mod, tuning):
    """the same 200-query batch through the 32x32-tile kernel, the 16x16-tile workgroup-cooperative kernel, split
    over several waves per chunk, and with 16 query groups in one wave"""
    say(f"kernel families {tuning}")
    w = rand_int8_workload(55, 60_000, 64, 200, scaled=True, with_ts=True)
    gpu = run_gpu(to_cuda(w), k=300, tuning=tuning)
    assert_exact(gpu, run_oracle(oracle_mod, w, 300), f"family {tuning}")


@pytest.mark.parametrize("n,d,B,k,scaled,with_ts", [(60_000, 64, 65, 100, False, False), (33_333, 128, 300, 200, True, False),
                                                    (20_001, 256, 130, 64, False, True), (40_000, 64, 600, 50, True, True),
                                                    (25_000, 128, 512, 100, True, False), (31, 64, 100, 40, True, False)])
def test_wide_tile_kernel_shapes(oracle_mod, n, d, B, k, scaled, with_ts):
    """32x32-tile kernel: one, two and four K-steps of 64 bytes, short rows, 1 / 2 / 4 query groups per wave, several
    passes, ragged item and query counts"""
    say(f"wide kernel n={n} d={d} B={B} k={k} scaled={scaled} ts={with_ts}")
    w = rand_int8_workload(n + B, n, d, B, scaled=scaled, with_ts=with_ts)
    gpu = run_gpu(to_cuda(w), k=k, tuning=dict(wide_min_batch=1))
    assert_exact(gpu, run_oracle(oracle_mod, w, k), f"wide n={n} d={d} B={B}")


def test_wide_tile_kernel_small_batch_and_compaction(oracle_mod):
    """forced for a 5-query batch; then ascending scores in one full sweep so that segments fill and are compacted"""
    import torch
    say("wide kernel forced, B=5; adversarial ascending order B=70")
    w = rand_int8_workload(77, 50_000, 64, 5, scaled=True)
    gpu = run_gpu(to_cuda(w), k=500, tuning=dict(wide_min_batch=1))
    assert_exact(gpu, run_oracle(oracle_mod, w, 500), "wide B=5")
    n, d, B, k = 300_000, 64, 70, 100
    rng = np.random.default_rng(6)
    level = (np.arange(n) * 120 // n).astype(np.int8)[:, None]
    emb = torch.from_numpy((level + rng.integers(0, 2, (n, d), dtype=np.int8)).astype(np.int8))
    Q = torch.from_numpy(np.ones((B, 1, d), np.int8))
    mask = torch.from_numpy(rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32).view(np.int32))
    f = S.make_filters(B); f["all_bits"][1] = 1; f["all_bits"][2] = 3; f["none_bits"][3] = 4
    scale = torch.from_numpy(rng.uniform(0.9, 1.1, n).astype(np.float32))
    w = dict(dtype=S.I8, d=d, m=1, k=k, emb=emb, scale=scale, mask=mask, ts=None, Q=Q, q_scale=None, filters=f)
    gpu = run_gpu(to_cuda(w), k=k, tuning=dict(max_levels=1, blocks_per_cu=1, wide_min_batch=1))
    assert_exact(gpu, run_oracle(oracle_mod, w, k), "wide adversarial scaled")


@pytest.mark.parametrize("d,B,n,k", [(128, 150, 60_000, 200), (64, 256, 45_001, 100), (32, 70, 30_000, 1000)])
def test_wide_tile_kernel_bf16(oracle_mod, d, B, n, k):
    """32x32-tile kernel on bf16 rows of 256, 128 and 64 bytes (cfg 2 generator with other shapes)"""
    say(f"wide kernel bf16 d={d} B={B} n={n} k={k}")
    w = S.config2(n=n, B=B, k=k, p=0.5, chunk=n, d=d)
    gpu = run_gpu(to_cuda(w), tuning=dict(wide_min_batch=1))
    assert_float_rule(oracle_mod, w, gpu, w["k"], label=f"wide bf16 d={d}")


def test_coop_kernel_bf16_and_multi_embedding(oracle_mod):
    say("coop kernel: bf16 d=128 B=150; bf16 d=64 m=8 B=40")
    w = S.config2(n=60_000, B=150, k=200, p=0.5, chunk=60_000)
    gpu = run_gpu(to_cuda(w), tuning=dict(coop_min_groups=2))
    assert_float_rule(oracle_mod, w, gpu, w["k"], label="coop bf16")
    w = S.config4(n=40_000, B=40, k=100, chunk=40_000)
    gpu = run_gpu(to_cuda(w), tuning=dict(coop_min_groups=2))
    assert_float_rule(oracle_mod, w, gpu, w["k"], label="coop bf16 m=8")


def test_batch_larger_than_one_pass(oracle_mod):
    say("B = 4200 (more than one pass of the register kernel)")
    w = rand_int8_workload(41, 3_000, 64, 4200, scaled=True)
    gpu = run_gpu(to_cuda(w), k=20)
    assert_exact(gpu, run_oracle(oracle_mod, w, 20), "B=4200")


def test_argument_errors_on_device():
    import torch
    import paper_2407_13218_amd as L
    say("argument errors")
    w = to_cuda(rand_int8_workload(1, 1000, 64, 2))
    ix = L.Index(1000, 64, S.I8, 0)
    with pytest.raises(L.LinrError) as e:
        ix.search(w["Q"], w["filters"], 10)
    assert e.value.code == -6                                   # nothing loaded yet
    with pytest.raises(L.LinrError) as e:
        L.index_load_fp32(ix.handle, w["emb"], w["mask"], None, 1000, L.SRC_DEVICE_BORROW)
    assert e.value.code == -3
    with pytest.raises(L.LinrError) as e:
        L.index_load_int8(ix.handle, w["emb"], w["scale"], w["mask"], None, 1001, L.SRC_DEVICE_BORROW)
    assert e.value.code == -5
    ix.load(w["emb"], w["mask"], row_scale=w["scale"])
    for k, code in ((0, -4), (L.MAX_K + 1, -4)):
        with pytest.raises(L.LinrError) as e:
            ix.search(w["Q"], w["filters"], k)
        assert e.value.code == code
    bad = w["filters"].copy(); bad["n_any"][1] = 5
    with pytest.raises(L.LinrError) as e:
        ix.search(w["Q"], bad, 10)
    assert e.value.code == -9
    bad = w["filters"].copy(); bad["ts_min"][0] = 5; bad["ts_max"][0] = 4
    with pytest.raises(L.LinrError) as e:
        ix.search(w["Q"], bad, 10)
    assert e.value.code == -9
    ids = torch.full((2, 10), 7, dtype=torch.int32, device="cuda")
    sc = torch.zeros((2, 10), device="cuda"); cnt = torch.zeros(2, dtype=torch.int32, device="cuda")
    ws = torch.empty(1024, dtype=torch.uint8, device="cuda")
    with pytest.raises(L.LinrError) as e:
        L.search_filtered(ix.handle, w["Q"], None, 2, 1, w["filters"], 10, ids, sc, None, cnt, ws, ws.numel(), 0, L.FILTERS_ON_HOST)
    assert e.value.code == -7
    torch.cuda.synchronize()
    assert torch.all(ids == 7)                                  # outputs untouched on error
    # host-sourced load (copied by the library) gives the same answer as the borrowed one
    a = ix.search(w["Q"], w["filters"], 10, q_scale=w["q_scale"])
    h = S.to_numpy(rand_int8_workload(1, 1000, 64, 2))
    ix2 = L.Index(1000, 64, S.I8, 0)
    ix2.load(h["emb"], h["mask"], row_scale=h["scale"])
    b = ix2.search(w["Q"], w["filters"], 10, q_scale=w["q_scale"])
    torch.cuda.synchronize()
    assert all(torch.equal(x, y) for x, y in zip(a, b) if x is not None)
    assert L.index_info(ix2.handle) == dict(n=1000, d=64, dtype=S.I8, has_ts=False, has_row_scale=True)
    ix.close(); ix2.close()


@pytest.mark.parametrize("tuning", [None, {"no_coop": 1}, {"max_qg": 2}, {"max_qg": 1}, {"force_generic": 1}, {"no_dense": 1}])
@pytest.mark.parametrize("B", [5, 40, 100])
def test_empty_ts_window_without_a_ts_column_is_ignored_by_every_kernel(oracle_mod, tuning, B):
    """filters in device memory are not validated; a window with ts_min > ts_max must then mean the same in every kernel
    the planner can pick: nothing, where the index has timestamps -- and no constraint at all where it has none"""
    from gpu_util import rand_int8_workload
    w = rand_int8_workload(4242 + B, 50_000, 64, B, scaled=True, with_ts=False)
    w["filters"]["ts_min"][::2] = 900
    w["filters"]["ts_max"][::2] = 100
    ora = run_oracle(oracle_mod, w, 30)
    dev = to_cuda(w)
    for strategy in ("masking", "prefilter"):
        assert_exact(run_gpu(dev, k=30, tuning=tuning, host_filters=False, strategy=strategy), ora,
                     f"empty window, no ts column, B={B}, {tuning}, {strategy}")
