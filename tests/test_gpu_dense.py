"""GPU parity of the large-batch int8 kernel (rows of 64 bytes, m = 1; the default from 65 queries on) against the CPU
oracle, bit for bit: every number of query groups per wave (4, 8, 16) and of query sets per workgroup (1, 2, 4), scaled
and raw ranking, timestamps, any-of clauses, ragged ends, batches above one pass, queries without a usable bound,
segments that fill up and are compacted, and the degenerate plans the tests of the other kernels use."""
import os
import numpy as np
import pytest

import synth_inputs as S
from gpu_util import run_gpu, run_oracle, assert_exact, to_cuda, rand_int8_workload

pytestmark = pytest.mark.gpu
THREADS = max(1, min(16, os.cpu_count() or 1))


def say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("scaled", [True, False])
@pytest.mark.parametrize("n,B,k,ts", [(100_003, 65, 100, False), (60_000, 128, 1000, True), (200_077, 129, 500, False),
                                      (90_000, 256, 200, True), (150_001, 300, 1000, False), (70_000, 512, 64, False),
                                      (50_000, 700, 300, True), (40_000, 1024, 1000, False), (30_000, 1100, 50, False),
                                      (100, 200, 10, False), (127, 70, 200, True), (129, 1024, 5, False)])
def test_dense_exact(oracle_mod, scaled, n, B, k, ts):
    say(f"dense int8 scaled={scaled} n={n} B={B} k={k} ts={ts}")
    w = rand_int8_workload(300 + n % 89 + B, n, 64, B, scaled=scaled, with_ts=ts)
    gpu = run_gpu(to_cuda(w), k=k)
    assert_exact(gpu, run_oracle(oracle_mod, w, k, nthreads=THREADS), f"dense n={n} B={B} k={k}")


@pytest.mark.parametrize("min_batch,B", [(1, 3), (1, 40), (1, 64), (100, 99), (100, 100)])
def test_dense_group_counts_and_threshold(oracle_mod, min_batch, B):
    """four groups per wave (batches of at most 64 when the kernel is forced on them), and the switch-over point"""
    say(f"dense forced from B={min_batch}: B={B}")
    w = rand_int8_workload(400 + B, 80_000, 64, B, scaled=True, with_ts=(B % 2 == 0))
    gpu = run_gpu(to_cuda(w), k=150, tuning=dict(dense_min_batch=min_batch))
    assert_exact(gpu, run_oracle(oracle_mod, w, 150, nthreads=THREADS), f"dense forced B={B}")


@pytest.mark.parametrize("groups,B", [(4, 200), (8, 256), (8, 500), (12, 100), (16, 70), (4, 300)])
def test_dense_forced_groups_per_wave(oracle_mod, groups, B):
    """a given number of query groups per wave: the batch is then split into more (or fewer) query sets and passes"""
    say(f"dense with {groups} groups per wave, B={B}")
    w = rand_int8_workload(450 + B, 60_000, 64, B, scaled=True, with_ts=(groups == 8))
    gpu = run_gpu(to_cuda(w), k=120, tuning=dict(dense_groups=groups))
    assert_exact(gpu, run_oracle(oracle_mod, w, 120, nthreads=THREADS), f"dense groups={groups} B={B}")


@pytest.mark.parametrize("tuning", [dict(max_levels=1), dict(max_levels=1, blocks_per_cu=1), dict(sample_ratio=2, min_sample=64),
                                    dict(min_sample=1, sample_ratio=64), dict(no_top_split=1), dict(no_dense=1)])
def test_dense_degenerate_plans(oracle_mod, tuning):
    say(f"dense plan {tuning}")
    w = rand_int8_workload(500, 250_000, 64, 140, scaled=True)
    gpu = run_gpu(to_cuda(w), k=300, tuning=tuning)
    assert_exact(gpu, run_oracle(oracle_mod, w, 300, nthreads=THREADS), f"dense tuning {tuning}")


def test_dense_split_schedules_of_the_last_sweeps(oracle_mod):
    """from 65 536 chunks on the last sweeps are split by their own factors (halving by default for this kernel): the
    default and forced factor lists, on the smallest index that has the split, with a ragged end (one workload, one
    oracle run, every list against it)"""
    n, B, k = 65_536 * 128 + 77, 72, 200
    w = rand_int8_workload(520, n, 64, B, scaled=True)
    want = run_oracle(oracle_mod, w, k, nthreads=THREADS)
    dev = to_cuda(w)
    for code in (0, 0x442, 0x22222222, 0x84, 0x248):
        say(f"dense split schedule {code:#x} n={n} B={B}")
        gpu = run_gpu(dev, k=k, tuning=dict(top_ratios=code) if code else None)
        assert_exact(gpu, want, f"dense split schedule {code:#x}")


def test_dense_adversarial_order_forces_compaction(oracle_mod):
    """Scores increase with the item id, one full sweep, one workgroup per CU: every wave keeps meeting better items, so its
    queue overflows into the segments, the segments fill up and are compacted in flight."""
    import torch
    n, d, B, k = 400_000, 64, 70, 100
    rng = np.random.default_rng(6)
    level = (np.arange(n) * 120 // n).astype(np.int8)[:, None]
    emb = torch.from_numpy((level + rng.integers(0, 2, (n, d), dtype=np.int8)).astype(np.int8))
    Q = torch.from_numpy(np.ones((B, 1, d), np.int8))
    mask = torch.from_numpy(rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32).view(np.int32))
    f = S.make_filters(B); f["all_bits"][1] = 1; f["all_bits"][2] = 3; f["none_bits"][3] = 4
    for scaled in (False, True):
        say(f"dense adversarial ascending order, scaled={scaled}")
        scale = torch.from_numpy(rng.uniform(0.9, 1.1, n).astype(np.float32)) if scaled else None
        w = dict(dtype=S.I8, d=d, m=1, k=k, emb=emb, scale=scale, mask=mask, ts=None, Q=Q, q_scale=None, filters=f)
        gpu = run_gpu(to_cuda(w), k=k, tuning=dict(max_levels=1, blocks_per_cu=1))
        assert_exact(gpu, run_oracle(oracle_mod, w, k, nthreads=THREADS), f"dense adversarial scaled={scaled}")


def test_dense_wide_spread_of_row_scales_and_signs(oracle_mod):
    """row scales over three orders of magnitude (the first test works from the largest one), zero scales, negative and
    zero bounds (queries whose best items score below zero), identical rows"""
    import torch
    n, B, k = 120_000, 96, 400
    rng = np.random.default_rng(8)
    w = rand_int8_workload(601, n, 64, B, scaled=True)
    sc = np.exp(rng.uniform(np.log(1e-3), np.log(2.0), n)).astype(np.float32)
    sc[rng.integers(0, n, 500)] = 0.0
    w["scale"] = torch.from_numpy(sc)
    w["Q"][: B // 3] = -torch.abs(w["Q"][: B // 3])                      # all-negative queries ...
    w["emb"][:, :] = torch.abs(w["emb"])                                 # ... against all-positive items: every score <= 0
    w["emb"][1000:1200] = w["emb"][1000]                                  # identical rows
    say("dense: wide spread of row scales, non-positive scores")
    gpu = run_gpu(to_cuda(w), k=k)
    assert_exact(gpu, run_oracle(oracle_mod, w, k, nthreads=THREADS), "dense scale spread")


def test_dense_device_filters_and_repeatability(oracle_mod):
    say("dense: device-resident filters, repeated calls")
    w = rand_int8_workload(23, 180_000, 64, 200, scaled=True, with_ts=True)
    wc = to_cuda(w)
    first = run_gpu(wc, k=256, host_filters=False)
    assert_exact(first, run_oracle(oracle_mod, w, 256, nthreads=THREADS), "dense device filters")
    for _ in range(3):
        again = run_gpu(wc, k=256, host_filters=False)
        for a, b in zip(first, again):
            assert np.array_equal(a, b)
