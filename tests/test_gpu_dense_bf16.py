"""The large-batch bf16 scan kernel (scan_kernel_dense_bf16: rows of 256 bytes, queries as the row operand, bounds
through the accumulator input; rows of 128 bytes with eight embeddings per query) against the oracle under the float
acceptance rule (Sec. 3.1; the batched regime of Sec. 5.3.2 on the benchmark's row shape, d = 128; the
multi-embedding score of Sec. 3.1.1)."""
import numpy as np
import pytest

import synth_inputs as S
from gpu_util import run_gpu, assert_float_rule, to_cuda

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def bf16_workload(seed, n, B, with_ts=False, clustered=False, filt="two bits", d=128, m=1):
    import torch
    g = torch.Generator().manual_seed(seed)
    if clustered:
        cen = S.l2_normalise(torch.randn(50, d, generator=g))
        emb = S.l2_normalise(cen[torch.randint(0, 50, (n,), generator=g)] + torch.randn(n, d, generator=g) * (0.3 / d ** 0.5))
        Q = S.l2_normalise(cen[torch.randint(0, 50, (B * m,), generator=g)] + torch.randn(B * m, d, generator=g) * (0.3 / d ** 0.5))
    else:
        emb = S.l2_normalise(torch.randn(n, d, generator=g)); Q = S.l2_normalise(torch.randn(B * m, d, generator=g))
    emb, Q = S.to_bf16_bits(emb), S.to_bf16_bits(Q.reshape(B, m, d))
    mask = S.bernoulli_masks(n, [0.5] * 32, "cpu", seed + 1)
    rng = np.random.default_rng(seed + 2)
    ts = torch.from_numpy(rng.integers(0, 1000, n).astype(np.uint32).view(np.int32)) if with_ts else None
    if filt == "two bits":
        f = S.required_bit_filters(B, 2, 0, 32, seed + 3)
    else:                                                   # mixed: pass-all, one bit, any-of groups, nothing passes, ~1 %
        f = S.make_filters(B)
        for b in range(B):
            kind = b % 5
            if kind == 1:
                f["all_bits"][b] = 1 << rng.integers(0, 32)
            elif kind == 2:
                f["any_bits"][b][0] = 0x0000F00F; f["any_bits"][b][1] = 1 << rng.integers(0, 32); f["n_any"][b] = 2
            elif kind == 3:
                f["all_bits"][b] = 0xFFFFFFFF
            elif kind == 4:
                f["all_bits"][b] = sum(1 << int(x) for x in rng.choice(32, 7, replace=False))
    if with_ts:
        f["ts_min"][1::2] = 200; f["ts_max"][1::2] = 800
    return dict(dtype=S.BF16, d=d, m=m, k=10, emb=emb, scale=None, mask=mask, ts=ts, Q=Q, q_scale=None, filters=f)


@pytest.mark.parametrize("n,B,k,with_ts,clustered,filt", [
    (60_000, 65, 100, False, False, "two bits"), (60_000, 128, 50, False, True, "mixed"), (100_003, 200, 300, True, False, "mixed"),
    (80_000, 256, 1000, False, True, "two bits"), (50_000, 300, 64, True, True, "two bits"), (40_000, 512, 100, False, False, "mixed"),
    (30_000, 700, 40, False, True, "mixed"), (1000, 256, 2000, False, False, "two bits"), (15, 100, 5, True, False, "mixed")])
def test_dense_bf16_float_rule(oracle_mod, n, B, k, with_ts, clustered, filt):
    """one, two and four query sets per workgroup, ragged item and query counts, several passes (B > 512), k > n,
    timestamps, clustered data (whole clusters tie closely), every kind of filter"""
    say(f"dense bf16 n={n} B={B} k={k} ts={with_ts} clustered={clustered} filters={filt}")
    w = bf16_workload(n + B, n, B, with_ts, clustered, filt)
    gpu = run_gpu(to_cuda(w), k=k)
    assert_float_rule(oracle_mod, w, gpu, k, label=f"dense bf16 n={n} B={B}")


@pytest.mark.parametrize("n,B,k,with_ts,clustered,filt", [
    (60_000, 33, 100, False, False, "two bits"), (60_000, 64, 50, False, True, "mixed"), (100_003, 100, 300, True, False, "mixed"),
    (80_000, 128, 500, False, True, "two bits"), (50_000, 129, 64, True, True, "two bits"), (30_000, 300, 40, False, True, "mixed"),
    (1000, 70, 2000, False, False, "two bits"), (15, 40, 5, True, False, "mixed")])
def test_dense_bf16_eight_embeddings_float_rule(oracle_mod, n, B, k, with_ts, clustered, filt):
    """rows of 128 bytes, eight embeddings per query (score = the largest of the eight dot products): one, two and four
    query sets, ragged counts, several passes (B > 128), k > n, timestamps, every kind of filter"""
    say(f"dense bf16 m=8 n={n} B={B} k={k} ts={with_ts} clustered={clustered} filters={filt}")
    w = bf16_workload(n + B, n, B, with_ts, clustered, filt, d=64, m=8)
    gpu = run_gpu(to_cuda(w), k=k)
    assert_float_rule(oracle_mod, w, gpu, k, label=f"dense bf16 m=8 n={n} B={B}")


def test_dense_bf16_eight_embeddings_small_batches_and_the_older_kernels(oracle_mod):
    """the kernel forced onto batches below its default threshold, and the same batch through the kernels it replaces"""
    w = bf16_workload(77, 90_000, 50, False, True, "two bits", d=64, m=8)
    dev = to_cuda(w)
    for B, tuning in ((50, None), (50, dict(no_dense=1)), (5, dict(dense_min_batch=1)), (32, dict(dense_min_batch=1))):
        say(f"dense bf16 m=8 B={B} tuning={tuning}")
        sub = dict(w); sub["Q"] = w["Q"][:B]; sub["filters"] = w["filters"][:B]
        dsub = dict(dev); dsub["Q"] = dev["Q"][:B].contiguous(); dsub["filters"] = dev["filters"][:B]
        gpu = run_gpu(dsub, k=150, tuning=tuning)
        assert_float_rule(oracle_mod, sub, gpu, 150, label=f"dense bf16 m=8 B={B} {tuning}")


def test_dense_bf16_agrees_with_the_cooperative_kernel(oracle_mod):
    """the same batch through both large-batch bf16 kernels: counts equal, id sets equal up to the tolerance band"""
    w = bf16_workload(99, 120_000, 256, False, True, "two bits")
    dev = to_cuda(w)
    a = run_gpu(dev, k=200)
    b = run_gpu(dev, k=200, tuning=dict(no_dense=1))
    assert np.array_equal(a[3], b[3])
    assert_float_rule(oracle_mod, w, a, 200, label="dense bf16")
    assert_float_rule(oracle_mod, w, b, 200, label="coop bf16")
    same = np.mean([len(set(a[0][q][:a[3][q]].tolist()) & set(b[0][q][:b[3][q]].tolist())) / max(1, a[3][q]) for q in range(256)])
    assert same > 0.999


def test_dense_bf16_compaction_and_forced_groups(oracle_mod):
    """ascending scores in one full sweep (segments fill and are compacted again and again); four groups per wave forced"""
    import torch
    n, B, k, d = 50_000, 130, 60, 128
    w = bf16_workload(5, n, B)
    base = S.l2_normalise(torch.randn(d, generator=torch.Generator().manual_seed(1)))
    x = base[None, :] * torch.linspace(0.2, 1.0, n)[:, None]               # scores of every query rise (or fall) with the id
    w["emb"] = S.to_bf16_bits(x)
    w["filters"] = S.make_filters(B)
    dev = to_cuda(w)
    for tuning in (dict(max_levels=1), dict(max_levels=1, dense_groups=4), dict(dense_groups=4)):
        gpu = run_gpu(dev, k=k, tuning=tuning)
        assert_float_rule(oracle_mod, w, gpu, k, label=f"dense bf16 compaction {tuning}")
