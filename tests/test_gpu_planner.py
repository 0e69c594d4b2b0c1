"""The planner behind linr_search_filtered (Sec. 3.1.2: masking or explicit pre-filtering; Sec. 5.3.1 - 5.3.2 for the
trade-off): its choice at the two ends of the pass-rate range, its estimate of the feasible pairs, and bit-identical
results with the oracle through its choice and through both forced strategies."""
import numpy as np
import pytest

import synth_inputs as S
from gpu_util import run_gpu, run_oracle, assert_exact, to_cuda, rand_int8_workload

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def workload(B, bits_of_query, seed=77, n=300_000):
    """int8 rows of 64 bytes with per-row scales; mask bits 0-7 set with probability 0.5, 8-15 with 0.2, 16-23 with 0.03"""
    import torch
    w = rand_int8_workload(seed, n, 64, B, scaled=True)
    rng = np.random.default_rng(seed + 1)
    p = np.array([0.5] * 8 + [0.2] * 8 + [0.03] * 8 + [0.5] * 8)
    bits = rng.random((n, 32)) < p
    mask = (bits.astype(np.uint64) << np.arange(32, dtype=np.uint64)).sum(axis=1).astype(np.uint32)
    w["mask"] = torch.from_numpy(mask.view(np.int32))
    f = S.make_filters(B)
    for b in range(B):
        f["all_bits"][b] = np.uint32(sum(1 << int(x) for x in bits_of_query(b, rng)))
    w["filters"] = f
    return w, mask


@pytest.mark.parametrize("B", [8, 96])
def test_planner_choice_and_parity_both_ways(oracle_mod, B):
    import paper_2407_13218_amd as L
    k = 50
    low = lambda b, rng: rng.choice(np.arange(16, 24), 2, replace=False)          # ~0.09 % of the items pass
    high = lambda b, rng: [int(rng.integers(0, 8))]                                  # ~50 %
    for name, pick, want in (("low", low, L.STRATEGY_PREFILTER), ("high", high, L.STRATEGY_MASKING)):
        w, mask = workload(B, pick)
        dev = to_cuda(w)
        ix = L.Index(w["emb"].shape[0], 64, S.I8, 0)
        ix.load(dev["emb"], dev["mask"], row_scale=dev["scale"])
        strategy, pairs = L.plan_filtered(ix.handle, w["filters"], B, 1, k)
        ix.close()
        true_pairs = sum(int(((mask & f) == f).sum()) for f in w["filters"]["all_bits"])
        say(f"planner B={B} pass {name}: strategy {strategy}, estimated pairs {pairs:.0f}, true {true_pairs}")
        assert strategy == want
        assert abs(pairs - true_pairs) <= 0.25 * true_pairs + 200
        ora = run_oracle(oracle_mod, w, k)
        for strat in ("auto", "masking", "prefilter"):
            assert_exact(run_gpu(dev, k=k, strategy=strat), ora, f"planner {name} B={B} {strat}")
        # filters in device memory: the planner cannot read them and masks; forcing still works
        assert_exact(run_gpu(dev, k=k, strategy="auto", host_filters=False), ora, f"planner {name} B={B} device filters")
        assert_exact(run_gpu(dev, k=k, strategy="prefilter", host_filters=False), ora, f"planner {name} B={B} device filters, forced")


def test_planner_flags_and_small_workspace(oracle_mod):
    import torch
    import paper_2407_13218_amd as L
    B, k = 8, 20
    w, _ = workload(B, lambda b, rng: rng.choice(np.arange(16, 24), 2, replace=False), seed=5, n=100_000)
    dev = to_cuda(w)
    ora = run_oracle(oracle_mod, w, k)
    ix = L.Index(w["emb"].shape[0], 64, S.I8, 0)
    ix.load(dev["emb"], dev["mask"], row_scale=dev["scale"])
    ids = torch.empty((B, k), dtype=torch.int32, device="cuda"); sc = torch.empty((B, k), dtype=torch.float32, device="cuda")
    raw = torch.empty((B, k), dtype=torch.int32, device="cuda"); cnt = torch.empty((B,), dtype=torch.int32, device="cuda")
    small = ix.workspace_bytes(B, 1, k)
    big = ix.planned_workspace_bytes(B, 1, k)
    assert big > small                                       # (else the next case would not test anything)
    ws = torch.empty(big, dtype=torch.uint8, device="cuda")
    Q = dev["Q"]
    # the planner wants pre-filtering here, the workspace only covers masking: it masks, and the answer is the same
    L.search_filtered(ix.handle, Q, dev["q_scale"], B, 1, w["filters"], k, ids, sc, raw, cnt, ws, small, 0, L.FILTERS_ON_HOST)
    torch.cuda.synchronize()
    assert_exact((ids.cpu().numpy().view(np.uint32), sc.cpu().numpy(), raw.cpu().numpy(), cnt.cpu().numpy().view(np.uint32)), ora, "small workspace")
    # forcing pre-filtering with that workspace is an error, as is forcing both
    with pytest.raises(L.LinrError):
        L.search_filtered(ix.handle, Q, dev["q_scale"], B, 1, w["filters"], k, ids, sc, raw, cnt, ws, small, 0, L.FILTERS_ON_HOST | L.PLAN_PREFILTER)
    with pytest.raises(L.LinrError):
        L.search_filtered(ix.handle, Q, dev["q_scale"], B, 1, w["filters"], k, ids, sc, raw, cnt, ws, big, 0,
                          L.FILTERS_ON_HOST | L.PLAN_PREFILTER | L.PLAN_MASKING)
    ix.close()
