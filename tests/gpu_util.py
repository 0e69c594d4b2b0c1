"""Helpers shared by the GPU parity tests: run a workload through the C ABI and compare
with the CPU oracle under the acceptance rule of each element type."""
import numpy as np

import synth_inputs as S


def run_gpu(w, k=None, tuning=None, want_raw=True, host_filters=True, prefilter=False, strategy="masking"):
    """w: workload dict of torch tensors already on the GPU (see synth_inputs).  strategy: "masking" (the scan kernels,
    what most tests are about), "prefilter" or "auto" (the planner of linr_search_filtered decides)."""
    import torch
    import paper_2407_13218_amd as L
    k = k or w["k"]
    if tuning is not None:
        L.set_tuning(**tuning)
    try:
        ix = L.Index(max(1, w["emb"].shape[0]), w["d"], w["dtype"], 0)
        ix.load(w["emb"], w["mask"], ts=w["ts"], row_scale=w["scale"])
        filt = w["filters"]
        if not host_filters:
            filt = torch.from_numpy(np.ascontiguousarray(filt).view(np.uint8).copy()).cuda()
        ids, sc, raw, cnt = ix.search(w["Q"], filt, k, q_scale=w["q_scale"], want_raw=want_raw, prefilter=prefilter, strategy=strategy)
        torch.cuda.synchronize()
        out = (ids.cpu().numpy().view(np.uint32), sc.cpu().numpy(),
               None if raw is None else raw.cpu().numpy(), cnt.cpu().numpy().view(np.uint32))
        ix.close()
        return out
    finally:
        if tuning is not None:
            L.set_tuning()


def run_oracle(oracle, w, k=None, nthreads=8):
    h = S.to_numpy(w)
    return oracle.search(w["dtype"], h["emb"], h["mask"], h["Q"], h["filters"], k or w["k"], row_scale=h["scale"],
                         ts=h["ts"], q_scale=h["q_scale"], nthreads=nthreads)


def assert_exact(gpu, ora, label=""):
    gi, gs, gr, gc = gpu
    oi, os_, or_, oc = ora
    assert np.array_equal(gc, oc), f"{label}: counts differ {gc[:8]} vs {oc[:8]}"
    bad = np.nonzero((gi != oi).any(axis=1))[0]
    assert bad.size == 0, f"{label}: ids differ for queries {bad[:8]}; first row gpu {gi[bad[0]][:8]} oracle {oi[bad[0]][:8]}"
    if gr is not None:
        assert np.array_equal(gr, or_), f"{label}: raw int32 scores differ"
    assert gs.tobytes() == os_.tobytes(), f"{label}: fp32 score bit patterns differ"


def assert_float_rule(oracle, w, gpu, k, rtol=1e-3, atol=1e-6, label=""):
    """counts equal; every returned id feasible with |s_gpu - s_o| <= rtol*|s_o| + atol; scores non-increasing with
    bit-equal neighbours in ascending id; id sets may differ from the oracle's only inside the tolerance band
    around the k-th score."""
    h = S.to_numpy(w)
    n = h["emb"].shape[0]
    gi, gs, _, gc = gpu
    kk = min(n, k + 256)
    oi, os_, _, oc = oracle.search(w["dtype"], h["emb"], h["mask"], h["Q"], h["filters"], kk, ts=h["ts"], nthreads=8)
    B = gi.shape[0]
    for b in range(B):
        c = int(gc[b])
        assert c == min(k, int(oc[b])), f"{label} q{b}: count {c} vs oracle {min(k, int(oc[b]))}"
        assert np.all(gi[b, c:] == S.NO_ID) and np.all(np.isneginf(gs[b, c:])), f"{label} q{b}: padding"
        if c == 0:
            continue
        ids = gi[b, :c].astype(np.uint64)
        assert len(set(ids.tolist())) == c, f"{label} q{b}: duplicate ids"
        rank, _, feas = oracle.pairs(w["dtype"], h["emb"], h["mask"], h["Q"], h["filters"], np.full(c, b), ids, ts=h["ts"])
        assert feas.all(), f"{label} q{b}: infeasible id returned"
        delta = rtol * np.abs(rank) + atol
        err = np.abs(gs[b, :c].astype(np.float64) - rank)
        assert np.all(err <= delta), f"{label} q{b}: score error {err.max()} (allowed {delta[err.argmax()]})"
        d = np.diff(gs[b, :c])
        assert np.all(d <= 0), f"{label} q{b}: scores increase"
        same = d == 0
        assert np.all(np.diff(ids.astype(np.int64))[same] > 0), f"{label} q{b}: equal scores not in ascending id"
        tau = float(os_[b, c - 1])                          # oracle's k-th (or last) score
        dt = rtol * abs(tau) + atol
        assert np.all(rank >= tau - dt), f"{label} q{b}: returned an item below the tolerance band"
        must = oi[b, :c][os_[b, :c] > tau + dt]
        missing = set(must.tolist()) - set(ids.tolist())
        assert not missing, f"{label} q{b}: clearly better items missing: {sorted(missing)[:5]}"


def to_cuda(w):
    import torch
    out = dict(w)
    for key in ("emb", "mask", "ts", "scale", "Q", "q_scale"):
        if w[key] is not None:
            out[key] = w[key].cuda().contiguous()
    return out


def rand_int8_workload(seed, n, d, B, m=1, scaled=True, with_ts=False, lo=-127, hi=127, filt_kind="mixed"):
    """random int8 index with mixed filters (pass-all, single bit, two bits + reverse, any-groups, pass-none)"""
    import torch
    rng = np.random.default_rng(seed)
    emb = torch.from_numpy(rng.integers(lo, hi + 1, (n, d), dtype=np.int8))
    Q = torch.from_numpy(rng.integers(lo, hi + 1, (B, m, d), dtype=np.int8))
    mask = torch.from_numpy(rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32).view(np.int32))
    ts = torch.from_numpy(rng.integers(0, 1000, n).astype(np.uint32).view(np.int32)) if with_ts else None
    scale = torch.from_numpy(rng.uniform(0.5, 2.0, n).astype(np.float32)) if scaled else None
    q_scale = torch.from_numpy(rng.uniform(0.5, 2.0, B).astype(np.float32))
    f = S.make_filters(B)
    for b in range(B):
        kind = b % 6 if filt_kind == "mixed" else filt_kind
        if kind == 1:
            f["all_bits"][b] = 1 << rng.integers(0, 32)
        elif kind == 2:
            f["all_bits"][b] = (1 << rng.integers(0, 16)) | (1 << rng.integers(16, 32))
            f["none_bits"][b] = 1 << rng.integers(0, 32)
        elif kind == 3:
            f["any_bits"][b][0] = 0x0000F00F; f["any_bits"][b][1] = 1 << rng.integers(0, 32); f["n_any"][b] = 2
        elif kind == 4:
            f["all_bits"][b] = 0xFFFFFFFF
        elif kind == 5:
            f["all_bits"][b] = sum(1 << int(x) for x in rng.choice(32, 7, replace=False))   # ~0.8 % pass
        if with_ts and b % 2 == 1:
            f["ts_min"][b] = 200; f["ts_max"][b] = 800
    return dict(dtype=S.I8, d=d, m=m, k=10, emb=emb, scale=scale, mask=mask, ts=ts, Q=Q, q_scale=q_scale, filters=f)
