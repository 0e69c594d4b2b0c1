"""The allocation-free entry point (linr_search_filtered_noalloc: callers that cannot allocate) against
linr_search_filtered, through the C ABI: two calls in a row on one GPU, the second with a smaller input, every output
bit for bit; a search that does not fit the fixed scratch array is refused before anything is written."""
import numpy as np
import pytest

import synth_inputs as S
from gpu_util import rand_int8_workload, to_cuda

pytestmark = pytest.mark.gpu


def _both(L, torch, w, k, poison):
    d = to_cuda(w)
    n, B = d["emb"].shape[0], d["Q"].shape[0]
    ix = L.Index(n, w["d"], w["dtype"], 0)
    ix.load(d["emb"], d["mask"], ts=d["ts"], row_scale=d["scale"])
    filt = torch.from_numpy(np.ascontiguousarray(w["filters"]).view(np.uint8).copy()).cuda()
    stream = torch.cuda.current_stream().cuda_stream
    need = ix.workspace_bytes(B, w["m"], k)
    assert need <= L.NOALLOC_SCRATCH_BYTES, need
    outs = []
    for which in ("workspace", "noalloc"):
        ids = torch.full((B, k), poison, dtype=torch.int32, device="cuda"); sc = torch.full((B, k), 7.0, dtype=torch.float32, device="cuda")
        raw = torch.full((B, k), poison, dtype=torch.int32, device="cuda"); cnt = torch.full((B,), poison, dtype=torch.int32, device="cuda")
        if which == "workspace":
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            L.search_filtered(ix.handle, d["Q"], d["q_scale"], B, w["m"], filt, k, ids, sc, raw, cnt, ws, need, stream, L.FILTERS_ON_DEVICE)
        else:
            L.search_filtered_noalloc(ix.handle, d["Q"], d["q_scale"], B, w["m"], filt, k, ids, sc, raw, cnt, stream, L.FILTERS_ON_DEVICE)
        torch.cuda.synchronize()
        outs.append((ids.cpu().numpy(), sc.cpu().numpy(), raw.cpu().numpy(), cnt.cpu().numpy()))
    ix.close()
    return outs


def test_noalloc_matches_workspace_entry_point_twice(oracle_mod):
    import torch
    import paper_2407_13218_amd as L
    # first call: 300 003 items, 3 queries (mixed filters, timestamps), k = 200; second, smaller: 40 001 items, 1 query, k = 50
    for seed, n, B, k in ((11, 300_003, 3, 200), (12, 40_001, 1, 50)):
        print(f"no-alloc entry point: n={n} B={B} k={k}", flush=True)
        w = rand_int8_workload(seed, n, 64, B, scaled=True, with_ts=True)
        a, b = _both(L, torch, w, k, poison=-123456)
        for x, y, name in zip(a, b, ("ids", "scores", "raw", "counts")):
            assert x.tobytes() == y.tobytes(), f"n={n}: {name} differ between the two entry points"
        # and both are the oracle's answer
        h = S.to_numpy(w)
        oi, os_, orw, oc = oracle_mod.search(S.I8, h["emb"], h["mask"], h["Q"], h["filters"], k, row_scale=h["scale"], ts=h["ts"],
                                             q_scale=h["q_scale"], nthreads=4)
        assert np.array_equal(b[0].view(np.uint32), oi) and b[1].tobytes() == os_.tobytes()
        assert np.array_equal(b[2], orw) and np.array_equal(b[3].view(np.uint32), oc)


def test_noalloc_refuses_what_does_not_fit():
    import torch
    import paper_2407_13218_amd as L
    w = rand_int8_workload(13, 2_000_000, 64, 64, scaled=True)
    d = to_cuda(w)
    ix = L.Index(2_000_000, 64, S.I8, 0)
    ix.load(d["emb"], d["mask"], row_scale=d["scale"])
    k = 1000
    assert ix.workspace_bytes(64, 1, k) > L.NOALLOC_SCRATCH_BYTES
    ids = torch.full((64, k), 5, dtype=torch.int32, device="cuda"); sc = torch.zeros((64, k), dtype=torch.float32, device="cuda")
    cnt = torch.full((64,), 5, dtype=torch.int32, device="cuda")
    filt = torch.from_numpy(np.ascontiguousarray(w["filters"]).view(np.uint8).copy()).cuda()
    with pytest.raises(L.LinrError) as err:
        L.search_filtered_noalloc(ix.handle, d["Q"], d["q_scale"], 64, 1, filt, k, ids, sc, None, cnt,
                                  torch.cuda.current_stream().cuda_stream, L.FILTERS_ON_DEVICE)
    assert err.value.code == -11 and "scratch" in str(err.value)
    torch.cuda.synchronize()
    assert int(ids.min()) == 5 and int(ids.max()) == 5 and int(cnt.min()) == 5        # nothing was touched
    ix.close()
