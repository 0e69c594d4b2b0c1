"""GPU parity of the search with attribute matching over clause lists (LiNR Sec. 3.1.1; 64-bit attributes as in the
benchmark of Sec. 5.3) against oracle.clause_search, through the C ABI.  int8 results are bit-exact; fp32 / bf16 cases
use integer-valued embeddings, so their scores are exact too and are compared bit by bit."""
import json
import os
import time

import numpy as np
import pytest

import synth_inputs as S

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


def say(msg):
    print(f"[{time.strftime('%H:%M:%S')}] {msg}", flush=True)


def dev(a):
    import torch
    if a is None:
        return None
    view = {np.dtype(np.uint16): np.int16, np.dtype(np.uint32): np.int32, np.dtype(np.uint64): np.int64}.get(a.dtype)
    return torch.from_numpy(a.view(view) if view else a).cuda()


def rows(rng, kind, n, d):
    if kind == "f32":
        return rng.integers(-4, 5, (n, d)).astype(np.float32), None
    if kind == "bf16":
        return (rng.integers(-4, 5, (n, d)).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16), None
    return rng.integers(-127, 128, (n, d), dtype=np.int8), rng.uniform(0.001, 0.02, n).astype(np.float32)


DT = {"f32": S.F32, "bf16": S.BF16, "i8": S.I8}


def run_case(oracle_mod, kind, d, n, B, k, values, counts, qv, qc, reverse, label, m=1):
    import torch
    import paper_2407_13218_amd as L
    rng = np.random.default_rng(n + B)
    emb, sc = rows(rng, kind, n, d)
    Q, _ = rows(rng, kind, B * m, d)
    Q = Q.reshape(B, m, d)
    qs = np.ones(B, np.float32) if kind == "i8" else None
    ix = L.Index(n, d, DT[kind], 0)
    ix.load(emb, np.zeros(n, np.uint32), row_scale=sc)
    ix.load_clauses(values, counts, reverse)
    want = oracle_mod.clause_search(DT[kind], emb, values, counts, Q, qv, qc, reverse, k, row_scale=sc, q_scale=qs, nthreads=4)
    for prefilter in (False, True):                            # both strategies (Sec. 3.1.1 masking, Sec. 3.1.2 pre-filtering)
        ids, scr, raw, cnt = ix.search_clauses(dev(Q), dev(qv), dev(qc), k, q_scale=dev(qs), prefilter=prefilter)
        torch.cuda.synchronize()
        got = (ids.cpu().numpy().view(np.uint32), scr.cpu().numpy(), raw.cpu().numpy(), cnt.cpu().numpy().view(np.uint32))
        lab = f"{label} ({'pre-filtering' if prefilter else 'masking'})"
        assert np.array_equal(got[3], want[3]), f"{lab}: counts {got[3][:8]} vs {want[3][:8]}"
        bad = np.nonzero((got[0] != want[0]).any(axis=1))[0]
        assert bad.size == 0, f"{lab}: ids differ for queries {bad[:6]}: gpu {got[0][bad[0]][:8]} oracle {want[0][bad[0]][:8]}"
        assert got[1].tobytes() == want[1].tobytes(), f"{lab}: score bits differ"
        if kind == "i8":
            assert np.array_equal(got[2], want[2]), f"{lab}: raw scores differ"
    ix.close()
    return want


def test_hand_example_on_the_gpu(oracle_mod):
    import torch
    import paper_2407_13218_amd as L
    from test_oracle_clauses_pins import pack
    g = json.load(open(os.path.join(HERE, "golden", "clause_lists_example.json")))
    v, c = pack(g["item_lists"], 2)
    qv, qc = pack([g["query_lists"]], 2)
    emb = np.zeros((5, 4), np.float32); emb[:, :2] = np.array(g["emb"], np.float32)
    Q = np.zeros((1, 1, 4), np.float32); Q[0, 0, :2] = g["query"]
    ix = L.Index(5, 4, S.F32, 0)
    ix.load(emb, np.zeros(5, np.uint32))
    ix.load_clauses(v, c, g["reverse"])
    for k, key in ((1, "top1"), (3, "top3")):
        ids, sc, _, cnt = ix.search_clauses(dev(Q), dev(qv), dev(qc), k)
        torch.cuda.synchronize()
        assert ids.cpu().numpy().view(np.uint32)[0].tolist() == g[key]["ids"] and sc.cpu().numpy()[0].tolist() == g[key]["scores"]
    ids, sc, _, cnt = ix.search_clauses(dev(Q), dev(qv), dev(qc), 5)
    assert int(cnt.cpu()[0]) == g["top5_count"]
    none = np.zeros((1, 2), np.uint8)
    ids, sc, _, _ = ix.search_clauses(dev(Q), dev(qv), dev(none), 1)
    assert ids.cpu().numpy().view(np.uint32)[0].tolist() == g["no_clauses_top1"]["ids"]
    ix.close()


@pytest.mark.parametrize("kind,d,n,B,k,C,max_len,qlen,reverse", [
    ("i8", 64, 20_000, 7, 50, 2, 1, 1, 0b10),         # the benchmark's shape: one attribute per clause, second clause reverse
    ("i8", 64, 33_333, 40, 100, 3, 3, 4, 0b101),      # lists of 0..3 attributes, two groups of queries
    ("f32", 32, 5_001, 70, 20, 5, 2, 2, 0b01010),     # three groups
    ("bf16", 128, 9_000, 1, 300, 1, 4, 6, 0),         # one clause, long lists
    ("i8", 64, 2_000, 33, 64, 8, 1, 2, 0xFF),         # eight reverse clauses
    ("bf16", 64, 12_345, 16, 2000, 2, 2, 3, 0),       # k above the number of feasible items for most queries
    ("i8", 64, 150_000, 3, 6000, 1, 1, 3, 0),         # k above 2048
])
def test_random_clause_lists(oracle_mod, kind, d, n, B, k, C, max_len, qlen, reverse):
    domain = 6
    values, counts = S.random_clause_lists(n, C, max_len, domain, seed=n)
    qv, qc = S.random_clause_lists(B, C, qlen, domain, seed=n + 1)
    want = run_case(oracle_mod, kind, d, n, B, k, values, counts, qv, qc, reverse, f"{kind} n={n} B={B} C={C}")
    say(f"{kind} n={n} B={B} C={C}: feasible counts {want[3].min()}..{want[3].max()} (k = {k})")


@pytest.mark.parametrize("low_pass", [False, True])
def test_job_search_shape(oracle_mod, low_pass):
    """the benchmark's clauses (geo match, company reverse match, optionally title match) at 300 000 items, top-2000"""
    n, B = 300_000, 16
    w = S.job_clauses(n=n, B=B, low_pass=low_pass)
    values = w["values"].numpy().view(np.uint64); counts = w["counts"].numpy()
    qv = w["q_values"].numpy().view(np.uint64); qc = w["q_counts"].numpy()
    want = run_case(oracle_mod, "bf16", 128, n, B, 2000, values, counts, qv, qc, w["reverse"], f"job clauses low_pass={low_pass}")
    say(f"job clauses low_pass={low_pass}: feasible per query {want[3].tolist()}")


def test_prefilter_with_many_feasible_items(oracle_mod):
    """queries without constraints: every item is feasible, the keys overflow the flat arrays into the segments"""
    values, counts = S.random_clause_lists(50_000, 1, 1, 5, seed=2)
    qv = np.zeros((3, 2), np.uint64); qc = np.zeros((3, 1), np.uint8)
    qv[1, 0] = values[0, 0]; qc[1, 0] = 1                         # one query keeps a constraint
    run_case(oracle_mod, "i8", 64, 50_000, 3, 10, values, counts, qv, qc, 0, "everything feasible")


def test_prefilter_with_a_million_feasible_items_and_overflow():
    """four million feasible items for one query: the two phases (a sample, then the rest against the bound the sample
    gave) keep the candidate arrays small and both strategies agree; with a deliberately small workspace plan the sample
    itself does not fit and the count says so (0xFFFFFFFF) while the other query is still answered"""
    import torch
    import paper_2407_13218_amd as L
    n = 4_000_000
    rng = np.random.default_rng(0)
    emb = rng.integers(-127, 128, (n, 64), dtype=np.int8)
    values = np.full((n, 1), 7, np.uint64); values[::1000, 0] = 9
    counts = np.ones((n, 1), np.uint8)
    ix = L.Index(n, 64, S.I8, 0)
    ix.load(emb, np.zeros(n, np.uint32))
    ix.load_clauses(values, counts, 0)
    qv = np.array([[7], [9]], np.uint64); qc = np.ones((2, 1), np.uint8)
    Q = dev(emb[:2].reshape(2, 1, 64))
    ids2, _, raw2, cnt2 = ix.search_clauses(Q, dev(qv), dev(qc), 5)
    ids, sc, raw, cnt = ix.search_clauses(Q, dev(qv), dev(qc), 5, prefilter=True)
    torch.cuda.synchronize()
    assert np.array_equal(cnt.cpu().numpy(), cnt2.cpu().numpy()) and np.array_equal(ids.cpu().numpy(), ids2.cpu().numpy())
    assert np.array_equal(raw.cpu().numpy(), raw2.cpu().numpy())
    L.set_tuning(blocks_per_cu=1)                             # 1024 slots x 192 keys + 4096: less than the 250 000 sampled keys (n / 16)
    try:
        ids, sc, raw, cnt = ix.search_clauses(Q, dev(qv), dev(qc), 5, prefilter=True)
        torch.cuda.synchronize()
    finally:
        L.set_tuning()
    cnt = cnt.cpu().numpy().view(np.uint32)
    assert cnt[0] == 0xFFFFFFFF and cnt[1] == 5
    assert np.array_equal(ids.cpu().numpy()[1], ids2.cpu().numpy()[1]) and np.array_equal(raw.cpu().numpy()[1], raw2.cpu().numpy()[1])
    ix.close()


def test_multi_embedding_queries(oracle_mod):
    values, counts = S.random_clause_lists(8_000, 2, 2, 5, seed=5)
    qv, qc = S.random_clause_lists(9, 2, 2, 5, seed=6)
    run_case(oracle_mod, "bf16", 64, 8_000, 9, 40, values, counts, qv, qc, 0b10, "m = 4", m=4)


def test_with_live_updates(oracle_mod):
    """deleted slots are infeasible for a clause search; upserted items get their lists through linr_index_upsert_clauses
    (without it they list nothing); both strategies against the oracle over the live items"""
    import torch
    import paper_2407_13218_amd as L
    rng = np.random.default_rng(2)
    n, cap, d, B, k = 6_000, 7_000, 64, 5, 80
    emb, sc = rows(rng, "i8", cap, d)
    Q, _ = rows(rng, "i8", B, d)
    Q = Q.reshape(B, 1, d); qs = np.ones(B, np.float32)
    values, counts = S.random_clause_lists(cap, 2, 2, 4, seed=9)
    qv, qc = S.random_clause_lists(B, 2, 2, 4, seed=10)
    qc[0] = 0                                                    # query 0 constrains nothing
    ix = L.Index(cap, d, S.I8, 0)
    ix.load(emb[:n], np.zeros(n, np.uint32), row_scale=sc[:n])
    ix.load_clauses(values[:n], counts[:n], 0b10)
    ix.enable_updates()
    live = np.zeros(cap, bool); live[:n] = True
    have_lists = live.copy()

    def check(label):
        keep = np.flatnonzero(live)
        cts = np.where(have_lists[keep, None], counts[keep], 0).astype(np.uint8)
        want = oracle_mod.clause_search(S.I8, emb[keep], values[keep], cts, Q, qv, qc, 0b10, k, row_scale=sc[keep], q_scale=qs)
        wid = np.where(want[0] == oracle_mod.NO_ID, oracle_mod.NO_ID, keep[np.minimum(want[0], len(keep) - 1)].astype(np.uint32))
        for prefilter in (False, True):
            ids, scr, raw, cnt = ix.search_clauses(dev(Q), dev(qv), dev(qc), k, q_scale=dev(qs), prefilter=prefilter)
            torch.cuda.synchronize()
            assert np.array_equal(cnt.cpu().numpy().view(np.uint32), want[3]), label
            assert np.array_equal(ids.cpu().numpy().view(np.uint32), wid), label
            assert scr.cpu().numpy().tobytes() == want[1].tobytes(), label

    gone = rng.choice(n, 2500, replace=False).astype(np.uint32)
    ix.delete(gone); live[gone] = False
    check("after deletes")
    fresh = np.arange(n, n + 400, dtype=np.uint32)
    ix.upsert(fresh, emb[fresh], np.zeros(400, np.uint32), row_scale=sc[fresh]); live[fresh] = True
    check("upserted items without lists")                        # they list nothing: only unconstrained / reverse clauses pass
    ix.upsert_clauses(fresh[:300], values[fresh[:300]], counts[fresh[:300]]); have_lists[fresh[:300]] = True
    check("lists for 300 of them (host source)")
    ix.upsert_clauses(fresh[300:], dev(values[fresh[300:]]), dev(counts[fresh[300:]])); have_lists[fresh[300:]] = True
    check("lists for the rest (device source)")
    reuse = gone[:100]                                           # deleted slots come back with new rows and lists
    ix.upsert_clauses(reuse, values[fresh[:100]], counts[fresh[:100]])
    values[reuse] = values[fresh[:100]]; counts[reuse] = counts[fresh[:100]]
    ix.upsert(reuse, emb[reuse], np.zeros(100, np.uint32), row_scale=sc[reuse]); live[reuse] = True
    check("reused slots")
    ix.close()


def test_clause_argument_errors():
    import paper_2407_13218_amd as L
    rng = np.random.default_rng(1)
    emb, sc = rows(rng, "i8", 100, 64)
    ix = L.Index(100, 64, S.I8, 0)
    ix.load(emb, np.zeros(100, np.uint32), row_scale=sc)
    Q = dev(emb[:2].reshape(2, 1, 64))
    qv = dev(np.zeros((2, 2), np.uint64)); qc = dev(np.zeros((2, 2), np.uint8))
    with pytest.raises(L.LinrError) as e:
        ix.search_clauses(Q, qv, qc, 5)                                   # no clause columns
    assert e.value.code == -10
    v = np.zeros((99, 2), np.uint64); c = np.zeros((99, 2), np.uint8)
    with pytest.raises(L.LinrError) as e:
        ix.load_clauses(v, c)                                             # not one row per item
    assert e.value.code == -5
    with pytest.raises(L.LinrError) as e:
        ix.load_clauses(np.zeros((100, 9), np.uint64), np.zeros((100, 9), np.uint8))   # more clauses than supported
    assert e.value.code == -2
    with pytest.raises(L.LinrError) as e:
        ix.load_clauses(np.zeros((100, 2), np.uint64), np.zeros((100, 2), np.uint8), reverse=0b100)   # reverse bit of no clause
    assert e.value.code == -2
    ix.close()
