"""GPU parity of live updates (upsert / delete with a high-water mark, LiNR Sec. 4 "Model Live Update") against the
reference model oracle.LiveIndex, through the C ABI.  Embeddings are small integers, so that fp32 / bf16 scores are
exact whatever the summation order and every comparison is bit-exact (the float tolerance rule is covered by the
other parity tests; here the update machinery is under test)."""
import json
import os
import threading
import time

import numpy as np
import pytest

import synth_inputs as S

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


def say(msg):
    print(f"[{time.strftime('%H:%M:%S')}] {msg}", flush=True)


def bf16_bits(x):
    return (np.asarray(x, np.float32).view(np.uint32) >> 16).astype(np.uint16)


def gen_rows(rng, kind, n, d):
    """(rows in the index's element type, row scales or None); integer values: exact dot products"""
    if kind == "f32":
        return rng.integers(-4, 5, (n, d)).astype(np.float32), None
    if kind == "bf16":
        return bf16_bits(rng.integers(-4, 5, (n, d)).astype(np.float32)), None
    if kind == "i8":
        return rng.integers(-127, 128, (n, d), dtype=np.int8), rng.uniform(0.001, 0.02, n).astype(np.float32)
    return S.random_codes(n, d, int(rng.integers(0, 1 << 30))), None          # "bits": d = bits per code


def dev(a):
    import torch
    if a is None:
        return None
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).cuda()
    if a.dtype == np.uint64:
        return torch.from_numpy(a.view(np.int64)).cuda()
    return torch.from_numpy(a).cuda()


def gpu_search(ix, kind, Qd, filt, k, qs=None):
    import torch
    if kind == "bits":
        ids, mt, cnt = ix.search_bits(Qd, filt, k)
        torch.cuda.synchronize()
        return ids.cpu().numpy().view(np.uint32), mt.cpu().numpy(), cnt.cpu().numpy().view(np.uint32)
    ids, sc, raw, cnt = ix.search(Qd, filt, k, q_scale=qs, strategy="masking")
    torch.cuda.synchronize()
    return ids.cpu().numpy().view(np.uint32), sc.cpu().numpy(), raw.cpu().numpy() if raw is not None else None, \
        cnt.cpu().numpy().view(np.uint32)


def compare(kind, gpu, ora, label):
    if kind == "bits":
        gi, gm, gc = gpu
        oi, om, oc = ora
        assert np.array_equal(gc, oc), f"{label}: counts {gc} vs {oc}"
        assert np.array_equal(gi, oi), f"{label}: ids differ"
        assert np.array_equal(gm, om), f"{label}: match counts differ"
        return
    gi, gs, gr, gc = gpu
    oi, os_, orw, oc = ora
    assert np.array_equal(gc, oc), f"{label}: counts {gc} vs {oc}"
    bad = np.nonzero((gi != oi).any(axis=1))[0]
    assert bad.size == 0, f"{label}: ids differ for queries {bad[:6]}: gpu {gi[bad[0]][:8]} oracle {oi[bad[0]][:8]}"
    assert gs.tobytes() == os_.tobytes(), f"{label}: score bits differ"
    if kind == "i8":
        assert np.array_equal(gr, orw), f"{label}: raw scores differ"


def test_hand_sequence_on_the_gpu(oracle_mod):
    """the sequence worked by hand (tests/golden/live_update_example.json), d padded from 2 to 4 with zeros"""
    import paper_2407_13218_amd as L
    g = json.load(open(os.path.join(HERE, "golden", "live_update_example.json")))

    def pad(rows):
        a = np.zeros((len(rows), 4), np.float32)
        a[:, :2] = np.array(rows, np.float32)
        return a
    ix = L.Index(g["capacity"], 4, S.F32, 0)
    ix.load(pad(g["load"]["emb"]), np.array(g["load"]["mask"], np.uint32))
    ix.enable_updates()
    q = dev(pad([g["query"]]).reshape(1, 1, 4))
    for st in g["steps"]:
        if st["op"] == "upsert":
            ix.upsert(st["slots"], pad(st["emb"]), np.array(st["mask"], np.uint32))
        elif st["op"] == "delete":
            ix.delete(st["slots"])
        for e in st["expect"]:
            f = S.make_filters(1)
            f["all_bits"] = e["all_bits"]
            ids, sc, _, cnt = gpu_search(ix, "f32", q, f, g["k"])
            c = int(cnt[0])
            assert c == len(e["ids"]) and ids[0, :c].tolist() == e["ids"] and sc[0, :c].tolist() == e["scores"], (st, e, ids, sc)
        ix.sync_updates()
        assert ix.info()["n"] == st["mark"]
    ix.close()


@pytest.mark.parametrize("kind,d,n0,cap,B,k", [
    ("i8", 64, 5000, 9000, 20, 100),
    ("f32", 32, 3000, 4000, 7, 50),
    ("bf16", 128, 2500, 6000, 70, 64),
    ("bits", 64, 4000, 7000, 9, 200),
    ("bits", 192, 1500, 3000, 3, 40),
    ("i8", 64, 300, 100_000, 130, 300),       # mostly empty capacity, k close to the number of live items
    ("bf16x8", 64, 3000, 5000, 40, 80),       # eight embeddings per query: the large-batch bf16 kernel for that shape
])
def test_random_updates_match_the_model(oracle_mod, kind, d, n0, cap, B, k):
    """upserts (fresh slots, reused slots, in-place; host and device sources) and deletes on the search stream, a search
    after every step compared with the reference model"""
    import paper_2407_13218_amd as L
    rng = np.random.default_rng(n0 + d)
    m = 8 if kind == "bf16x8" else 1
    kind = "bf16" if kind == "bf16x8" else kind
    with_ts = kind in ("i8", "bits")
    dtype = {"f32": S.F32, "bf16": S.BF16, "i8": S.I8, "bits": S.BITS}[kind]
    emb, sc = gen_rows(rng, kind, n0, d)
    mask = rng.integers(0, 1 << 31, n0, dtype=np.uint32) & rng.integers(0, 1 << 31, n0, dtype=np.uint32)
    ts = rng.integers(0, 1000, n0, dtype=np.uint32) if with_ts else None
    if kind == "bits":
        li = oracle_mod.LiveIndex(None, d, cap, has_ts=with_ts, code_words=emb.shape[1])
    else:
        li = oracle_mod.LiveIndex(dtype, d, cap, has_ts=with_ts, has_scale=sc is not None)
    li.load(emb, mask, ts=ts, scale=sc)
    ix = L.Index(cap, d, dtype, 0)
    ix.load(emb, mask, ts=ts, row_scale=sc)                    # host arrays: library-owned columns of `cap` slots
    ix.enable_updates()
    Q, _ = gen_rows(rng, kind, B * m, d)
    Qd = dev(Q) if kind == "bits" else dev(Q.reshape(B, m, d))
    qs = np.ones(B, np.float32) if kind == "i8" else None
    qsd = dev(qs)
    filt = S.make_filters(B)
    for b in range(B):
        if b % 3 == 1:
            filt["all_bits"][b] = 1 << int(rng.integers(0, 31))
        if b % 3 == 2:
            filt["none_bits"][b] = 1 << int(rng.integers(0, 31))
            filt["any_bits"][b][0] = 0x00FF00FF; filt["n_any"][b] = 1
        if with_ts and b % 4 == 3:
            filt["ts_min"][b] = 100; filt["ts_max"][b] = 900

    def check(label):
        if kind == "bits":
            ora = li.bits_search(d, Q, filt, k)
        else:
            ora = li.search(Q.reshape(B, m, d), filt, k, q_scale=qs, nthreads=4)
        compare(kind, gpu_search(ix, kind, Qd, filt, k, qsd), ora, label)

    check("after load")
    for step in range(14):
        r = step % 7
        if r in (0, 1, 4):                                    # upsert: a mix of fresh, live and deleted slots
            u = int(rng.integers(1, 400))
            hi = min(cap, li.mark + (u if r != 4 else 3 * u))
            slots = rng.choice(hi, min(u, hi), replace=False).astype(np.uint32)
            e, s = gen_rows(rng, kind, len(slots), d)
            mk = rng.integers(0, 1 << 32, len(slots), dtype=np.uint32) & rng.integers(0, 1 << 32, len(slots), dtype=np.uint32)
            t = rng.integers(0, 1000, len(slots), dtype=np.uint32) if with_ts else None
            li.upsert(slots, e, mk, ts=t, scale=s)
            if step % 2 == 0:
                ix.upsert(slots, e, mk, ts=t, row_scale=s)
            else:
                ix.upsert(slots, dev(e), dev(mk), ts=dev(t), row_scale=dev(s))
            label = f"step {step}: upsert of {len(slots)} slots (mark {li.mark})"
        elif r in (2, 5):                                     # delete live and already empty slots
            cand = rng.choice(li.mark, min(li.mark, int(rng.integers(1, 600))), replace=False).astype(np.uint32)
            li.delete(cand)
            ix.delete(cand)
            label = f"step {step}: delete of {len(cand)} slots"
        elif r == 3:                                          # the current best answers of query 0 disappear
            first = li.bits_search(d, Q, filt, k)[0][0] if kind == "bits" else li.search(Q.reshape(B, m, d), filt, k, q_scale=qs)[0][0]
            victims = first[first != S.NO_ID][:10]
            if len(victims):
                li.delete(victims); ix.delete(victims)
            label = f"step {step}: delete of the top answers"
        else:                                                 # one slot far above the mark: the slots between stay empty
            slot = np.array([min(cap - 1, li.mark + 1000)], np.uint32)
            e, s = gen_rows(rng, kind, 1, d)
            mk = np.array([0], np.uint32); t = np.array([500], np.uint32) if with_ts else None
            li.upsert(slot, e, mk, ts=t, scale=s)
            ix.upsert(slot, e, mk, ts=t, row_scale=s)
            label = f"step {step}: upsert far above the mark (mark {li.mark})"
        check(label)
    ix.sync_updates()
    assert ix.info()["n"] == li.mark
    ix.close()


def test_codes_follow_the_rows(oracle_mod):
    """an fp32 index with Sign-OPORP codes: after upserts and deletes the quantised search equals the oracle's over the
    codes of the live rows"""
    import paper_2407_13218_amd as L
    rng = np.random.default_rng(12)
    d, kb, n0, cap, B, T = 64, 64, 3000, 5000, 6, 80
    emb = rng.standard_normal((n0, d)).astype(np.float32)
    mask = rng.integers(0, 16, n0, dtype=np.uint32)
    perm, signs = S.oporp_draw(d, 3)
    li = oracle_mod.LiveIndex(None, kb, cap, code_words=1)
    li.load(oracle_mod.sign_oporp(S.F32, emb, perm, signs, kb), mask)
    ix = L.Index(cap, d, S.F32, 0)
    ix.load(emb, mask)
    ix.build_bits(perm, signs, kb)
    ix.enable_updates()
    Q = rng.standard_normal((B, d)).astype(np.float32)
    qbits = ix.quantize(dev(Q))
    qb_h = qbits.cpu().numpy().view(np.uint64)
    assert np.array_equal(qb_h, oracle_mod.sign_oporp(S.F32, Q, perm, signs, kb))
    filt = S.make_filters(B)
    filt["all_bits"][1] = 1
    for step in range(4):
        slots = rng.choice(min(cap, li.mark + 300), 250, replace=False).astype(np.uint32)
        e = rng.standard_normal((250, d)).astype(np.float32)
        m = rng.integers(0, 16, 250, dtype=np.uint32)
        li.upsert(slots, oracle_mod.sign_oporp(S.F32, e, perm, signs, kb), m)
        if step % 2:
            ix.upsert(slots, dev(e), dev(m))
        else:
            ix.upsert(slots, e, m)
        dl = rng.choice(li.mark, 200, replace=False).astype(np.uint32)
        li.delete(dl); ix.delete(dl)
        compare("bits", gpu_search(ix, "bits", qbits, filt, T), li.bits_search(kb, qb_h, filt, T), f"step {step}")
    ix.close()


def test_updates_from_another_thread_and_stream(oracle_mod):
    """one thread upserts fresh slots and deletes old ones on its own stream while this thread searches; every answer in
    between is well-formed, and after linr_index_sync_updates the index equals the model"""
    import torch
    import paper_2407_13218_amd as L
    rng = np.random.default_rng(44)
    d, n0, cap, B, k = 64, 200_000, 260_000, 4, 100
    emb, sc = gen_rows(rng, "i8", n0, d)
    mask = rng.integers(0, 8, n0, dtype=np.uint32)
    li = oracle_mod.LiveIndex(S.I8, d, cap, has_scale=True)
    li.load(emb, mask, scale=sc)
    ix = L.Index(cap, d, S.I8, 0)
    ix.load(emb, mask, row_scale=sc)
    ix.enable_updates()
    Q, _ = gen_rows(rng, "i8", B, d)
    Qd = dev(Q.reshape(B, 1, d)); qs = np.ones(B, np.float32); qsd = dev(qs)
    filt = S.make_filters(B)
    batches = []
    mark = n0
    for i in range(120):
        u = 100
        slots = np.arange(mark, mark + u, dtype=np.uint32); mark += u
        e, s = gen_rows(rng, "i8", u, d)
        m = rng.integers(0, 8, u, dtype=np.uint32)
        dl = rng.choice(n0, 50, replace=False).astype(np.uint32)
        batches.append((slots, e, s, m, dl))
    side = torch.cuda.Stream()
    err = []

    def updater():
        try:
            for slots, e, s, m, dl in batches:
                ix.upsert(slots, e, m, row_scale=s, stream=side.cuda_stream)
                ix.delete(dl, stream=side.cuda_stream)
        except Exception as ex:                                   # noqa: BLE001
            err.append(ex)
    th = threading.Thread(target=updater)
    th.start()
    rounds = 0
    while th.is_alive() or rounds < 3:
        ids, scr, raw, cnt = gpu_search(ix, "i8", Qd, filt, k, qsd)
        assert np.all(cnt == k) and np.all(ids < cap)
        assert np.all(np.diff(scr.astype(np.float64), axis=1) <= 0)
        assert all(len(set(row.tolist())) == k for row in ids)
        rounds += 1
    th.join()
    assert not err, err
    ix.sync_updates()
    for slots, e, s, m, dl in batches:
        li.upsert(slots, e, m, scale=s)
        li.delete(dl)
    assert ix.info()["n"] == li.mark
    compare("i8", gpu_search(ix, "i8", Qd, filt, k, qsd), li.search(Q.reshape(B, 1, d), filt, k, q_scale=qs, nthreads=4),
            "after the concurrent updates")
    say(f"{rounds} searches ran next to {len(batches)} update batches")
    ix.close()


def test_update_argument_errors():
    import paper_2407_13218_amd as L
    rng = np.random.default_rng(1)
    emb = rng.integers(-5, 5, (100, 64), dtype=np.int8)
    sc = np.ones(100, np.float32)
    mask = np.zeros(100, np.uint32)
    ts = np.zeros(100, np.uint32)
    ix = L.Index(150, 64, S.I8, 0)
    ix.load(emb, mask, ts=ts, row_scale=sc)
    one = (emb[:1], mask[:1])
    with pytest.raises(L.LinrError) as e:
        ix.upsert([3], *one, ts=ts[:1], row_scale=sc[:1])       # updates not enabled yet
    assert e.value.code == -10
    ix.enable_updates()
    ix.enable_updates()                                          # idempotent
    with pytest.raises(L.LinrError) as e:
        ix.upsert([150], *one, ts=ts[:1], row_scale=sc[:1])      # beyond the capacity
    assert e.value.code == -5
    with pytest.raises(L.LinrError) as e:
        ix.upsert([7, 7], emb[:2], mask[:2], ts=ts[:2], row_scale=sc[:2])   # one slot twice
    assert e.value.code == -2
    with pytest.raises(L.LinrError) as e:
        ix.upsert([7], *one, row_scale=sc[:1])                   # the index has timestamps
    assert e.value.code == -1
    with pytest.raises(L.LinrError) as e:
        ix.delete([100])                                         # at the mark
    assert e.value.code == -5
    ix.upsert([120], *one, ts=ts[:1], row_scale=sc[:1])
    ix.delete([110])                                             # empty slot below the (pending) mark: no-op
    ix.sync_updates()
    assert ix.info()["n"] == 121
    ix.close()
    bad = L.Index(10, 64, S.I8, 0)
    m2 = np.zeros(10, np.uint32); m2[4] = 0x80000000
    bad.load(emb[:10], m2, row_scale=sc[:10])
    with pytest.raises(L.LinrError) as e:
        bad.enable_updates()                                     # a resident mask uses bit 31
    assert e.value.code == -9
    bad.close()
