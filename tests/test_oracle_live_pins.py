"""Pins of the live-update reference model (oracle.LiveIndex; LiNR Sec. 4 "Model Live Update") against things other
than itself: a sequence worked by hand, an independently kept dictionary of documents, and invariants."""
import json
import os
import numpy as np
import pytest

import synth_inputs as S

HERE = os.path.dirname(os.path.abspath(__file__))


def filt(all_bits=0, none_bits=0):
    f = S.make_filters(1)
    f["all_bits"] = all_bits
    f["none_bits"] = none_bits
    return f


def test_hand_sequence(oracle_mod):
    g = json.load(open(os.path.join(HERE, "golden", "live_update_example.json")))
    li = oracle_mod.LiveIndex(oracle_mod.F32, g["d"], g["capacity"])
    li.load(np.array(g["load"]["emb"], np.float32), np.array(g["load"]["mask"], np.uint32))
    q = np.array([g["query"]], np.float32)
    for st in g["steps"]:
        if st["op"] == "upsert":
            li.upsert(st["slots"], np.array(st["emb"], np.float32), np.array(st["mask"], np.uint32))
        elif st["op"] == "delete":
            li.delete(st["slots"])
        assert li.mark == st["mark"]
        for e in st["expect"]:
            ids, sc, _, cnt = li.search(q, filt(e["all_bits"]), g["k"])
            c = int(cnt[0])
            assert c == len(e["ids"]), (st, e)
            assert ids[0, :c].tolist() == e["ids"], (st, e)
            assert sc[0, :c].tolist() == e["scores"], (st, e)
            assert np.all(ids[0, c:] == oracle_mod.NO_ID)


@pytest.mark.parametrize("dtype_name", ["f32", "i8"])
def test_random_operations_against_a_dictionary_of_documents(oracle_mod, dtype_name):
    """The same stream of operations is applied to a plain dict {slot: document}; after every few operations the
    model's answer must equal the exhaustive search over the dict's documents sorted by slot."""
    rng = np.random.default_rng(5)
    d, cap, n0, k, B = 16, 300, 120, 12, 3
    dtype = oracle_mod.F32 if dtype_name == "f32" else oracle_mod.I8

    def rows(n):
        if dtype == oracle_mod.F32:
            return rng.standard_normal((n, d)).astype(np.float32), None
        return rng.integers(-127, 128, (n, d), dtype=np.int8), rng.uniform(0.001, 0.02, n).astype(np.float32)

    emb, sc = rows(n0)
    mask = rng.integers(0, 16, n0, dtype=np.uint32)
    ts = rng.integers(0, 1000, n0, dtype=np.uint32)
    li = oracle_mod.LiveIndex(dtype, d, cap, has_ts=True, has_scale=sc is not None)
    li.load(emb, mask, ts=ts, scale=sc)
    docs = {i: (emb[i], mask[i], ts[i], None if sc is None else sc[i]) for i in range(n0)}
    Q, qs = rows(B)
    f = S.make_filters(B)
    f["all_bits"] = [1, 0, 2]
    f["ts_min"] = [0, 100, 0]
    for step in range(60):
        if rng.random() < 0.6:
            u = int(rng.integers(1, 6))
            slots = rng.choice(cap, u, replace=False)
            e, s = rows(u)
            m = rng.integers(0, 16, u, dtype=np.uint32)
            t = rng.integers(0, 1000, u, dtype=np.uint32)
            li.upsert(slots, e, m, ts=t, scale=s)
            for j, sl in enumerate(slots.tolist()):
                docs[sl] = (e[j], m[j], t[j], None if s is None else s[j])
        else:
            live = sorted(docs)
            if live:
                victims = rng.choice(live, min(len(live), int(rng.integers(1, 8))), replace=False)
                li.delete(victims)
                for v in victims.tolist():
                    del docs[v]
        if step % 5 == 4:
            assert li.mark >= (max(docs) + 1 if docs else 0)
            order = sorted(docs)
            de = np.stack([docs[s][0] for s in order]); dm = np.array([docs[s][1] for s in order], np.uint32)
            dt = np.array([docs[s][2] for s in order], np.uint32)
            ds = None if sc is None else np.array([docs[s][3] for s in order], np.float32)
            ids, scr, raw, cnt = oracle_mod.search(dtype, de, dm, Q, f, k, row_scale=ds, ts=dt,
                                                   q_scale=None if qs is None else np.ones(B, np.float32))
            gi, gs, gr, gc = li.search(Q, f, k, q_scale=None if qs is None else np.ones(B, np.float32))
            assert np.array_equal(gc, cnt)
            for b in range(B):
                c = int(cnt[b])
                assert gi[b, :c].tolist() == [order[j] for j in ids[b, :c]]
                assert gs[b, :c].tobytes() == scr[b, :c].tobytes()


def test_invariants(oracle_mod):
    rng = np.random.default_rng(9)
    d, cap, n0, k = 8, 64, 40, 10
    emb = rng.standard_normal((n0, d)).astype(np.float32)
    mask = rng.integers(0, 8, n0, dtype=np.uint32)
    Q = rng.standard_normal((2, d)).astype(np.float32)
    f = S.make_filters(2)
    li = oracle_mod.LiveIndex(oracle_mod.F32, d, cap)
    li.load(emb, mask)
    base = li.search(Q, f, k)
    # an untouched model answers like the exhaustive search over the loaded arrays
    ref = oracle_mod.search(oracle_mod.F32, emb, mask, Q, f, k)
    assert all(np.array_equal(a, b) for a, b in zip(base, ref))
    # upserting a slot's own content changes nothing; delete followed by the same upsert restores the answer
    li.upsert([3, 7], emb[[3, 7]], mask[[3, 7]])
    assert all(np.array_equal(a, b) for a, b in zip(li.search(Q, f, k), base))
    top = int(base[0][0, 0])
    li.delete([top])
    after = li.search(Q, f, k)
    assert top not in after[0][0].tolist() and after[0][0, 0] == base[0][0, 1]
    li.upsert([top], emb[[top]], mask[[top]])
    assert all(np.array_equal(a, b) for a, b in zip(li.search(Q, f, k), base))
    # a deleted id never comes back, whatever k
    li.delete([1, 2, 3])
    ids, _, _, cnt = li.search(Q, f, cap)
    assert int(cnt[0]) == n0 - 3 and not {1, 2, 3} & set(ids[0, :int(cnt[0])].tolist())
    # skipped slots below a raised mark hold nothing
    li.upsert([60], emb[[0]], mask[[0]])
    assert li.mark == 61
    ids, _, _, cnt = li.search(Q, f, cap)
    got = set(ids[0, :int(cnt[0])].tolist())
    assert got == (set(range(n0)) - {1, 2, 3}) | {60}
    # deleting everything leaves nothing; deleting an empty slot below the mark is a no-op, above it an error
    li.delete(sorted(got))
    li.delete([50])
    assert int(li.search(Q, f, k)[3].max()) == 0
    with pytest.raises(IndexError):
        li.delete([61])
    with pytest.raises(IndexError):
        li.upsert([cap], emb[[0]], mask[[0]])
    # the order of operations on different slots does not matter
    a = oracle_mod.LiveIndex(oracle_mod.F32, d, cap); a.load(emb, mask)
    b = oracle_mod.LiveIndex(oracle_mod.F32, d, cap); b.load(emb, mask)
    a.delete([5]); a.upsert([45], emb[[9]], mask[[9]]); a.upsert([6], emb[[10]], mask[[10]])
    b.upsert([6], emb[[10]], mask[[10]]); b.upsert([45], emb[[9]], mask[[9]]); b.delete([5])
    assert all(np.array_equal(x, y) for x, y in zip(a.search(Q, f, k), b.search(Q, f, k)))


def test_codes_index(oracle_mod):
    """the same model over 1-bit codes: answers equal the exhaustive bit-matching search over the live codes"""
    rng = np.random.default_rng(3)
    n0, cap, T = 50, 80, 9
    codes = S.random_codes(n0, 64, 1)
    mask = rng.integers(0, 4, n0, dtype=np.uint32)
    li = oracle_mod.LiveIndex(None, 64, cap, code_words=1)
    li.load(codes, mask)
    q = S.random_codes(2, 64, 2)
    f = S.make_filters(2)
    new = S.random_codes(3, 64, 3)
    li.upsert([70, 2, 55], new, np.array([1, 1, 1], np.uint32))
    li.delete([0, 10])
    keep = [i for i in range(n0) if i not in (0, 10, 2)]
    slots = sorted(keep + [70, 2, 55])
    allc = {**{i: (codes[i], mask[i]) for i in keep}, 70: (new[0], 1), 2: (new[1], 1), 55: (new[2], 1)}
    dc = np.stack([allc[s][0] for s in slots]); dm = np.array([allc[s][1] for s in slots], np.uint32)
    ids, mt, cnt = oracle_mod.bits_search(dc, 64, dm, q, f, T)
    gi, gm, gc = li.bits_search(64, q, f, T)
    assert np.array_equal(gc, cnt) and np.array_equal(gm, mt)
    assert gi.tolist() == [[slots[j] for j in row] for row in ids.tolist()]
