"""Reference model of an index under live updates (LiNR Sec. 4, "Model Live Update": Upsert and Delete on
pre-allocated columns with a high-water mark) -- plain numpy, TEST INFRASTRUCTURE only.

The state is the definition itself: a table of `capacity` slots, a flag per slot saying whether it currently
holds an item, and the high-water mark (one past the highest slot ever written).  A search sees exactly the
slots that hold an item: they are gathered in ascending slot order into dense arrays, handed to the exhaustive
oracle (linr_oracle.search / bits_search), and the dense positions are mapped back to slot numbers.  Gathering
in ascending order keeps the tie rule (equal score: lower id first) in terms of slot numbers.

Readings (the paper names the two calls and the techniques, not their semantics):
  * an item is addressed by its slot number, which is also the id a search returns; the mapping from document
    keys to slots belongs to the ingestor;
  * upsert(slot) writes every column of the slot and makes it visible, whether the slot was empty, deleted or
    live; the mark rises to slot + 1 if needed; slots skipped below the new mark stay empty;
  * delete(slot) hides the slot; deleting an empty slot below the mark is a no-op, at or above the mark an error;
  * on an updatable index bit 31 of an item's attribute mask is not an attribute: it is stored as 0.
"""
from __future__ import annotations

import numpy as np

from . import linr_oracle as O

MASK_BITS = np.uint32(0x7FFFFFFF)


class LiveIndex:
    def __init__(self, dtype, d, capacity, has_ts=False, has_scale=False, code_words=0):
        """dtype: O.F32 / O.BF16 / O.I8, or None with code_words > 0 for an index of 1-bit codes."""
        self.dtype, self.d, self.capacity = dtype, d, capacity
        if dtype is None:
            self.emb = np.zeros((capacity, code_words), np.uint64)
        else:
            self.emb = np.zeros((capacity, d), {O.F32: np.float32, O.BF16: np.uint16, O.I8: np.int8}[dtype])
        self.mask = np.zeros(capacity, np.uint32)
        self.ts = np.zeros(capacity, np.uint32) if has_ts else None
        self.scale = np.zeros(capacity, np.float32) if has_scale else None
        self.live = np.zeros(capacity, bool)
        self.mark = 0

    def load(self, emb, mask, ts=None, scale=None):
        n = emb.shape[0]
        assert n <= self.capacity
        self.live[:] = False
        self.emb[:n] = emb
        self.mask[:n] = np.asarray(mask, np.uint32) & MASK_BITS
        if self.ts is not None:
            self.ts[:n] = ts
        if self.scale is not None:
            self.scale[:n] = scale
        self.live[:n] = True
        self.mark = n

    def upsert(self, slots, emb, mask, ts=None, scale=None):
        slots = np.asarray(slots, np.int64)
        assert len(set(slots.tolist())) == len(slots), "slots of one call must be distinct"
        for j, s in enumerate(slots.tolist()):
            if not 0 <= s < self.capacity:
                raise IndexError("slot beyond the capacity")
            self.emb[s] = emb[j]
            self.mask[s] = np.uint32(mask[j]) & MASK_BITS
            if self.ts is not None:
                self.ts[s] = ts[j]
            if self.scale is not None:
                self.scale[s] = scale[j]
            self.live[s] = True
            self.mark = max(self.mark, s + 1)

    def delete(self, slots):
        for s in np.asarray(slots, np.int64).tolist():
            if not 0 <= s < self.mark:
                raise IndexError("slot at or above the high-water mark")
            self.live[s] = False

    def _dense(self):
        sl = np.flatnonzero(self.live[:self.mark])
        return sl, self.emb[sl], self.mask[sl], None if self.ts is None else self.ts[sl], \
            None if self.scale is None else self.scale[sl]

    @staticmethod
    def _back(ids, counts, sl):
        out = np.full(ids.shape, O.NO_ID, np.uint32)
        for b in range(ids.shape[0]):
            c = int(counts[b])
            out[b, :c] = sl[ids[b, :c].astype(np.int64)]
        return out

    def search(self, Q, filters, k, q_scale=None, nthreads=1):
        """(ids [B,k] as slot numbers, scores, raw, counts) over the items currently held."""
        sl, emb, mask, ts, scale = self._dense()
        B = Q.shape[0]
        if len(sl) == 0:
            return (np.full((B, k), O.NO_ID, np.uint32), np.full((B, k), -np.inf, np.float32),
                    np.full((B, k), np.iinfo(np.int32).min, np.int32), np.zeros(B, np.uint32))
        ids, sc, raw, cnt = O.search(self.dtype, emb, mask, Q, filters, k, row_scale=scale, ts=ts, q_scale=q_scale,
                                     nthreads=nthreads)
        return self._back(ids, cnt, sl), sc, raw, cnt

    def bits_search(self, k_bits, qbits, filters, T):
        sl, codes, mask, ts, _ = self._dense()
        B = qbits.shape[0]
        if len(sl) == 0:
            return (np.full((B, T), O.NO_ID, np.uint32), np.full((B, T), np.iinfo(np.int32).min, np.int32),
                    np.zeros(B, np.uint32))
        ids, mt, cnt = O.bits_search(codes, k_bits, mask, qbits, filters, T, ts=ts)
        return self._back(ids, cnt, sl), mt, cnt
