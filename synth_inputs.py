"""Seeded synthetic inputs for the filtered exhaustive top-k path.

This module only *produces inputs* (embeddings, attribute columns, queries,
filters) and the byte layout of the filter record.  It contains none of the
retrieval arithmetic (no scoring, no predicate evaluation, no selection) and is
the one module that the CPU oracle's tests and the HIP library's tests, smoke and
bench all import.  The oracle and the library never import each other.

The paper's indexes (job search: ~15.5 M items, d = 128, two or three clauses, ~11 %
down to ~0.01 % of items feasible, top-2000; notifications: 1e9 members, d = 64;
Sec. 5.3 and the stretch test) are internal and unavailable, so every workload
here is a seeded stand-in with the same shapes and pass-rate regimes:

  cfg 1: N=1e5,  d=64  fp32, i.i.d. N(0,1) rows L2-normalised, B=16, 3 required bits (12.5 %), k=100
  cfg 2: N=1e7,  d=128 bf16, 1000 Gaussian clusters, B=256, 2 required bits at p in {.9,.5,.1}, k=1000
  cfg 3: N=5e7,  d=64  int8 per-row scale, clustered, B in {1,16,64,512}, 1 bit AND ts >= now-7d (7 %), k=1000
  cfg 4: N=2e7,  d=64  bf16, clustered, 128 queries x m=8 embeddings, ~5 %, k=500
  cfg 5: N=1e9,  d=64  int8 per-row scale, 10000 clusters, B in {1,32,256,1024}, 50 % / 5 % / 0.1 %, k=1000

Clustered rows: centre drawn uniformly on the unit sphere, item = centre + Gaussian
noise of total norm ~ sigma (per-coordinate sigma / sqrt(d)), then L2-normalised;
each item picks its centre i.i.d., so clusters are interleaved in memory.
"""
from __future__ import annotations

import math
import numpy as np
import torch

SEED0 = 20240713
NOW = 1_720_000_000
DAY = 86_400

F32, BF16, I8, BITS = 0, 1, 2, 3
NO_ID = 0xFFFFFFFF
MAX_ANY = 4

#: byte layout of one query's filter record (40 bytes, little endian)
FILTER_DTYPE = np.dtype([
    ("all_bits", "<u4"), ("none_bits", "<u4"), ("any_bits", "<u4", (MAX_ANY,)),
    ("n_any", "<u4"), ("ts_min", "<u4"), ("ts_max", "<u4"), ("_pad", "<u4"),
])
assert FILTER_DTYPE.itemsize == 40


def make_filters(B: int) -> np.ndarray:
    """B filter records that pass every item."""
    f = np.zeros(B, dtype=FILTER_DTYPE)
    f["ts_max"] = 0xFFFFFFFF
    return f


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def l2_normalise(x: torch.Tensor) -> torch.Tensor:
    return x / x.norm(dim=-1, keepdim=True).clamp_min(1e-30)


def quantize_rows(x: torch.Tensor):
    """Symmetric int8 codes with one fp32 scale per row: scale = max|x| / 127,
    code = clamp(round_half_even(x / scale), -127, 127); an all-zero row gets
    scale 1 and zero codes."""
    x = x.to(torch.float32)
    amax = x.abs().amax(dim=-1)
    scale = torch.where(amax > 0, amax / 127.0, torch.ones_like(amax)).to(torch.float32)
    codes = torch.round(x / scale.unsqueeze(-1)).clamp_(-127, 127).to(torch.int8)
    return codes, scale


def quantize_queries(q: torch.Tensor):
    """q is [B, m, d]; one scale per query over all m*d values."""
    B = q.shape[0]
    codes, scale = quantize_rows(q.reshape(B, -1))
    return codes.reshape(q.shape), scale


def to_bf16_bits(x: torch.Tensor) -> torch.Tensor:
    """fp32 -> bf16 (round to nearest even) returned as int16 bit patterns."""
    return x.to(torch.bfloat16).view(torch.int16)


def unit_centres(C: int, d: int, device, seed: int) -> torch.Tensor:
    return l2_normalise(torch.randn(C, d, generator=_gen(device, seed), device=device, dtype=torch.float32))


def clustered_rows(n: int, centres: torch.Tensor, sigma: float, device, seed: int,
                   sort_by_cluster: bool = False) -> torch.Tensor:
    g = _gen(device, seed)
    C, d = centres.shape
    which = torch.randint(0, C, (n,), generator=g, device=device)
    if sort_by_cluster:
        which, _ = torch.sort(which)
    noise = torch.randn(n, d, generator=g, device=device, dtype=torch.float32) * (sigma / math.sqrt(d))
    return l2_normalise(centres[which] + noise)


def bernoulli_masks(n: int, p_bits, device, seed: int) -> torch.Tensor:
    """uint32 attribute masks (held as int32 bit patterns); bit j set with probability p_bits[j]."""
    g = _gen(device, seed)
    out = torch.zeros(n, dtype=torch.int64, device=device)
    for j, p in enumerate(p_bits):
        bit = (torch.rand(n, generator=g, device=device) < float(p)).to(torch.int64)
        out |= bit << j
    out = torch.where(out >= 2 ** 31, out - 2 ** 32, out)
    return out.to(torch.int32)


def uniform_ts(n: int, device, seed: int, days: int = 30) -> torch.Tensor:
    g = _gen(device, seed)
    lo = NOW - days * DAY
    t = torch.randint(lo, NOW, (n,), generator=g, device=device, dtype=torch.int64)
    return torch.where(t >= 2 ** 31, t - 2 ** 32, t).to(torch.int32)


def required_bit_filters(B: int, n_req: int, bit_lo: int, bit_hi: int, seed: int) -> np.ndarray:
    """Each query requires n_req distinct bits drawn from [bit_lo, bit_hi)."""
    rng = np.random.default_rng(seed)
    f = make_filters(B)
    for b in range(B):
        bits = rng.choice(np.arange(bit_lo, bit_hi), size=n_req, replace=False)
        f["all_bits"][b] = np.uint32(sum(1 << int(x) for x in bits))
    return f


# ----------------------------------------------------------------------------
# the five workloads (any of them can be shrunk with n=/B= for tests)
# ----------------------------------------------------------------------------

def _seed(cfg: int, stream: int) -> int:
    return SEED0 + 1000 * cfg + stream


def config1(device="cpu", n=100_000, B=16, k=100):
    d = 64
    emb = l2_normalise(torch.randn(n, d, generator=_gen(device, _seed(1, 1)), device=device))
    Q = l2_normalise(torch.randn(B, 1, d, generator=_gen(device, _seed(1, 4)), device=device))
    mask = bernoulli_masks(n, [0.5] * 32, device, _seed(1, 2))
    filt = required_bit_filters(B, 3, 0, 32, _seed(1, 5))
    return dict(dtype=F32, d=d, m=1, k=k, emb=emb, scale=None, mask=mask, ts=None, Q=Q, q_scale=None, filters=filt)


def config2(device="cpu", n=10_000_000, B=256, k=1000, p=0.5, C=1000, sigma=0.3, chunk=4_000_000, d=128):
    cen = unit_centres(C, d, device, _seed(2, 0))
    emb = torch.empty(n, d, dtype=torch.int16, device=device)
    for i, s in enumerate(range(0, n, chunk)):
        e = min(n, s + chunk)
        emb[s:e] = to_bf16_bits(clustered_rows(e - s, cen, sigma, device, _seed(2, 1) + 7919 * i))
    gq = _gen(device, _seed(2, 4))
    qc = cen[torch.randint(0, C, (B,), generator=gq, device=device)]
    Q = l2_normalise(qc + torch.randn(B, d, generator=gq, device=device) * (sigma / math.sqrt(d)))
    Q = to_bf16_bits(Q).reshape(B, 1, d)
    mask = bernoulli_masks(n, [p] * 32, device, _seed(2, 2))
    filt = required_bit_filters(B, 2, 0, 32, _seed(2, 5))
    return dict(dtype=BF16, d=d, m=1, k=k, emb=emb, scale=None, mask=mask, ts=None, Q=Q, q_scale=None, filters=filt)


def _clustered_int8(n, d, cen, sigma, device, seed, chunk, sort_by_cluster=False):
    emb = torch.empty(n, d, dtype=torch.int8, device=device)
    scale = torch.empty(n, dtype=torch.float32, device=device)
    for i, s in enumerate(range(0, n, chunk)):
        e = min(n, s + chunk)
        c, sc = quantize_rows(clustered_rows(e - s, cen, sigma, device, seed + 7919 * i, sort_by_cluster))
        emb[s:e] = c
        scale[s:e] = sc
    return emb, scale


def config3(device="cpu", n=50_000_000, B=16, k=1000, C=1000, sigma=0.3, chunk=8_000_000):
    d = 64
    cen = unit_centres(C, d, device, _seed(3, 0))
    emb, scale = _clustered_int8(n, d, cen, sigma, device, _seed(3, 1), chunk)
    gq = _gen(device, _seed(3, 4))
    qc = cen[torch.randint(0, C, (B,), generator=gq, device=device)]
    Qf = l2_normalise(qc + torch.randn(B, d, generator=gq, device=device) * (sigma / math.sqrt(d)))
    Q, q_scale = quantize_queries(Qf.reshape(B, 1, d))
    mask = bernoulli_masks(n, [0.3] * 32, device, _seed(3, 2))
    ts = uniform_ts(n, device, _seed(3, 3))
    filt = required_bit_filters(B, 1, 0, 32, _seed(3, 5))
    filt["ts_min"] = NOW - 7 * DAY
    return dict(dtype=I8, d=d, m=1, k=k, emb=emb, scale=scale, mask=mask, ts=ts, Q=Q, q_scale=q_scale, filters=filt)


def config4(device="cpu", n=20_000_000, B=128, m=8, k=500, C=1000, sigma=0.3, chunk=4_000_000):
    d = 64
    cen = unit_centres(C, d, device, _seed(4, 0))
    emb = torch.empty(n, d, dtype=torch.int16, device=device)
    for i, s in enumerate(range(0, n, chunk)):
        e = min(n, s + chunk)
        emb[s:e] = to_bf16_bits(clustered_rows(e - s, cen, sigma, device, _seed(4, 1) + 7919 * i))
    gq = _gen(device, _seed(4, 4))
    qc = cen[torch.randint(0, C, (B * m,), generator=gq, device=device)]      # m different centres per query
    Q = l2_normalise(qc + torch.randn(B * m, d, generator=gq, device=device) * (sigma / math.sqrt(d)))
    Q = to_bf16_bits(Q).reshape(B, m, d)
    p = math.sqrt(0.05)
    mask = bernoulli_masks(n, [p] * 32, device, _seed(4, 2))
    filt = required_bit_filters(B, 2, 0, 32, _seed(4, 5))
    return dict(dtype=BF16, d=d, m=m, k=k, emb=emb, scale=None, mask=mask, ts=None, Q=Q, q_scale=None, filters=filt)


#: cfg 5 bit groups -> (first bit, last bit + 1, per-bit probability, required bits, pass rate)
CFG5_GROUPS = {
    "50%": (0, 8, 0.5, 1),
    "5%": (8, 16, math.sqrt(0.05), 2),
    "0.1%": (16, 24, math.sqrt(0.001), 2),
}


def config5(device="cpu", n=1_000_000_000, B=32, k=1000, selectivity="5%", C=10_000, sigma=0.3,
            chunk=16_000_000, index=None):
    """`index` may carry (emb, scale, mask) of an earlier call so that a sweep over B /
    selectivity reuses the resident 72 GB."""
    d = 64
    cen = unit_centres(C, d, device, _seed(5, 0))
    if index is None:
        emb, scale = _clustered_int8(n, d, cen, sigma, device, _seed(5, 1), chunk)
        p_bits = [0.5] * 8 + [math.sqrt(0.05)] * 8 + [math.sqrt(0.001)] * 8 + [0.5] * 8
        mask = torch.empty(n, dtype=torch.int32, device=device)
        for i, s in enumerate(range(0, n, 4 * chunk)):
            e = min(n, s + 4 * chunk)
            mask[s:e] = bernoulli_masks(e - s, p_bits, device, _seed(5, 2) + 7919 * i)
    else:
        emb, scale, mask = index
    gq = _gen(device, _seed(5, 4) + B)
    qc = cen[torch.randint(0, C, (B,), generator=gq, device=device)]
    Qf = l2_normalise(qc + torch.randn(B, d, generator=gq, device=device) * (sigma / math.sqrt(d)))
    Q, q_scale = quantize_queries(Qf.reshape(B, 1, d))
    lo, hi, _, nreq = CFG5_GROUPS[selectivity]
    filt = required_bit_filters(B, nreq, lo, hi, _seed(5, 5) + B)
    return dict(dtype=I8, d=d, m=1, k=k, emb=emb, scale=scale, mask=mask, ts=None, Q=Q, q_scale=q_scale, filters=filt)


def to_numpy(w: dict) -> dict:
    """Host copies (numpy) of a workload's tensors; masks/ts as uint32, bf16 as uint16."""
    out = dict(w)
    for key in ("emb", "Q"):
        t = w[key].cpu().numpy()
        out[key] = t.view(np.uint16) if w["dtype"] == BF16 else t
    out["mask"] = w["mask"].cpu().numpy().view(np.uint32)
    out["ts"] = None if w["ts"] is None else w["ts"].cpu().numpy().view(np.uint32)
    out["scale"] = None if w["scale"] is None else w["scale"].cpu().numpy()
    out["q_scale"] = None if w["q_scale"] is None else w["q_scale"].cpu().numpy()
    return out


def oporp_draw(d: int, seed: int = 0):
    """The random inputs of Sign-OPORP (one permutation of the d coordinates, one +-1 vector), numpy, seeded.
    They are inputs of the method on both sides; no part of the method is computed here."""
    rng = np.random.default_rng(_seed(9, seed))
    return rng.permutation(d).astype(np.uint32), rng.choice(np.array([-1, 1], np.int8), d)


def oporp_draws(d: int, reps: int, seed: int = 0):
    """`reps` independent draws of the random inputs of Sign-OPORP, as [reps, d] arrays (codes longer than d bits)."""
    rng = np.random.default_rng(_seed(9, 50 + seed))
    perm = np.stack([rng.permutation(d) for _ in range(reps)]).astype(np.uint32)
    return perm, rng.choice(np.array([-1, 1], np.int8), (reps, d))


def random_codes(n: int, k_bits: int, seed: int = 0):
    """n uniformly random codes of k_bits bits as [n, ceil(k_bits/64)] uint64 (unused high bits zero)."""
    rng = np.random.default_rng(_seed(9, 100 + seed))
    W = (k_bits + 63) // 64
    hi = rng.integers(0, 2 ** 63, (n, W), dtype=np.uint64)
    codes = hi * np.uint64(2) + rng.integers(0, 2, (n, W), dtype=np.uint64)
    rem = k_bits - 64 * (W - 1)
    if rem < 64:
        codes[:, W - 1] &= np.uint64((1 << rem) - 1)
    return codes


# ---------------------------------------------------------------------------
# attribute clause lists (the representation of the paper's job-search benchmark, Sec. 5.3: geo-location match,
# company-name reverse match, optionally job-title exact match; one 64-bit attribute per item / query and clause)
# ---------------------------------------------------------------------------
_ATTR_MULT = 0x9E3779B97F4A7C15          # spreads small category numbers over 64 bits (an id, not a hash of anything)


def _zipf_draw(n, categories, s, device, seed):
    """n category numbers in [0, categories) with P(c) proportional to 1 / (c + 1)^s"""
    w = 1.0 / torch.arange(1, categories + 1, dtype=torch.float64, device=device) ** s
    cdf = torch.cumsum(w / w.sum(), 0)
    u = torch.rand(n, generator=_gen(device, seed), device=device, dtype=torch.float64)
    return torch.searchsorted(cdf, u).clamp_(max=categories - 1)


def _attr_ids(cat, clause):
    """64-bit attribute ids (int64 bit patterns) of category numbers; different clauses never share an id"""
    x = (cat.to(torch.int64) + 1 + clause * 1_000_003)
    return x * torch.tensor(_ATTR_MULT - (1 << 64), dtype=torch.int64, device=cat.device)      # wraps modulo 2^64


def job_clauses(device="cpu", n=15_500_000, B=16, low_pass=False, seed=0):
    """values [n, C] int64, counts [n, C] uint8 (all ones), reverse mask, and the same for B queries.
    Clause 0 geo (200 categories, Zipf 1.25: about 11 % of the items share a random query's geo), clause 1 company
    (50 000 categories, uniform; REVERSE: items of the query's company are excluded), clause 2 (low_pass) job title
    (20 000 categories, Zipf 1.0: a few titles match up to 9 % of the items, most a few thousand)."""
    C = 3 if low_pass else 2
    spec = [(200, 1.25), (50_000, 0.0), (20_000, 1.0)][:C]
    vals = torch.empty((n, C), dtype=torch.int64, device=device)
    qv = torch.empty((B, C), dtype=torch.int64, device=device)
    for c, (cats, s) in enumerate(spec):
        vals[:, c] = _attr_ids(_zipf_draw(n, cats, s, device, _seed(7, 10 * seed + c)), c)
        qv[:, c] = _attr_ids(_zipf_draw(B, cats, s, device, _seed(7, 10 * seed + 5 + c)), c)
    return dict(values=vals, counts=torch.ones((n, C), dtype=torch.uint8, device=device), reverse=0b10,
                q_values=qv, q_counts=torch.ones((B, C), dtype=torch.uint8, device=device), n_clauses=C)


def random_clause_lists(n, C, max_len, domain, seed, width=None):
    """numpy: n rows of C lists with 0..max_len attributes each from [1, domain] (sorted inside each list), packed back to
    back.  Returns values [n, width] uint64, counts [n, C] uint8."""
    rng = np.random.default_rng(_seed(8, seed))
    width = width or C * max_len
    counts = rng.integers(0, max_len + 1, (n, C), dtype=np.uint8)
    values = np.zeros((n, width), np.uint64)
    draw = rng.integers(1, domain + 1, (n, C, max_len), dtype=np.uint64) * np.uint64(_ATTR_MULT)
    draw.sort(axis=2)
    off = np.zeros(n, np.int64)
    for c in range(C):
        for a in range(max_len):
            sel = counts[:, c] > a
            values[np.flatnonzero(sel), off[sel] + a] = draw[sel, c, a]
        off += counts[:, c]
    return values, counts
