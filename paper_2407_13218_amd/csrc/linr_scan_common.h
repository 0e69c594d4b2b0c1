// Building blocks shared by the scan kernels (linr_kernels.hip, linr_kernels_dense.hip): matrix-core tile
// products, the sweep walker, per-wave candidate segments with in-wave compaction, the final flush into the
// per-query flat arrays, and the survivor path of the 16x16-tile kernels.  (LiNR, arXiv 2407.13218, Sec. 3.1.1:
// scoring and feasibility; Sec. 3.1.2: infeasible items never reach selection.)
#pragma once
#include "linr_device.h"

template <int DT> struct AccOf { typedef v4f type; };
template <> struct AccOf<LINR_I8> { typedef v4i type; };

// One 64-byte K-step of a 16x16 tile: lane l supplies bytes [16*(l/16), +16) of row l%16
// of each operand; the result lane l holds D[4*(l/16)+r][l%16], r = 0..3 (rows = items).
template <int DT>
__device__ __forceinline__ typename AccOf<DT>::type mfma_kstep(v4i a, v4i b, typename AccOf<DT>::type c)
{
    if constexpr (DT == LINR_I8) {
        return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0);
    } else if constexpr (DT == LINR_BF16) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
    } else {
        v4f af = __builtin_bit_cast(v4f, a), bf = __builtin_bit_cast(v4f, b);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(af[0], bf[0], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(af[1], bf[1], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(af[2], bf[2], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(af[3], bf[3], c, 0, 0, 0);
        return c;
    }
}

// ---------------------------------------------------------------------------
// per-wave LDS: the chunk being scored (A operand fragments + side columns).  The
// fragment area doubles as the histogram of the rare in-wave compaction.
// ---------------------------------------------------------------------------
struct WaveLds {
    v4i a[8][64];          // [tile * KS + kstep][lane]
    float sc[128];         // row scales of the chunk's items
    uint32_t mk[128];      // attribute masks
    uint32_t ts[128];      // timestamps
};

// Which of the 256 histogram buckets holds the `need`-th largest element, counting from
// bucket 255 down?  One wave; lane l owns buckets 4l..4l+3.  Returns the bucket, the number of
// elements in higher buckets (`above`) and the bucket's own count.  `hist` must be LDS.
__device__ __forceinline__ void wave_find_bucket(const uint32_t* hist, uint32_t need, int lane,
                                                 uint32_t& bsel, uint32_t& above, uint32_t& in_bucket)
{
    const v4u h = *(const v4u*)(hist + 4 * lane);
    const uint32_t mine = h[0] + h[1] + h[2] + h[3];
    uint32_t suf = mine;                                  // sum over lanes >= this one
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t v = __shfl_down(suf, o);
        if (lane + o < 64) suf += v;
    }
    uint32_t ab = suf - mine;                             // elements in buckets owned by higher lanes
    const bool here = (ab < need) && (need <= suf);
    uint32_t b_l = 0, cnt_l = 0;
    if (here) {
        if (ab + h[3] >= need) { b_l = 4 * lane + 3; cnt_l = h[3]; }
        else if (ab + h[3] + h[2] >= need) { ab += h[3]; b_l = 4 * lane + 2; cnt_l = h[2]; }
        else if (ab + h[3] + h[2] + h[1] >= need) { ab += h[3] + h[2]; b_l = 4 * lane + 1; cnt_l = h[1]; }
        else { ab += h[3] + h[2] + h[1]; b_l = 4 * lane; cnt_l = h[0]; }
    }
    const u64 m = __ballot(here);
    const int src = m ? (__ffsll((long long)m) - 1) : 0;  // m == 0 only if need exceeds the population
    bsel = __shfl(b_l, src);
    above = __shfl(ab, src);
    in_bucket = __shfl(cnt_l, src);
}

// k-th largest of c distinct keys held in global memory, by one wave (rare path).
__device__ __forceinline__ u64 wave_select_kth(const u64* base, uint32_t c, uint32_t k, uint32_t* hist, int lane)
{
    u64 prefix = 0;
    uint32_t need = k;
    for (int shift = 56; shift >= 0; shift -= 8) {
        *(v4u*)(hist + 4 * lane) = (v4u){0, 0, 0, 0};
        wave_sync();
        for (uint32_t idx = lane; idx < c; idx += 64) {
            u64 key = aload64(base + idx);
            bool match = (shift == 56) || ((key >> (shift + 8)) == (prefix >> (shift + 8)));
            if (match) atomicAdd(&hist[(uint32_t)(key >> shift) & 255u], 1u);
        }
        wave_sync();
        uint32_t bsel, above, inb;
        wave_find_bucket(hist, need, lane, bsel, above, inb);
        need -= above;
        prefix |= (u64)bsel << shift;
        wave_sync();
    }
    return prefix;
}

// Shrink one (slot, query) segment to its k best keys and publish the k-th as a bound.
__device__ __forceinline__ void wave_compact_segment(u64* base, uint32_t* cnt_p, u64* tau_p, uint32_t c, uint32_t k,
                                                     uint32_t* hist, int lane)
{
    u64 kth = wave_select_kth(base, c, k, hist, lane);
    uint32_t out = 0;
    for (uint32_t i0 = 0; i0 < c; i0 += 64) {
        uint32_t idx = i0 + lane;
        u64 key = idx < c ? aload64(base + idx) : 0ull;
        bool keep = idx < c && key >= kth;
        u64 bal = __ballot(keep);
        uint32_t rank = __popcll(bal & ((1ull << lane) - 1ull));
        if (keep) __hip_atomic_store(base + out + rank, key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        out += __popcll(bal);
    }
    if (lane == 0) {
        __hip_atomic_store(cnt_p, out, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        atomicMax(tau_p, kth);
    }
    __threadfence();
    wave_sync();
}

// ---------------------------------------------------------------------------
// Scan building blocks shared by the register-resident-query kernel and the kernel
// that streams query fragments from LDS.
// ---------------------------------------------------------------------------
// Position of one chunk-slot inside a sweep.  A sweep with chunk stride S visits the chunks
// c = lc * S whose level index lc is NOT a multiple of skip_mod (those belonged to earlier, coarser
// sweeps; skip_mod == 0: visit every lc).  `di` enumerates the visited chunks densely; slot s takes
// di = s, s + nslots, ...  The (q, r) pair tracks di / (skip_mod-1), di % (skip_mod-1) incrementally.
struct SweepWalk {
    uint32_t di, n_dense, step, mod, m1, q, r, step_q, step_r;
    __device__ __forceinline__ void init(uint32_t slot, const linr_scan_args& A)
    {
        di = slot; n_dense = (uint32_t)A.n_dense; step = A.nslots; mod = A.skip_mod;
        m1 = mod ? mod - 1 : 1; q = r = step_q = step_r = 0;
        if (mod) { q = di / m1; r = di % m1; step_q = step / m1; step_r = step % m1; }
    }
    // the same walk for a slot that is one of `nstep` (not A.nslots) walkers
    __device__ __forceinline__ void init_strided(uint32_t slot, uint32_t nstep, const linr_scan_args& A)
    {
        di = slot; n_dense = (uint32_t)A.n_dense; step = nstep; mod = A.skip_mod;
        m1 = mod ? mod - 1 : 1; q = r = step_q = step_r = 0;
        if (mod) { q = di / m1; r = di % m1; step_q = step / m1; step_r = step % m1; }
    }
    __device__ __forceinline__ bool valid() const { return di < n_dense; }
    __device__ __forceinline__ u64 lc() const { return mod ? (u64)q * mod + r + 1 : (u64)di; }
    __device__ __forceinline__ void advance()
    {
        di = (di + step < di) ? 0xFFFFFFFFu : di + step;      // saturate instead of wrapping
        q += step_q; r += step_r;
        if (r >= m1) { r -= m1; ++q; }
    }
};

template <int VK, int KS>
struct ChunkRegs {
    v4i ra[8];                 // 8 KB of rows in MFMA operand layout
    uint32_t rsc[2], rmk[2], rts[2];   // side columns of items lane and lane + 64 of the chunk
};

// Issue the loads of level chunk `lc` (8 KB of rows + side columns) into registers.
// Fast path (whole chunk inside the index, rows exactly KS*64 bytes): one uniform base plus a
// per-lane 32-bit offset.  General path: rows and side entries past the end of the index are read
// from the last item instead (their candidates are discarded later by the `item < n` test) and
// 16-byte pieces past the end of a short row read as zero.
template <int VK, int KS>
__device__ __forceinline__ void issue_chunk(ChunkRegs<VK, KS>& R, const linr_scan_args& A, u64 lc, int lane, bool has_ts)
{
    constexpr int TPC = 8 / KS;
    constexpr int CH = 16 * TPC;
    const int row = lane & 15, g4 = lane >> 4;
    const char* embp = (const char*)A.emb;
    const uint32_t rb = A.row_bytes;
    const u64 item0 = lc * A.stride * CH;
    if (item0 + CH <= A.n && rb == (uint32_t)KS * 64u) {
        const char* cb = embp + item0 * (u64)(KS * 64);
        const uint32_t lane_off = (uint32_t)row * (KS * 64) + (uint32_t)g4 * 16;
#pragma unroll
        for (int t = 0; t < TPC; ++t)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                R.ra[t * KS + ks] = __builtin_nontemporal_load((const v4i*)(cb + (lane_off + (uint32_t)(t * 16 * KS * 64 + ks * 64))));
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            if (h * 64 < CH && lane < CH - h * 64) {
                const u64 it = item0 + h * 64 + lane;
                if (VK == LINR_VK_I8_SCALED) R.rsc[h] = __builtin_nontemporal_load((const uint32_t*)A.row_scale + it);
                R.rmk[h] = __builtin_nontemporal_load(A.mask + it);
                if (has_ts) R.rts[h] = __builtin_nontemporal_load(A.ts + it);
            }
        }
        return;
    }
    const u64 last = A.n - 1;
#pragma unroll
    for (int t = 0; t < TPC; ++t) {
        u64 it = item0 + t * 16 + row;
        it = it < last ? it : last;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            uint32_t off = ks * 64 + g4 * 16;
            v4i z = {0, 0, 0, 0};
            if (off < rb) z = *(const v4i*)(embp + it * rb + off);
            R.ra[t * KS + ks] = z;
        }
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        if (h * 64 < CH && lane < CH - h * 64) {
            u64 it = item0 + h * 64 + lane;
            it = it < last ? it : last;
            if (VK == LINR_VK_I8_SCALED) R.rsc[h] = ((const uint32_t*)A.row_scale)[it];
            R.rmk[h] = A.mask[it];
            if (has_ts) R.rts[h] = A.ts[it];
        }
    }
}

// registers -> this wave's LDS area; returns max(row scale of the chunk) when asked for
template <int VK, int KS, bool WANT_SMAX>
__device__ __forceinline__ float stage_chunk(const ChunkRegs<VK, KS>& R, WaveLds& L, int lane, bool has_ts)
{
    constexpr int CH = 16 * (8 / KS);
    float smax = 0.0f;
    if constexpr (WANT_SMAX) {
        if (lane < CH) smax = __uint_as_float(R.rsc[0]);
        if (CH > 64 && lane < CH - 64) smax = fmaxf(smax, __uint_as_float(R.rsc[1]));
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) smax = fmaxf(smax, __shfl_xor(smax, o));
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) L.a[j][lane] = R.ra[j];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        if (h * 64 < CH && lane < CH - h * 64) {
            if (VK == LINR_VK_I8_SCALED) L.sc[h * 64 + lane] = __uint_as_float(R.rsc[h]);
            L.mk[h * 64 + lane] = R.rmk[h];
            if (has_ts) L.ts[h * 64 + lane] = R.rts[h];
        }
    }
    wave_sync();
    return smax;
}

// conservative integer form of "raw * row_scale >= thr" for a whole chunk (thr > 0 only)
__device__ __forceinline__ int int_bound(float thr, float smax)
{
    float x = thr * __builtin_amdgcn_rcpf(smax) * 0.999f;
    return (thr > 0.0f) ? ((x >= 2.0e9f) ? INT_MAX : (int)x) : INT_MIN;
}

// Scaled int8 rows of at most 256 dimensions: the accumulator starts at the bit pattern of
// 1.5 * 2^23, so that (bits of accumulator) read as fp32 equal 12582912 + raw exactly
// (|raw| < 2^22).  One fused multiply-add, fma(acc_as_float, scale, -(12582912 - 2) * scale), then
// gives raw * scale + 2 * scale to within 0.75 * scale: never below the exact product for a
// positive scale, and tight enough for the cheap first test (the bound it is compared with is
// additionally lowered by 2^-14 relative).  The exact value is recomputed for survivors.
#define LINR_MAGIC_BITS 0x4B400000
#define LINR_MAGIC_F 12582912.0f
#define LINR_MAGIC_U (12582912.0f - 2.0f)

__device__ __forceinline__ float lowered(float thr)          // thr - 2^-14 |thr| (infinities unchanged)
{
    return (fabsf(thr) < 3.0e38f) ? thr - fabsf(thr) * 6.1035156e-5f : thr;
}
__device__ __forceinline__ float lowered_pos(float thr)      // same, and "no usable bound" for thr <= 0
{
    return thr > 0.0f ? lowered(thr) : -INFINITY;
}
// keep a loop-invariant value in its registers instead of re-materialising it every iteration
__device__ __forceinline__ void pin(v4i& x) { asm volatile("" : "+v"(x)); }
__device__ __forceinline__ void pin(v4f& x) { asm volatile("" : "+v"(x)); }
__device__ __forceinline__ void pin(int& x) { asm volatile("" : "+v"(x)); }

// Query-side state in LDS (pointers to arrays indexed by the wave-local query number).
struct QSide {
    uint32_t* cnt;          // entries appended so far to this wave's segment of the query (wave private)
    float* thr_f;           // lower bound of the ranking value (float kinds)
    int* thr_i;             // same for raw int8 ranking
    const uint32_t* fall;   // filter: bits that must be set            } an item passes both iff
    const uint32_t* fnone;  // filter: all_bits | none_bits (care mask)  } (mask & care) == must
    const uint32_t* tsmin;  // filter: ts window
    const uint32_t* tsmax;
    const uint32_t* fflag;  // bit 0: the filter has any-of clauses (read the full record from global)
};

__device__ __forceinline__ void load_query_side(const QSide& qs, uint32_t ql, uint32_t qi, const linr_scan_args& A,
                                                bool with_filter)
{
    float tf; int ti;
    if (qi < A.B) {
        u64 t = aload64(A.tau + qi);
        uint32_t hi = (uint32_t)(t >> 32);
        tf = t ? unord_f32(hi) : -INFINITY;
        ti = t ? unord_i32(hi) : INT_MIN;
    } else {
        tf = INFINITY;
        ti = INT_MAX;
    }
    qs.thr_f[ql] = tf;
    qs.thr_i[ql] = ti;
    if (with_filter) {
        linr_filter F;
        if (qi < A.B) F = A.filters[qi];
        else { F.all_bits = 0xFFFFFFFFu; F.none_bits = 0xFFFFFFFFu; F.n_any = 0; F.ts_min = 1; F.ts_max = 0; }
        const uint32_t none = F.none_bits | A.dead_bit;                 // a slot marked as empty fails every filter
        const bool impossible = (F.all_bits & none) != 0u;              // a bit both required and forbidden
        ((uint32_t*)qs.fall)[ql] = impossible ? 0xFFFFFFFFu : F.all_bits;
        ((uint32_t*)qs.fnone)[ql] = impossible ? 0u : (F.all_bits | none);
        ((uint32_t*)qs.tsmin)[ql] = F.ts_min;
        ((uint32_t*)qs.tsmax)[ql] = F.ts_max;
        ((uint32_t*)qs.fflag)[ql] = F.n_any ? 1u : 0u;
    }
}

// Stage A for the four items x one query a lane holds after the matrix product: can any of
// them still matter?  Exact for float / raw int.  Scaled int8: with MAGIC accumulators
// fma(acc_as_float, scale, -MAGIC*scale) against a bound lowered by the rounding slack,
// otherwise the conservative per-chunk integer bound.
template <int VK, bool MAGIC, typename acc_t>
__device__ __forceinline__ bool tile_hot(const acc_t& acc, float thr_f, int thr_int, float smax4, float umax4)
{
    if constexpr (VK == LINR_VK_FLOAT) {
        float mx = fmaxf(fmaxf(acc[0], acc[1]), fmaxf(acc[2], acc[3]));
        return mx >= thr_f;
    } else if constexpr (VK == LINR_VK_I8_SCALED && MAGIC) {
        // max_r(raw_r * scale_r) <= max_r(raw_r) * max_r(scale_r) whenever that maximum is >= 0; bounds <= 0 are
        // passed in as -inf by the caller, so a negative maximum is (correctly) never hot against a positive bound
        int mx = max(max(acc[0], acc[1]), max(acc[2], acc[3]));
        return __builtin_fmaf(__int_as_float(mx), smax4, -umax4) >= thr_f;
    } else {
        int mx = max(max(acc[0], acc[1]), max(acc[2], acc[3]));
        return mx >= thr_int;
    }
}

// Stage A with the bitmask / timestamp part of the predicate folded in (used when a wave holds few
// query groups and the pass is HBM-bound, so the vector ALU has time for it): an item only counts
// if it can pass its query's all/none bits and ts window.  Any-of clauses are left to stage C.
template <int VK, bool MAGIC, bool TS, typename acc_t>
__device__ __forceinline__ bool tile_hot_pred(const acc_t& acc, float thr_f, int thr_int, const v4f& sc4, const v4f& u4,
                                              const v4u& mk4, const v4u& ts4, uint32_t fa, uint32_t fn, uint32_t t0, uint32_t t1)
{
    bool hot = false;                         // bitwise, not short-circuit: no divergent branches
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        bool feas = (mk4[r] & fn) == fa;
        if constexpr (TS) feas = feas & ((ts4[r] - t0) <= t1);          // t1 holds ts_max - ts_min here
        bool above;
        if constexpr (VK == LINR_VK_FLOAT) above = acc[r] >= thr_f;
        else if constexpr (VK == LINR_VK_I8_SCALED && MAGIC)
            above = __builtin_fmaf(__int_as_float(acc[r]), sc4[r], -u4[r]) >= thr_f;
        else above = acc[r] >= thr_int;
        hot = hot | (feas & above);
    }
    return hot;
}

// Stages B and C (rare), entered by the whole wave when some lane's stage A fired:
//   B1  the cheap part of the predicate (care-mask compare, ts window) for the lane's four items, only in
//       lanes whose own stage A fired -- at low pass rates most hot tiles end here;
//   B2  exact ranking values of the remaining items against the query's bound;
//   C   any-of clauses (full filter record), key append to the wave's segment of that query.
// QUEUED: the keys go to a wave-private queue in LDS instead (qcount, qkey, qql: count, keys, wave-local query
// numbers; the caller guarantees room for the 256 keys one call can produce) and no global store is made here.
// load_sc / load_ts: callables that return the row scales / timestamps of the lane's four items (v4f / v4u).
template <int VK, bool MAGIC, int CH, bool QUEUED = false, typename acc_t, typename FSc, typename FTs>
__device__ __forceinline__ void tile_survivors(const acc_t& acc, bool lane_hot, const v4u& mk4, uint32_t fa, uint32_t fn,
                                               const QSide& qs, uint32_t ql, uint32_t qi, int ib,
                                               u64 item0, FSc load_sc, FTs load_ts,
                                               const linr_scan_args& A, uint32_t slot, bool has_ts, uint32_t& need_compact,
                                               uint32_t* qcount = nullptr, u64* qkey = nullptr, uint8_t* qql = nullptr)
{
    uint32_t cand = 0;
    v4u ts4 = {0, 0, 0, 0};
    if (lane_hot && qi < A.B) {
        cand = ((mk4[0] & fn) == fa ? 1u : 0u) | ((mk4[1] & fn) == fa ? 2u : 0u) | ((mk4[2] & fn) == fa ? 4u : 0u) |
               ((mk4[3] & fn) == fa ? 8u : 0u);
        if (has_ts) {
            ts4 = load_ts();
            const uint32_t t0 = qs.tsmin[ql], t1 = qs.tsmax[ql];
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (!(ts4[r] >= t0 && ts4[r] <= t1)) cand &= ~(1u << r);
        }
    }
    if (!wave_any(cand != 0u)) return;

    uint32_t surv = 0;
    uint32_t hi[4];
    if constexpr (VK == LINR_VK_I8_SCALED) {
        const float tf = qs.thr_f[ql];
        const v4f sc4 = load_sc();
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int raw = MAGIC ? acc[r] - LINR_MAGIC_BITS : acc[r];
            float s = (float)raw * sc4[r];
            if (s >= tf) surv |= 1u << r;
            hi[r] = ord_f32(s);
        }
    } else if constexpr (VK == LINR_VK_FLOAT) {
        const float tf = qs.thr_f[ql];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (acc[r] >= tf) surv |= 1u << r;
            hi[r] = ord_f32(acc[r]);
        }
    } else {
        const int ti = qs.thr_i[ql];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (acc[r] >= ti) surv |= 1u << r;
            hi[r] = ord_i32(acc[r]);
        }
    }
    surv &= cand;
    if (!wave_any(surv != 0u)) return;

    if (surv) {
        const bool complex = (qs.fflag[ql] & 1u) != 0u;
        u64* seg_p = A.seg + ((u64)slot * A.B + qi) * A.cap;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const u64 item = item0 + ib + r;
            bool ok = ((surv >> r) & 1u) && item < A.n;
            if (ok && complex) ok = filter_pass(A.filters[qi], mk4[r], has_ts, ts4[r]);
            if (ok) {
                u64 key = ((u64)hi[r] << 32) | (u64)(uint32_t)~(uint32_t)item;
                if constexpr (QUEUED) {
                    const uint32_t pos = atomicAdd(qcount, 1u);
                    qkey[pos] = key;
                    qql[pos] = (uint8_t)ql;
                } else {
                    uint32_t pos = atomicAdd(&qs.cnt[ql], 1u);
                    if (pos < A.cap) seg_p[pos] = key;
                    if (pos + 1 + CH > A.cap) need_compact = 1u;
                }
            }
        }
    }
}

// Rare: some segment of this wave (wave-local queries 0 .. nq) is nearly full.
template <int CH>
// (qmap, if given, maps a wave-local query number to its query index; else query q_first + ql)
__device__ __forceinline__ void compact_full_segments(const linr_scan_args& A, const QSide& qs, uint32_t slot, uint32_t q_first,
                                                      uint32_t nq, uint32_t* hist, int lane, const uint16_t* qmap = nullptr)
{
    __threadfence();
    for (uint32_t q0 = 0; q0 < nq; q0 += 64) {
        uint32_t ql = q0 + lane;
        uint32_t c = 0;
        if (ql < nq && (qmap ? (uint32_t)qmap[ql] : q_first + ql) < A.B) c = qs.cnt[ql];
        u64 todo = __ballot(c + CH > A.cap);
        while (todo) {
            int src = __ffsll((long long)todo) - 1;
            todo &= todo - 1;
            uint32_t lsel = q0 + src;
            uint32_t qsel = qmap ? (uint32_t)qmap[lsel] : q_first + lsel;
            uint32_t csel = __shfl(c, src);
            if (csel > A.cap) csel = A.cap;
            wave_compact_segment(A.seg + ((u64)slot * A.B + qsel) * A.cap, &qs.cnt[lsel], A.tau + qsel, csel, A.k, hist, lane);
        }
    }
}

// End of a scan wave: move what it collected for each of its queries into the query's shared flat
// array.  One atomic per non-empty segment reserves the range; the copy itself is done by the whole wave
// over the concatenation of its segments (a prefix over the segment sizes in `scratch`, 2*nq+1 words of
// LDS, tells each lane which segment its element belongs to), so all loads are independent.  If a range
// does not fit, the wave records where the valid part of the flat array ends (fvalid) and leaves those
// keys in the per-slot segment, whose count it publishes for the merge to pick up.
__device__ __forceinline__ void flush_segments(const linr_scan_args& A, const QSide& qs, uint32_t slot, uint32_t q_first,
                                               uint32_t nq, int lane, uint32_t* scratch, const uint16_t* qmap = nullptr)
{
    uint32_t* pre = scratch;               // [nq + 1] exclusive prefix of the sizes to copy
    uint32_t* dstb = scratch + nq + 1;     // [nq] start of the reserved range in the flat array
    uint32_t running = 0;
    for (uint32_t q0 = 0; q0 < nq; q0 += 64) {
        const uint32_t ql = q0 + lane, qi = (qmap && ql < nq) ? (uint32_t)qmap[ql] : q_first + ql;
        uint32_t c = (ql < nq && qi < A.B) ? qs.cnt[ql] : 0u;
        uint32_t base = 0;
        if (c) {
            // the flat array of a query is split into LINR_FLAT_REGIONS regions with one counter each (in its own
            // 64-byte line), so that the waves of a sweep do not all hit one address
            const uint32_t reg = slot % LINR_FLAT_REGIONS;
            const u64 ci = ((u64)qi * LINR_FLAT_REGIONS + reg) * LINR_COUNTER_STRIDE;
            base = atomicAdd(A.gcnt + ci, c);
            if (base + c > A.flat_cap / LINR_FLAT_REGIONS) {
                atomicMin(A.fvalid + ci, base);
                A.cnt[(u64)qi * A.nslots + slot] = c;
                c = 0;
            }
            base += reg * (A.flat_cap / LINR_FLAT_REGIONS);
        }
        uint32_t incl = c;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            uint32_t v = __shfl_up(incl, o);
            if (lane >= o) incl += v;
        }
        if (ql < nq) { pre[ql] = running + incl - c; dstb[ql] = base; }
        running += __shfl(incl, 63);
    }
    if (lane == 0) pre[nq] = running;
    wave_sync();
    for (uint32_t t = lane; t < running; t += 64) {
        uint32_t lo = 0, hi = nq;
        while (hi - lo > 1) {
            uint32_t mid = (lo + hi) >> 1;
            if (pre[mid] <= t) lo = mid; else hi = mid;
        }
        const uint32_t j = t - pre[lo], qi = qmap ? (uint32_t)qmap[lo] : q_first + lo;
        const u64 key = own_load64(A.seg + ((u64)slot * A.B + qi) * A.cap + j);
        A.flat[(u64)qi * A.flat_cap + dstb[lo] + j] = key;
    }
}


template <int QG>
struct WaveQ {
    uint32_t cnt[QG * 16];
    float thr_f[QG * 16];
    int thr_i[QG * 16];
    uint32_t fall[QG * 16], fnone[QG * 16], tsmin[QG * 16], tsmax[QG * 16], fflag[QG * 16];
};
