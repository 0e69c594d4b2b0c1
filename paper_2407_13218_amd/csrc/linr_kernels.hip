// HIP kernels (gfx950 / CDNA4) of the exhaustive filtered top-k path:
//   scan  : streams the item matrix once, scores 16-item x 16-query tiles on the
//           matrix cores, prunes against each query's running lower bound, evaluates
//           the attribute predicate for the survivors only and appends their 64-bit
//           keys to per-(wave slot, query) candidate segments;
//   merge : per query, exact selection of the k best keys over all segments (radix
//           select + bitonic sort), either publishing the k-th key as the next
//           sweep's lower bound or writing the final ids / scores.
// LiNR (arXiv 2407.13218) Sec. 3.1.1 defines the scoring and the feasibility rule,
// Sec. 3.1.2 the pre-filter semantics (infeasible items never reach selection) and
// Sec. 6 "Custom filtering kernel" names the fusion of filter, matrix product and
// top-k that this file implements.
//
// Key of a candidate: (orderable(ranking value) << 32) | ~item_id, so that a larger
// key means "better score, then lower id"; all keys of one query are distinct.
#include "linr_internal.h"
#include <limits.h>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef unsigned long long u64;

#define WPB LINR_WAVES_PER_BLOCK

// ---------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
__device__ __forceinline__ u64 wave_ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }
__device__ __forceinline__ bool wave_any(bool p) { return wave_ballot(p) != 0ull; }

// monotone map fp32 -> uint32 (−0.0 is first folded into +0.0 so that both compare equal)
__device__ __forceinline__ uint32_t ord_f32(float s)
{
    s = s + 0.0f;
    uint32_t u = __float_as_uint(s);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float unord_f32(uint32_t o)
{
    uint32_t u = (o & 0x80000000u) ? (o ^ 0x80000000u) : ~o;
    return __uint_as_float(u);
}
__device__ __forceinline__ uint32_t ord_i32(int x) { return (uint32_t)x ^ 0x80000000u; }
__device__ __forceinline__ int unord_i32(uint32_t o) { return (int)(o ^ 0x80000000u); }

__device__ __forceinline__ u64 aload64(const u64* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// read back what this wave itself stored earlier (same compute unit, same L2: no device-wide flush needed)
__device__ __forceinline__ u64 own_load64(const u64* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ void own_stores_done()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}
__device__ __forceinline__ uint32_t aload32(const uint32_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Sec. 3.1.1 feasibility rule over the 32-bit attribute mask and the timestamp window
__device__ __forceinline__ bool filter_pass(const linr_filter& f, uint32_t mask, bool has_ts, uint32_t ts)
{
    bool ok = ((mask & f.all_bits) == f.all_bits) && ((mask & f.none_bits) == 0u);
#pragma unroll
    for (uint32_t g = 0; g < (uint32_t)LINR_MAX_ANY; ++g)
        ok = ok && (g >= f.n_any || (mask & f.any_bits[g]) != 0u);
    if (has_ts) ok = ok && (ts >= f.ts_min) && (ts <= f.ts_max);
    return ok;
}

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
        const bool impossible = (F.all_bits & F.none_bits) != 0u;       // a bit both required and forbidden
        ((uint32_t*)qs.fall)[ql] = impossible ? 0xFFFFFFFFu : F.all_bits;
        ((uint32_t*)qs.fnone)[ql] = impossible ? 0u : (F.all_bits | F.none_bits);
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
template <int VK, bool MAGIC, int CH, typename acc_t>
__device__ __forceinline__ void tile_survivors(const acc_t& acc, bool lane_hot, const v4u& mk4, uint32_t fa, uint32_t fn,
                                               const QSide& qs, uint32_t ql, uint32_t qi, int ib,
                                               u64 item0, const float* l_sc, const uint32_t* l_ts,
                                               const linr_scan_args& A, uint32_t slot, bool has_ts, uint32_t& need_compact)
{
    uint32_t cand = 0;
    v4u ts4 = {0, 0, 0, 0};
    if (lane_hot && qi < A.B) {
        cand = ((mk4[0] & fn) == fa ? 1u : 0u) | ((mk4[1] & fn) == fa ? 2u : 0u) | ((mk4[2] & fn) == fa ? 4u : 0u) |
               ((mk4[3] & fn) == fa ? 8u : 0u);
        if (has_ts) {
            ts4 = *(const v4u*)&l_ts[ib];
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
        v4f sc4 = *(const v4f*)&l_sc[ib];
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
                uint32_t pos = atomicAdd(&qs.cnt[ql], 1u);
                if (pos < A.cap) seg_p[pos] = key;
                if (pos + 1 + CH > A.cap) need_compact = 1u;
            }
        }
    }
}

// Rare: some segment of this wave (wave-local queries 0 .. nq) is nearly full.
template <int CH>
__device__ __forceinline__ void compact_full_segments(const linr_scan_args& A, const QSide& qs, uint32_t slot, uint32_t q_first,
                                                      uint32_t nq, uint32_t* hist, int lane)
{
    __threadfence();
    for (uint32_t q0 = 0; q0 < nq; q0 += 64) {
        uint32_t ql = q0 + lane;
        uint32_t c = 0;
        if (ql < nq && q_first + ql < A.B) c = qs.cnt[ql];
        u64 todo = __ballot(c + CH > A.cap);
        while (todo) {
            int src = __ffsll((long long)todo) - 1;
            todo &= todo - 1;
            uint32_t lsel = q0 + src;
            uint32_t qsel = q_first + lsel;
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
                                               uint32_t nq, int lane, uint32_t* scratch)
{
    uint32_t* pre = scratch;               // [nq + 1] exclusive prefix of the sizes to copy
    uint32_t* dstb = scratch + nq + 1;     // [nq] start of the reserved range in the flat array
    uint32_t running = 0;
    for (uint32_t q0 = 0; q0 < nq; q0 += 64) {
        const uint32_t ql = q0 + lane, qi = q_first + ql;
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
        const uint32_t j = t - pre[lo], qi = q_first + lo;
        const u64 key = own_load64(A.seg + ((u64)slot * A.B + qi) * A.cap + j);
        A.flat[(u64)qi * A.flat_cap + dstb[lo] + j] = key;
    }
}

// ---------------------------------------------------------------------------
// scan kernel, queries register resident
//   DT element type, VK ranking-value kind, KS 64-byte K-steps per row,
//   M embeddings per query (max-aggregated), QG 16-query groups per wave.
// Work split: wave `gw` belongs to chunk-slot gw / nsplit and owns query groups
// [split*QG, split*QG+QG); slot s visits level chunks s, s+nslots, ...  No block
// barrier is used, so waves are fully independent.
// ---------------------------------------------------------------------------
template <int QG>
struct WaveQ {
    uint32_t cnt[QG * 16];
    float thr_f[QG * 16];
    int thr_i[QG * 16];
    uint32_t fall[QG * 16], fnone[QG * 16], tsmin[QG * 16], tsmax[QG * 16], fflag[QG * 16];
};

template <int DT, int VK, int KS, int M, int QG, bool TS>
__global__ void __launch_bounds__(64 * WPB, (QG * M * KS <= 1 ? 4 : QG * M * KS <= 4 ? 3 : QG * M * KS <= 8 ? 2 : 1))
scan_kernel(linr_scan_args A)
{
    constexpr int TPC = 8 / KS;
    constexpr int CH = 16 * TPC;
    constexpr int NQ = QG * 16;
    constexpr bool MAGIC = (VK == LINR_VK_I8_SCALED) && (KS * 64 <= 256);
    constexpr bool PRED_A = QG <= 2;           // evaluate all/none bits + ts window already in stage A
    using acc_t = typename AccOf<DT>::type;

    __shared__ WaveLds lds_all[WPB];
    __shared__ WaveQ<QG> wq_all[WPB];
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    WaveLds& L = lds_all[wib];
    WaveQ<QG>& W = wq_all[wib];
    const QSide qs = {W.cnt, W.thr_f, W.thr_i, W.fall, W.fnone, W.tsmin, W.tsmax, W.fflag};
    const int row = lane & 15, g4 = lane >> 4;
    const uint32_t gw = blockIdx.x * WPB + wib;
    const uint32_t split = gw % A.nsplit, slot = gw / A.nsplit;
    if (slot >= A.nslots) return;
    const uint32_t sg0 = split * QG;
    const uint32_t q_first = sg0 * 16;
    const bool has_ts = A.ts != nullptr;
    const uint32_t rb = A.row_bytes;

    // ---- query fragments (B operand)
    v4i q[QG][M][KS];
#pragma unroll
    for (int i = 0; i < QG; ++i) {
        uint32_t qi = (sg0 + i) * 16 + row;
#pragma unroll
        for (int e = 0; e < M; ++e)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                uint32_t off = ks * 64 + g4 * 16;
                v4i z = {0, 0, 0, 0};
                if (qi < A.B && off < rb)
                    z = *(const v4i*)((const char*)A.Q + ((u64)qi * M + e) * rb + off);
                q[i][e][ks] = z;
            }
    }

    // ---- query-side state: segment counters, bounds, compact filters
    for (uint32_t ql = lane; ql < (uint32_t)NQ; ql += 64) {
        W.cnt[ql] = 0;
        load_query_side(qs, ql, q_first + ql, A, true);
    }
    wave_sync();
    float thr_f[QG], thr_lo[QG];          // lane l tracks query row l%16 of each group
    int thr_i[QG];
#pragma unroll
    for (int i = 0; i < QG; ++i) {
        thr_f[i] = W.thr_f[i * 16 + row]; thr_i[i] = W.thr_i[i * 16 + row];
        thr_lo[i] = PRED_A ? lowered(thr_f[i]) : lowered_pos(thr_f[i]);
    }
    uint32_t f_all[QG], f_none[QG], f_t0[QG], f_t1[QG];
#pragma unroll
    for (int i = 0; i < QG; ++i) {
        f_all[i] = W.fall[i * 16 + row]; f_none[i] = W.fnone[i * 16 + row];
        f_t0[i] = W.tsmin[i * 16 + row]; f_t1[i] = W.tsmax[i * 16 + row] - f_t0[i];     // window as (start, length)
        if (W.tsmax[i * 16 + row] < W.tsmin[i * 16 + row]) { f_all[i] = 0xFFFFFFFFu; f_none[i] = 0u; }   // empty window
    }

    ChunkRegs<VK, KS> R;
    R.rsc[0] = R.rsc[1] = R.rmk[0] = R.rmk[1] = R.rts[0] = R.rts[1] = 0u;
    uint32_t need_compact = 0u;
    uint32_t since_refresh = 0;
    SweepWalk walk;
    walk.init(slot, A);
    u64 lc = walk.lc();
    if (walk.valid()) issue_chunk<VK, KS>(R, A, lc, lane, has_ts);
    acc_t acc0 = MAGIC ? (acc_t){LINR_MAGIC_BITS, LINR_MAGIC_BITS, LINR_MAGIC_BITS, LINR_MAGIC_BITS} : (acc_t){0, 0, 0, 0};
    pin(acc0);

    while (walk.valid()) {
        const u64 item0 = lc * A.stride * CH;
        const float smax = stage_chunk<VK, KS, (VK == LINR_VK_I8_SCALED && !MAGIC)>(R, L, lane, has_ts);
        // bounds in the form stage A compares against
        float tcf[QG];
        int tci[QG];
#pragma unroll
        for (int i = 0; i < QG; ++i) {
            tcf[i] = (VK == LINR_VK_I8_SCALED && MAGIC) ? thr_lo[i] : thr_f[i];      // thr_lo: see below
            tci[i] = (VK == LINR_VK_I8_SCALED && !MAGIC) ? int_bound(thr_f[i], smax) : thr_i[i];
        }

        walk.advance();
        const u64 nlc = walk.lc();
        if (walk.valid()) issue_chunk<VK, KS>(R, A, nlc, lane, has_ts);               // in flight while scoring

#pragma unroll 1
        for (int t = 0; t < TPC; ++t) {
            v4i a[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) a[ks] = L.a[t * KS + ks][lane];
            const int ib = t * 16 + 4 * g4;              // first of this lane's four items in the chunk
            v4f sc4 = {0, 0, 0, 0}, u4 = {0, 0, 0, 0};
            float smax4 = 0.0f, umax4 = 0.0f;
            if constexpr (MAGIC) {
                sc4 = *(const v4f*)&L.sc[ib];
                if constexpr (PRED_A) u4 = sc4 * LINR_MAGIC_U;
                else { smax4 = fmaxf(fmaxf(sc4[0], sc4[1]), fmaxf(sc4[2], sc4[3])); umax4 = smax4 * LINR_MAGIC_U; }
            }
            const v4u mk4 = *(const v4u*)&L.mk[ib];
            v4u ts4 = {0, 0, 0, 0};
            if constexpr (PRED_A && TS) ts4 = *(const v4u*)&L.ts[ib];
            // all matrix products of the tile first, then one branch-free pass of stage A over the groups
            acc_t acc[QG];
#pragma unroll
            for (int i = 0; i < QG; ++i) {
#pragma unroll
                for (int e = 0; e < M; ++e) {
                    acc_t tmp = acc0;
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) tmp = mfma_kstep<DT>(a[ks], q[i][e][ks], tmp);
                    if (e == 0) acc[i] = tmp;
                    else {
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[i][r] = acc[i][r] > tmp[r] ? acc[i][r] : tmp[r];
                    }
                }
            }
            u64 hot[QG];
            u64 any_hot = 0;
#pragma unroll
            for (int i = 0; i < QG; ++i) {
                if constexpr (PRED_A)
                    hot[i] = wave_ballot(tile_hot_pred<VK, MAGIC, TS>(acc[i], tcf[i], tci[i], sc4, u4, mk4, ts4, f_all[i], f_none[i],
                                                                   f_t0[i], f_t1[i]));
                else
                    hot[i] = wave_ballot(tile_hot<VK, MAGIC>(acc[i], tcf[i], tci[i], smax4, umax4));
                any_hot |= hot[i];
            }
            if (any_hot) {
#pragma unroll
                for (int i = 0; i < QG; ++i)
                    if (hot[i])
                        tile_survivors<VK, MAGIC, CH>(acc[i], (hot[i] >> lane) & 1ull, mk4, f_all[i], f_none[i], qs, i * 16 + row,
                                                      q_first + i * 16 + row, ib, item0, L.sc, L.ts, A, slot, has_ts, need_compact);
            }
        }
        wave_sync();

        bool refresh = ++since_refresh >= 16;
        if (wave_any(need_compact != 0u)) {
            compact_full_segments<CH>(A, qs, slot, q_first, NQ, (uint32_t*)&L.a[0][0], lane);
            need_compact = 0u;
            refresh = true;
        }
        if (refresh) {
            for (uint32_t ql = lane; ql < (uint32_t)NQ; ql += 64) load_query_side(qs, ql, q_first + ql, A, false);
            wave_sync();
#pragma unroll
            for (int i = 0; i < QG; ++i) {
                thr_f[i] = W.thr_f[i * 16 + row]; thr_i[i] = W.thr_i[i * 16 + row];
                thr_lo[i] = PRED_A ? lowered(thr_f[i]) : lowered_pos(thr_f[i]);
            }
            since_refresh = 0;
        }
        lc = nlc;
    }
    own_stores_done();
    flush_segments(A, qs, slot, q_first, NQ, lane, (uint32_t*)&L);       // the chunk staging area is free now
}

// ---------------------------------------------------------------------------
// scan kernel, workgroup-cooperative: the four waves of a workgroup form ONE chunk-slot.  Each
// wave loads a quarter of every chunk into a shared, double-buffered LDS area (one barrier per
// chunk) and scores the whole chunk against its own QG query groups (wave w owns groups
// [w*QG, w*QG+QG)), so 4*QG*16 queries are answered per pass while every wave keeps only QG
// groups of fragments and accumulators in registers -- several waves per SIMD stay resident and
// the matrix pipe of one wave overlaps the vector work of another.
// ---------------------------------------------------------------------------
struct ChunkLds {
    v4i a[8][64];
    float sc[128];
    uint32_t mk[128];
    uint32_t ts[128];
};

template <int VK, int KS>
struct CoopRegs {
    v4i ra[2];
    uint32_t rsc, rmk, rts;
};

template <int VK, int KS>
__device__ __forceinline__ void issue_coop(CoopRegs<VK, KS>& R, const linr_scan_args& A, u64 lc, int lane, int wib, bool has_ts)
{
    constexpr int TPC = 8 / KS;
    constexpr int CH = 16 * TPC;
    const int row = lane & 15, g4 = lane >> 4;
    const char* embp = (const char*)A.emb;
    const uint32_t rb = A.row_bytes;
    const u64 item0 = lc * A.stride * CH;
    const u64 last = A.n - 1;
    const bool fast = item0 + CH <= A.n && rb == (uint32_t)KS * 64u;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int f = wib * 2 + j, t = f / KS, ks = f % KS;
        if (fast) {
            R.ra[j] = __builtin_nontemporal_load((const v4i*)(embp + item0 * (u64)(KS * 64) +
                                                            ((uint32_t)(t * 16 + row) * (KS * 64) + (uint32_t)(ks * 64 + g4 * 16))));
        } else {
            u64 it = item0 + t * 16 + row;
            it = it < last ? it : last;
            uint32_t off = ks * 64 + g4 * 16;
            v4i z = {0, 0, 0, 0};
            if (off < rb) z = *(const v4i*)(embp + it * rb + off);
            R.ra[j] = z;
        }
    }
    const int idx = wib * 32 + lane;
    if (lane < 32 && idx < CH) {
        u64 it = item0 + idx;
        it = it < last ? it : last;
        if (VK == LINR_VK_I8_SCALED) R.rsc = __builtin_nontemporal_load((const uint32_t*)A.row_scale + it);
        R.rmk = __builtin_nontemporal_load(A.mask + it);
        if (has_ts) R.rts = __builtin_nontemporal_load(A.ts + it);
    }
}

template <int VK, int KS>
__device__ __forceinline__ void stage_coop(const CoopRegs<VK, KS>& R, ChunkLds& C, int lane, int wib, bool has_ts)
{
    constexpr int CH = 16 * (8 / KS);
    C.a[wib * 2][lane] = R.ra[0];
    C.a[wib * 2 + 1][lane] = R.ra[1];
    const int idx = wib * 32 + lane;
    if (lane < 32 && idx < CH) {
        if (VK == LINR_VK_I8_SCALED) C.sc[idx] = __uint_as_float(R.rsc);
        C.mk[idx] = R.rmk;
        if (has_ts) C.ts[idx] = R.rts;
    }
}

template <int DT, int VK, int KS, int M, int QG>
__global__ void __launch_bounds__(64 * WPB, (QG * M * KS <= 2 ? 4 : QG * M * KS <= 8 ? 3 : 2)) scan_kernel_coop(linr_scan_args A)
{
    constexpr int TPC = 8 / KS;
    constexpr int CH = 16 * TPC;
    constexpr int NQ = QG * 16;
    constexpr bool MAGIC = (VK == LINR_VK_I8_SCALED);
    static_assert(VK != LINR_VK_I8_SCALED || KS * 64 <= 256, "scaled int8 rows longer than 256 use another kernel");
    using acc_t = typename AccOf<DT>::type;

    __shared__ ChunkLds chunk[2];
    __shared__ WaveQ<QG> wq_all[WPB];
    __shared__ uint32_t hist_all[WPB][256];
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    WaveQ<QG>& W = wq_all[wib];
    const QSide qs = {W.cnt, W.thr_f, W.thr_i, W.fall, W.fnone, W.tsmin, W.tsmax, W.fflag};
    const int row = lane & 15, g4 = lane >> 4;
    const uint32_t slot = blockIdx.x;
    if (slot >= A.nslots) return;                       // uniform for the workgroup
    const uint32_t sg0 = wib * QG;
    const uint32_t q_first = sg0 * 16;
    const bool active = q_first < A.B;                  // waves past the batch still load and synchronise
    const bool has_ts = A.ts != nullptr;
    const uint32_t rb = A.row_bytes;

    v4i q[QG][M][KS];
#pragma unroll
    for (int i = 0; i < QG; ++i) {
        uint32_t qi = (sg0 + i) * 16 + row;
#pragma unroll
        for (int e = 0; e < M; ++e)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                uint32_t off = ks * 64 + g4 * 16;
                v4i z = {0, 0, 0, 0};
                if (qi < A.B && off < rb)
                    z = *(const v4i*)((const char*)A.Q + ((u64)qi * M + e) * rb + off);
                q[i][e][ks] = z;
            }
    }
    for (uint32_t ql = lane; ql < (uint32_t)NQ; ql += 64) {
        W.cnt[ql] = 0;
        load_query_side(qs, ql, q_first + ql, A, true);
    }
    wave_sync();
    float tcf[QG];            // lane l tracks query row l%16 of each group; already in stage A's form
    int tci[QG];
    uint32_t f_all[QG], f_none[QG];
#pragma unroll
    for (int i = 0; i < QG; ++i) {
        tcf[i] = MAGIC ? lowered_pos(W.thr_f[i * 16 + row]) : W.thr_f[i * 16 + row];
        tci[i] = W.thr_i[i * 16 + row];
        f_all[i] = W.fall[i * 16 + row]; f_none[i] = W.fnone[i * 16 + row];
    }

    CoopRegs<VK, KS> R;
    R.rsc = R.rmk = R.rts = 0u;
    uint32_t need_compact = 0u;
    uint32_t since_refresh = 0;
    acc_t acc0 = MAGIC ? (acc_t){LINR_MAGIC_BITS, LINR_MAGIC_BITS, LINR_MAGIC_BITS, LINR_MAGIC_BITS} : (acc_t){0, 0, 0, 0};
    pin(acc0);
    SweepWalk walk;
    walk.init(slot, A);
    u64 lc = walk.lc();
    if (walk.valid()) issue_coop<VK, KS>(R, A, lc, lane, wib, has_ts);
    int buf = 0;

    while (walk.valid()) {
        const u64 item0 = lc * A.stride * CH;
        ChunkLds& C = chunk[buf];
        stage_coop<VK, KS>(R, C, lane, wib, has_ts);
        __syncthreads();
        walk.advance();
        const u64 nlc = walk.lc();
        if (walk.valid()) issue_coop<VK, KS>(R, A, nlc, lane, wib, has_ts);

        if (active) {
#pragma unroll 1
            for (int t = 0; t < TPC; ++t) {
                v4i a[KS];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) a[ks] = C.a[t * KS + ks][lane];
                const int ib = t * 16 + 4 * g4;
                float smax4 = 0.0f, umax4 = 0.0f;
                if constexpr (MAGIC) {
                    v4f sc4 = *(const v4f*)&C.sc[ib];
                    smax4 = fmaxf(fmaxf(sc4[0], sc4[1]), fmaxf(sc4[2], sc4[3]));
                    umax4 = smax4 * LINR_MAGIC_U;
                }
                const v4u mk4 = *(const v4u*)&C.mk[ib];
                acc_t acc[QG];
#pragma unroll
                for (int i = 0; i < QG; ++i) {
#pragma unroll
                    for (int e = 0; e < M; ++e) {
                        acc_t tmp = acc0;
#pragma unroll
                        for (int ks = 0; ks < KS; ++ks) tmp = mfma_kstep<DT>(a[ks], q[i][e][ks], tmp);
                        if (e == 0) acc[i] = tmp;
                        else {
#pragma unroll
                            for (int r = 0; r < 4; ++r) acc[i][r] = acc[i][r] > tmp[r] ? acc[i][r] : tmp[r];
                        }
                    }
                }
                u64 hot[QG];
                u64 any_hot = 0;
#pragma unroll
                for (int i = 0; i < QG; ++i) {
                    hot[i] = wave_ballot(tile_hot<VK, MAGIC>(acc[i], tcf[i], tci[i], smax4, umax4));
                    any_hot |= hot[i];
                }
                if (any_hot) {
#pragma unroll
                    for (int i = 0; i < QG; ++i)
                        if (hot[i])
                            tile_survivors<VK, MAGIC, CH>(acc[i], (hot[i] >> lane) & 1ull, mk4, f_all[i], f_none[i], qs, i * 16 + row,
                                                          q_first + i * 16 + row, ib, item0, C.sc, C.ts, A, slot, has_ts, need_compact);
                }
            }
            bool refresh = ++since_refresh >= 16;
            if (wave_any(need_compact != 0u)) {
                compact_full_segments<CH>(A, qs, slot, q_first, NQ, hist_all[wib], lane);
                need_compact = 0u;
                refresh = true;
            }
            if (refresh) {
                for (uint32_t ql = lane; ql < (uint32_t)NQ; ql += 64) load_query_side(qs, ql, q_first + ql, A, false);
                wave_sync();
#pragma unroll
                for (int i = 0; i < QG; ++i) {
                    tcf[i] = MAGIC ? lowered_pos(W.thr_f[i * 16 + row]) : W.thr_f[i * 16 + row];
                    tci[i] = W.thr_i[i * 16 + row];
                }
                since_refresh = 0;
            }
        }
        lc = nlc;
        buf ^= 1;
    }
    if (active) {
        own_stores_done();
        flush_segments(A, qs, slot, q_first, NQ, lane, hist_all[wib]);   // 2 * NQ + 1 <= 256 words
    }
}

// ---------------------------------------------------------------------------
// scan kernel, query fragments and query-side state streamed from LDS: any m, any
// number of query groups (up to the LDS budget the host plans for); one chunk-slot per
// wave.  Dynamic LDS: [n_frag][64] v4i fragments, 7 workgroup-shared arrays of nq16
// words (bounds, compact filters), then one counter array of nq16 words per wave.
// ---------------------------------------------------------------------------
template <int DT, int VK, int KS>
__global__ void __launch_bounds__(64 * WPB) scan_kernel_lds(linr_scan_args A)
{
    constexpr int TPC = 8 / KS;
    constexpr int CH = 16 * TPC;
    constexpr bool MAGIC = (VK == LINR_VK_I8_SCALED) && (KS * 64 <= 256);
    using acc_t = typename AccOf<DT>::type;

    __shared__ WaveLds lds_all[WPB];
    extern __shared__ v4i dyn_lds[];
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    WaveLds& L = lds_all[wib];
    const int row = lane & 15, g4 = lane >> 4;
    const uint32_t slot = blockIdx.x * WPB + wib;
    const bool has_ts = A.ts != nullptr;
    const uint32_t rb = A.row_bytes;
    const uint32_t nsg = (A.B + 15) / 16, m = A.m, nq16 = nsg * 16;
    const uint32_t nfrag = nsg * m * KS;
    v4i* qf = dyn_lds;
    uint32_t* words = (uint32_t*)(dyn_lds + (size_t)nfrag * 64);
    const QSide qs = {words + 7 * nq16 + wib * nq16, (float*)words, (int*)(words + nq16), words + 2 * nq16, words + 3 * nq16,
                      words + 4 * nq16, words + 5 * nq16, words + 6 * nq16};

    for (uint32_t f = wib; f < nfrag; f += WPB) {
        uint32_t ks = f % KS, e = (f / KS) % m, sg = f / (KS * m);
        uint32_t qi = sg * 16 + row, off = ks * 64 + g4 * 16;
        v4i z = {0, 0, 0, 0};
        if (qi < A.B && off < rb) z = *(const v4i*)((const char*)A.Q + ((u64)qi * m + e) * rb + off);
        qf[(size_t)f * 64 + lane] = z;
    }
    for (uint32_t ql = threadIdx.x; ql < nq16; ql += 64 * WPB) load_query_side(qs, ql, ql, A, true);
    for (uint32_t ql = lane; ql < nq16; ql += 64) qs.cnt[ql] = 0;
    __syncthreads();
    if (slot >= A.nslots) return;

    ChunkRegs<VK, KS> R;
    R.rsc[0] = R.rsc[1] = R.rmk[0] = R.rmk[1] = R.rts[0] = R.rts[1] = 0u;
    uint32_t need_compact = 0u;
    SweepWalk walk;
    walk.init(slot, A);
    u64 lc = walk.lc();
    if (walk.valid()) issue_chunk<VK, KS>(R, A, lc, lane, has_ts);
    acc_t acc0 = MAGIC ? (acc_t){LINR_MAGIC_BITS, LINR_MAGIC_BITS, LINR_MAGIC_BITS, LINR_MAGIC_BITS} : (acc_t){0, 0, 0, 0};
    pin(acc0);

    while (walk.valid()) {
        const u64 item0 = lc * A.stride * CH;
        const float smax = stage_chunk<VK, KS, (VK == LINR_VK_I8_SCALED && !MAGIC)>(R, L, lane, has_ts);
        walk.advance();
        const u64 nlc = walk.lc();
        if (walk.valid()) issue_chunk<VK, KS>(R, A, nlc, lane, has_ts);

#pragma unroll 1
        for (int t = 0; t < TPC; ++t) {
            v4i a[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) a[ks] = L.a[t * KS + ks][lane];
            const int ib = t * 16 + 4 * g4;
            float smax4 = 0.0f, umax4 = 0.0f;
            if constexpr (MAGIC) {
                v4f sc4 = *(const v4f*)&L.sc[ib];
                smax4 = fmaxf(fmaxf(sc4[0], sc4[1]), fmaxf(sc4[2], sc4[3]));
                umax4 = smax4 * LINR_MAGIC_U;
            }
            const v4u mk4 = *(const v4u*)&L.mk[ib];
#pragma unroll 1
            for (uint32_t sg = 0; sg < nsg; ++sg) {
                acc_t acc;
#pragma unroll 1
                for (uint32_t e = 0; e < m; ++e) {
                    acc_t tmp = acc0;
                    const v4i* qp = qf + ((size_t)(sg * m + e) * KS) * 64 + lane;
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) tmp = mfma_kstep<DT>(a[ks], qp[ks * 64], tmp);
                    if (e == 0) acc = tmp;
                    else {
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[r] = acc[r] > tmp[r] ? acc[r] : tmp[r];
                    }
                }
                const uint32_t qi = sg * 16 + row;
                float tf = qs.thr_f[qi];
                int tc = qs.thr_i[qi];
                if constexpr (VK == LINR_VK_I8_SCALED) {
                    if constexpr (MAGIC) tf = lowered_pos(tf);
                    else tc = int_bound(tf, smax);
                }
                const bool lane_hot = tile_hot<VK, MAGIC>(acc, tf, tc, smax4, umax4);
                if (wave_any(lane_hot))
                    tile_survivors<VK, MAGIC, CH>(acc, lane_hot, mk4, qs.fall[qi], qs.fnone[qi], qs, qi, qi, ib, item0, L.sc, L.ts, A,
                                                  slot, has_ts, need_compact);
            }
        }
        wave_sync();

        if (wave_any(need_compact != 0u)) {
            compact_full_segments<CH>(A, qs, slot, 0, nq16, (uint32_t*)&L.a[0][0], lane);
            need_compact = 0u;
            // publish the raised bounds to the workgroup (monotone, so a racing reader is only conservative)
            for (uint32_t ql = lane; ql < nq16; ql += 64) load_query_side(qs, ql, ql, A, false);
            wave_sync();
        }
        lc = nlc;
    }
    own_stores_done();
    flush_segments(A, qs, slot, 0, nq16, lane, (uint32_t*)&L);           // 2 * nq16 + 1 words <= the staging area
}

// ---------------------------------------------------------------------------
// init: no bound yet, nothing carried, all segments empty
// ---------------------------------------------------------------------------
__global__ void init_kernel(u64* tau, uint32_t* ccnt, uint32_t* gcnt, uint32_t* fvalid, uint32_t* cnt, u64 n_cnt, uint32_t B)
{
    u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    u64 stride = (u64)gridDim.x * blockDim.x;
    for (u64 j = i; j < n_cnt; j += stride) cnt[j] = 0;
    for (u64 j = i; j < B; j += stride) { tau[j] = 0; ccnt[j] = 0; }
    const u64 nreg = (u64)B * LINR_FLAT_REGIONS;
    for (u64 j = i; j < nreg; j += stride) { gcnt[j * LINR_COUNTER_STRIDE] = 0; fvalid[j * LINR_COUNTER_STRIDE] = 0xFFFFFFFFu; }
}

// ---------------------------------------------------------------------------
// merge kernel: one workgroup of 1024 lanes per query.
// Candidates of query b: the keys carried from the previous merge (carry[b][0 .. ccnt[b])), the regions of
// its flat array that the scan waves flushed into, and -- only if some wave could not flush (a region's
// fvalid was lowered) -- the per-slot segments.  Exact selection of the k best: 8-bit radix select (keys are
// distinct), then either carry them to the next sweep (and publish the k-th as its bound) or sort and write
// the result.
// ---------------------------------------------------------------------------
#define MT 1024
#define MERGE_LDS_KEYS 8192
#define NPIECE (LINR_FLAT_REGIONS + 1)
struct MergeLds {
    union {
        u64 keys[MERGE_LDS_KEYS];                 // all candidates, when they fit and nothing was spilled
        uint32_t pre[LINR_MAX_SLOTS + 1];         // exclusive prefix of segment counts (spilled case)
    } u;
    u64 win[LINR_MAX_K];
    uint32_t part[MT];
    uint32_t hist[256];
    uint32_t ppre[NPIECE + 1];                    // exclusive prefix over carry + flat regions
    uint32_t nwin, bsel, above, done, spilled;
};

enum { MERGE_FROM_LDS = 0, MERGE_FROM_FLAT = 1, MERGE_FROM_ALL = 2 };

// start of piece p of query b (piece 0: carried keys, piece r + 1: region r of the flat array)
__device__ __forceinline__ const u64* piece_ptr(const linr_merge_args& A, uint32_t b, uint32_t p)
{
    if (p == 0) return A.carry + (u64)b * A.k;
    return A.flat + (u64)b * A.flat_cap + (u64)(p - 1) * (A.flat_cap / LINR_FLAT_REGIONS);
}

// Calls f(key) once for every candidate of the query, by the whole workgroup.  From LDS when they were
// staged there; else wave w walks pieces w, w + 16, ... with consecutive lanes on consecutive keys; the
// per-slot segments (spilled case only) are located through the prefix array.
template <typename F>
__device__ __forceinline__ void for_each_candidate(const linr_merge_args& A, const MergeLds& S, int mode, uint32_t m_flat,
                                                   uint32_t Mtot, uint32_t b, uint32_t tid, F f)
{
    if (mode == MERGE_FROM_LDS) {
        for (uint32_t i = tid; i < m_flat; i += MT) f(S.u.keys[i]);
        return;
    }
    const uint32_t wave = tid >> 6, lane = tid & 63;
    for (uint32_t p = wave; p < NPIECE; p += MT / 64) {
        const uint32_t c = S.ppre[p + 1] - S.ppre[p];
        const u64* src = piece_ptr(A, b, p);
        for (uint32_t j = lane; j < c; j += 64) f(src[j]);
    }
    if (mode == MERGE_FROM_ALL) {
        for (uint32_t g = tid; g < Mtot - m_flat; g += MT) {
            uint32_t lo = 0, hi = A.nslots;
            while (hi - lo > 1) {
                uint32_t mid = (lo + hi) >> 1;
                if (S.u.pre[mid] <= g) lo = mid; else hi = mid;
            }
            f(A.seg[((u64)lo * A.B + b) * A.cap + (g - S.u.pre[lo])]);
        }
    }
}

__device__ __forceinline__ int dot_i8_row(const int8_t* q, const int8_t* x, uint32_t d)
{
    int s = 0;
    for (uint32_t j = 0; j < d; ++j) s += (int)q[j] * (int)x[j];
    return s;
}

__global__ void __launch_bounds__(MT) merge_kernel(linr_merge_args A)
{
    __shared__ MergeLds S;
    const uint32_t b = blockIdx.x, tid = threadIdx.x;
    const uint32_t ns = A.nslots;
    uint32_t* cnt = A.cnt + (u64)b * ns;

    // 1. where the candidates are
    if (tid == 0) S.spilled = 0;
    __syncthreads();
    if (tid < 64) {                                    // NPIECE = 65 pieces: lane 0 also takes the carry
        const uint32_t rcap = A.flat_cap / LINR_FLAT_REGIONS;
        const u64 ci = ((u64)b * LINR_FLAT_REGIONS + tid) * LINR_COUNTER_STRIDE;
        uint32_t m = A.gcnt[ci];
        const uint32_t fv = A.fvalid[ci];
        if (fv != 0xFFFFFFFFu) S.spilled = 1;
        if (m > fv) m = fv;
        if (m > rcap) m = rcap;
        uint32_t incl = m;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            uint32_t v = __shfl_up(incl, o);
            if ((int)tid >= o) incl += v;
        }
        uint32_t cc = A.ccnt[b];
        if (cc > A.k) cc = A.k;
        S.ppre[tid + 1] = cc + incl - m;              // region tid is piece tid + 1
        if (tid == 0) S.ppre[0] = 0;
        if (tid == 63) S.ppre[NPIECE] = cc + incl;
    }
    __syncthreads();
    const uint32_t m_flat = S.ppre[NPIECE];
    const bool spilled = S.spilled != 0;
    uint32_t Mtot = m_flat;
    int mode;
    if (spilled) {
        mode = MERGE_FROM_ALL;
        const uint32_t per = (ns + MT - 1) / MT;
        uint32_t local = 0;
        for (uint32_t j = 0; j < per; ++j) {
            uint32_t s = tid * per + j;
            if (s < ns) { uint32_t c = cnt[s]; local += c < A.cap ? c : A.cap; }
        }
        S.part[tid] = local;
        __syncthreads();
        for (uint32_t o = 1; o < MT; o <<= 1) {
            uint32_t v = tid >= o ? S.part[tid - o] : 0;
            __syncthreads();
            S.part[tid] += v;
            __syncthreads();
        }
        uint32_t run = S.part[tid] - local;
        for (uint32_t j = 0; j < per; ++j) {
            uint32_t s = tid * per + j;
            if (s < ns) { S.u.pre[s] = run; uint32_t c = cnt[s]; run += c < A.cap ? c : A.cap; }
        }
        if (tid == MT - 1) S.u.pre[ns] = S.part[MT - 1];
        __syncthreads();
        Mtot += S.u.pre[ns];
    } else if (m_flat <= MERGE_LDS_KEYS) {
        // stage everything in LDS: wave w copies pieces w, w + 16, ...
        const uint32_t wave = tid >> 6, lane = tid & 63;
        for (uint32_t p = wave; p < NPIECE; p += MT / 64) {
            const uint32_t o = S.ppre[p], c = S.ppre[p + 1] - o;
            const u64* src = piece_ptr(A, b, p);
            for (uint32_t j = lane; j < c; j += 64) S.u.keys[o + j] = src[j];
        }
        mode = MERGE_FROM_LDS;
        __syncthreads();
    } else {
        mode = MERGE_FROM_FLAT;
    }

    // 2. k-th largest key.  Once the remaining bucket is taken whole the low bits of the bound may stay zero:
    //    the selected set is already fixed.  A bound that seeds the next sweep is resolved down to the full
    //    score word first.
    u64 kth = 0;
    if (Mtot >= A.k) {
        u64 prefix = 0;
        uint32_t need = A.k;
        for (int shift = 56; shift >= 0; shift -= 8) {
            if (tid < 256) S.hist[tid] = 0;
            __syncthreads();
            const u64 want = shift == 56 ? 0ull : (prefix >> (shift + 8));
            for_each_candidate(A, S, mode, m_flat, Mtot, b, tid, [&](u64 key) {
                const bool match = (shift == 56) || ((key >> (shift + 8)) == want);
                if (match) atomicAdd(&S.hist[(uint32_t)(key >> shift) & 255u], 1u);
            });
            __syncthreads();
            if (tid < 64) {
                uint32_t bsel, above, inb;
                wave_find_bucket(S.hist, need, (int)tid, bsel, above, inb);
                if (tid == 0) { S.bsel = bsel; S.above = above; S.done = (inb == need - above) ? 1u : 0u; }
            }
            __syncthreads();
            need -= S.above;
            prefix |= (u64)S.bsel << shift;
            const uint32_t done = S.done;
            __syncthreads();
            if (done && (A.final_level || shift <= 32)) break;
        }
        kth = prefix;
    }
    if (!A.final_level && tid == 0 && Mtot >= A.k) {
        u64 cur = A.tau[b];
        if (kth > cur) A.tau[b] = kth;
    }

    // 3. gather the winners (all candidates when there are fewer than k)
    if (tid == 0) S.nwin = 0;
    __syncthreads();
    for_each_candidate(A, S, mode, m_flat, Mtot, b, tid, [&](u64 key) {
        if (key >= kth) {
            uint32_t p = atomicAdd(&S.nwin, 1u);
            if (p < LINR_MAX_K) S.win[p] = key;
        }
    });
    __syncthreads();
    const uint32_t nwin = S.nwin < A.k ? S.nwin : A.k;

    if (!A.final_level) {
        // carry them into the next sweep's merge and empty the flat regions
        for (uint32_t j = tid; j < nwin; j += MT) A.carry[(u64)b * A.k + j] = S.win[j];
        if (tid == 0) A.ccnt[b] = nwin;
        if (tid < LINR_FLAT_REGIONS) {
            const u64 ci = ((u64)b * LINR_FLAT_REGIONS + tid) * LINR_COUNTER_STRIDE;
            A.gcnt[ci] = 0; A.fvalid[ci] = 0xFFFFFFFFu;
        }
    } else {
        // sort them, write the outputs
        uint32_t P = 1;
        while (P < nwin) P <<= 1;
        for (uint32_t j = nwin + tid; j < P; j += MT) S.win[j] = 0ull;
        __syncthreads();
        for (uint32_t size = 2; size <= P; size <<= 1)
            for (uint32_t str = size >> 1; str > 0; str >>= 1) {
                for (uint32_t j = tid; j < P; j += MT) {
                    uint32_t o = j ^ str;
                    if (o > j) {
                        u64 x = S.win[j], y = S.win[o];
                        bool desc = (j & size) == 0;
                        if (desc ? (x < y) : (x > y)) { S.win[j] = y; S.win[o] = x; }
                    }
                }
                __syncthreads();
            }
        for (uint32_t j = tid; j < A.k; j += MT) {
            u64 o = (u64)b * A.k + j;
            if (j < nwin) {
                u64 key = S.win[j];
                uint32_t id = ~(uint32_t)key;
                uint32_t hi = (uint32_t)(key >> 32);
                A.out_ids[o] = id;
                if (A.dtype == LINR_I8) {
                    int best = INT_MIN;
                    const int8_t* x = (const int8_t*)A.emb + (u64)id * A.row_bytes;
                    for (uint32_t e = 0; e < A.m; ++e) {
                        int r = dot_i8_row((const int8_t*)A.Q + ((u64)b * A.m + e) * A.row_bytes, x, A.d);
                        best = r > best ? r : best;
                    }
                    float qs = A.q_scale ? A.q_scale[b] : 1.0f;
                    float rank = (A.vk == LINR_VK_I8_SCALED) ? (float)best * A.row_scale[id] : (float)best;
                    A.out_scores[o] = rank * qs;
                    if (A.out_raw) A.out_raw[o] = best;
                } else {
                    A.out_scores[o] = unord_f32(hi);
                }
            } else {
                A.out_ids[o] = LINR_NO_ID;
                A.out_scores[o] = -INFINITY;
                if (A.out_raw && A.dtype == LINR_I8) A.out_raw[o] = INT_MIN;
            }
        }
        if (tid == 0) A.out_counts[b] = nwin;
    }
    // 4. leave the per-slot segments empty for the next sweep (they were only used if a wave spilled)
    if (spilled) {
        __syncthreads();
        for (uint32_t s = tid; s < ns; s += MT) cnt[s] = 0u;
    }
}

// ---------------------------------------------------------------------------
// host launchers
// ---------------------------------------------------------------------------
hipError_t linr_launch_init(unsigned long long* tau, uint32_t* ccnt, uint32_t* gcnt, uint32_t* fvalid, uint32_t* cnt,
                            uint64_t n_cnt, uint32_t B, hipStream_t s)
{
    uint64_t want = (n_cnt + 255) / 256;
    uint32_t grid = (uint32_t)(want < 1 ? 1 : (want > 2048 ? 2048 : want));
    hipLaunchKernelGGL(init_kernel, dim3(grid), dim3(256), 0, s, (u64*)tau, ccnt, gcnt, fvalid, cnt, (u64)n_cnt, B);
    return hipGetLastError();
}

hipError_t linr_launch_merge(const linr_merge_args& a, hipStream_t s)
{
    if (a.nslots > LINR_MAX_SLOTS || a.k > LINR_MAX_K) return hipErrorInvalidValue;
    hipLaunchKernelGGL(merge_kernel, dim3(a.B), dim3(MT), 0, s, a);
    return hipGetLastError();
}

// One dispatcher for three questions about a scan kernel variant: does it exist, how many
// workgroups of it fit a compute unit, launch it.
enum { ACT_EXISTS = 0, ACT_OCCUPANCY = 1, ACT_LAUNCH = 2 };
struct ScanAct {
    int what;
    uint32_t grid;
    uint32_t dyn;
    hipStream_t s;
    const linr_scan_args* a;
    int blocks_per_cu;       // out (ACT_OCCUPANCY)
};

template <typename K>
static hipError_t scan_act(K kern, ScanAct& act)
{
    if (act.what == ACT_EXISTS) return hipSuccess;
    if (act.dyn > 0) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)act.dyn);
        if (e != hipSuccess) return e;
    }
    if (act.what == ACT_OCCUPANCY) {
        int nb = 0;
        hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kern, 64 * WPB, act.dyn);
        act.blocks_per_cu = nb;
        return e;
    }
    hipLaunchKernelGGL(kern, dim3(act.grid), dim3(64 * WPB), act.dyn, act.s, *act.a);
    return hipGetLastError();
}

#define SCAN_CASE(DT, VK, KS_, M_, QG_)                                                           \
    if (dtype == DT && vk == VK && ks == KS_ && m == M_ && qg == QG_) {                           \
        if (QG_ <= 2 && ts) return scan_act(scan_kernel<DT, VK, KS_, M_, QG_, (QG_ <= 2)>, act);  \
        return scan_act(scan_kernel<DT, VK, KS_, M_, QG_, false>, act);                           \
    }

static hipError_t scan_dispatch(int dtype, int vk, uint32_t ks, uint32_t m, uint32_t qg, bool ts, ScanAct& act)
{
    // int8 d<=64 (one K-step), scaled and raw
    SCAN_CASE(LINR_I8, LINR_VK_I8_SCALED, 1, 1, 1)  SCAN_CASE(LINR_I8, LINR_VK_I8_SCALED, 1, 1, 2)
    SCAN_CASE(LINR_I8, LINR_VK_I8_SCALED, 1, 1, 4)  SCAN_CASE(LINR_I8, LINR_VK_I8_SCALED, 1, 1, 8)
    SCAN_CASE(LINR_I8, LINR_VK_I8_SCALED, 1, 1, 16)
    SCAN_CASE(LINR_I8, LINR_VK_I8_RAW, 1, 1, 1)     SCAN_CASE(LINR_I8, LINR_VK_I8_RAW, 1, 1, 2)
    SCAN_CASE(LINR_I8, LINR_VK_I8_RAW, 1, 1, 4)     SCAN_CASE(LINR_I8, LINR_VK_I8_RAW, 1, 1, 8)
    SCAN_CASE(LINR_I8, LINR_VK_I8_RAW, 1, 1, 16)
    // bf16 d<=128 (cfg 2) and d<=64 with m = 8 (cfg 4) / m = 1
    SCAN_CASE(LINR_BF16, LINR_VK_FLOAT, 4, 1, 1)    SCAN_CASE(LINR_BF16, LINR_VK_FLOAT, 4, 1, 2)
    SCAN_CASE(LINR_BF16, LINR_VK_FLOAT, 4, 1, 4)    SCAN_CASE(LINR_BF16, LINR_VK_FLOAT, 4, 1, 8)
    SCAN_CASE(LINR_BF16, LINR_VK_FLOAT, 2, 8, 1)    SCAN_CASE(LINR_BF16, LINR_VK_FLOAT, 2, 8, 2)
    SCAN_CASE(LINR_BF16, LINR_VK_FLOAT, 2, 1, 1)    SCAN_CASE(LINR_BF16, LINR_VK_FLOAT, 2, 1, 4)
    SCAN_CASE(LINR_BF16, LINR_VK_FLOAT, 2, 1, 16)
    // fp32 d<=64 (cfg 1)
    SCAN_CASE(LINR_F32, LINR_VK_FLOAT, 4, 1, 1)     SCAN_CASE(LINR_F32, LINR_VK_FLOAT, 4, 1, 2)
    SCAN_CASE(LINR_F32, LINR_VK_FLOAT, 4, 1, 4)     SCAN_CASE(LINR_F32, LINR_VK_FLOAT, 4, 1, 8)
    return hipErrorInvalidDeviceFunction;
}

#define COOP_CASE(DT, VK, KS_, M_, QG_)                                                           \
    if (dtype == DT && vk == VK && ks == KS_ && m == M_ && qg == QG_)                             \
        return scan_act(scan_kernel_coop<DT, VK, KS_, M_, QG_>, act);

static hipError_t coop_dispatch(int dtype, int vk, uint32_t ks, uint32_t m, uint32_t qg, ScanAct& act)
{
    COOP_CASE(LINR_I8, LINR_VK_I8_SCALED, 1, 1, 1) COOP_CASE(LINR_I8, LINR_VK_I8_SCALED, 1, 1, 2)
    COOP_CASE(LINR_I8, LINR_VK_I8_SCALED, 1, 1, 4)
    COOP_CASE(LINR_I8, LINR_VK_I8_RAW, 1, 1, 1)    COOP_CASE(LINR_I8, LINR_VK_I8_RAW, 1, 1, 2)
    COOP_CASE(LINR_I8, LINR_VK_I8_RAW, 1, 1, 4)
    COOP_CASE(LINR_BF16, LINR_VK_FLOAT, 4, 1, 1)   COOP_CASE(LINR_BF16, LINR_VK_FLOAT, 4, 1, 2)
    COOP_CASE(LINR_BF16, LINR_VK_FLOAT, 4, 1, 4)
    COOP_CASE(LINR_BF16, LINR_VK_FLOAT, 2, 1, 1)   COOP_CASE(LINR_BF16, LINR_VK_FLOAT, 2, 1, 2)
    COOP_CASE(LINR_BF16, LINR_VK_FLOAT, 2, 1, 4)
    COOP_CASE(LINR_BF16, LINR_VK_FLOAT, 2, 8, 1)   COOP_CASE(LINR_BF16, LINR_VK_FLOAT, 2, 8, 2)
    COOP_CASE(LINR_F32, LINR_VK_FLOAT, 4, 1, 1)    COOP_CASE(LINR_F32, LINR_VK_FLOAT, 4, 1, 2)
    COOP_CASE(LINR_F32, LINR_VK_FLOAT, 4, 1, 4)
    return hipErrorInvalidDeviceFunction;
}

#define LDS_CASE(DT, VK, KS_)                                                                      \
    if (dtype == DT && vk == VK && ks == KS_) return scan_act(scan_kernel_lds<DT, VK, KS_>, act);

static hipError_t lds_dispatch(int dtype, int vk, uint32_t ks, ScanAct& act)
{
    LDS_CASE(LINR_I8, LINR_VK_I8_SCALED, 1) LDS_CASE(LINR_I8, LINR_VK_I8_SCALED, 2)
    LDS_CASE(LINR_I8, LINR_VK_I8_SCALED, 4) LDS_CASE(LINR_I8, LINR_VK_I8_SCALED, 8)
    LDS_CASE(LINR_I8, LINR_VK_I8_RAW, 1)    LDS_CASE(LINR_I8, LINR_VK_I8_RAW, 2)
    LDS_CASE(LINR_I8, LINR_VK_I8_RAW, 4)    LDS_CASE(LINR_I8, LINR_VK_I8_RAW, 8)
    LDS_CASE(LINR_BF16, LINR_VK_FLOAT, 1)   LDS_CASE(LINR_BF16, LINR_VK_FLOAT, 2)
    LDS_CASE(LINR_BF16, LINR_VK_FLOAT, 4)   LDS_CASE(LINR_BF16, LINR_VK_FLOAT, 8)
    LDS_CASE(LINR_F32, LINR_VK_FLOAT, 1)    LDS_CASE(LINR_F32, LINR_VK_FLOAT, 2)
    LDS_CASE(LINR_F32, LINR_VK_FLOAT, 4)    LDS_CASE(LINR_F32, LINR_VK_FLOAT, 8)
    return hipErrorInvalidDeviceFunction;
}

int linr_fast_variant_exists(int dtype, int vk, uint32_t ks, uint32_t m, uint32_t qg)
{
    ScanAct act{}; act.what = ACT_EXISTS;
    return scan_dispatch(dtype, vk, ks, m, qg, false, act) == hipSuccess;
}

int linr_coop_variant_exists(int dtype, int vk, uint32_t ks, uint32_t m, uint32_t qg)
{
    ScanAct act{}; act.what = ACT_EXISTS;
    return coop_dispatch(dtype, vk, ks, m, qg, act) == hipSuccess;
}

uint32_t linr_lds_scan_dynamic_bytes(uint32_t B, uint32_t m, uint32_t ks)
{
    uint32_t nsg = (B + 15) / 16;
    return nsg * m * ks * 1024u + nsg * 16u * 4u * (7u + WPB);
}

static hipError_t plan_dispatch(const linr_plan& p, int dtype, uint32_t B, uint32_t m, bool ts, ScanAct& act)
{
    if (p.generic) {
        act.dyn = linr_lds_scan_dynamic_bytes(B, m, p.ks);
        return lds_dispatch(dtype, p.vk, p.ks, act);
    }
    act.dyn = 0;
    if (p.coop) return coop_dispatch(dtype, p.vk, p.ks, m, p.qg, act);
    return scan_dispatch(dtype, p.vk, p.ks, m, p.qg, ts, act);
}

// workgroups of the planned scan kernel that are resident per compute unit (0 on error)
int linr_scan_blocks_per_cu(const linr_plan& p, int dtype, uint32_t B, uint32_t m, int has_ts)
{
    ScanAct act{}; act.what = ACT_OCCUPANCY;
    if (plan_dispatch(p, dtype, B, m, has_ts != 0, act) != hipSuccess) return 0;
    return act.blocks_per_cu;
}

hipError_t linr_launch_scan(const linr_plan& p, int dtype, const linr_scan_args& a, hipStream_t s)
{
    ScanAct act{}; act.what = ACT_LAUNCH; act.grid = p.grid; act.s = s; act.a = &a;
    return plan_dispatch(p, dtype, a.B, a.m, a.ts != nullptr, act);
}
