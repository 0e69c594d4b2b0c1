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
__device__ __forceinline__ bool wave_any(bool p) { return __ballot(p) != 0ull; }

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
template <int VK, int KS>
struct ChunkRegs {
    v4i ra[8];
    v4u rsc, rmk, rts;
};

// Issue the loads of level chunk `lc` (8 KB of rows + side columns) into registers.
template <int VK, int KS>
__device__ __forceinline__ void issue_chunk(ChunkRegs<VK, KS>& R, const linr_scan_args& A, u64 lc, int lane, bool has_ts)
{
    constexpr int TPC = 8 / KS;
    constexpr int CH = 16 * TPC;
    const int row = lane & 15, g4 = lane >> 4;
    const char* embp = (const char*)A.emb;
    const uint32_t rb = A.row_bytes;
    const u64 item0 = lc * A.stride * CH;
    if (item0 + CH <= A.n) {
#pragma unroll
        for (int t = 0; t < TPC; ++t)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                uint32_t off = ks * 64 + g4 * 16;
                v4i z = {0, 0, 0, 0};
                if (off < rb) z = __builtin_nontemporal_load((const v4i*)(embp + (item0 + t * 16 + row) * rb + off));
                R.ra[t * KS + ks] = z;
            }
        if (lane < CH / 4) {
            if (VK == LINR_VK_I8_SCALED) R.rsc = __builtin_nontemporal_load((const v4u*)(A.row_scale + item0 + 4 * lane));
            R.rmk = __builtin_nontemporal_load((const v4u*)(A.mask + item0 + 4 * lane));
            if (has_ts) R.rts = __builtin_nontemporal_load((const v4u*)(A.ts + item0 + 4 * lane));
        }
    } else {                                     // ragged last chunk: rows past the end read as zero
#pragma unroll
        for (int t = 0; t < TPC; ++t)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                uint32_t off = ks * 64 + g4 * 16;
                u64 it = item0 + t * 16 + row;
                v4i z = {0, 0, 0, 0};
                if (off < rb && it < A.n) z = *(const v4i*)(embp + it * rb + off);
                R.ra[t * KS + ks] = z;
            }
        if (lane < CH / 4) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                u64 it = item0 + 4 * lane + r;
                bool in = it < A.n;
                R.rsc[r] = (VK == LINR_VK_I8_SCALED && in) ? __float_as_uint(A.row_scale[it]) : 0u;
                R.rmk[r] = in ? A.mask[it] : 0u;
                R.rts[r] = (has_ts && in) ? A.ts[it] : 0u;
            }
        }
    }
}

// registers -> this wave's LDS area; returns 0.999 / max(row scale of the chunk) for the scaled int8 path
template <int VK, int KS>
__device__ __forceinline__ float stage_chunk(const ChunkRegs<VK, KS>& R, WaveLds& L, int lane, bool has_ts)
{
    constexpr int CH = 16 * (8 / KS);
    float rinv = 0.0f;
    if constexpr (VK == LINR_VK_I8_SCALED) {
        float smax = 0.0f;
        if (lane < CH / 4)
            smax = fmaxf(fmaxf(__uint_as_float(R.rsc[0]), __uint_as_float(R.rsc[1])),
                         fmaxf(__uint_as_float(R.rsc[2]), __uint_as_float(R.rsc[3])));
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) smax = fmaxf(smax, __shfl_xor(smax, o));
        rinv = 0.999f / smax;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) L.a[j][lane] = R.ra[j];
    if (lane < CH / 4) {
        if (VK == LINR_VK_I8_SCALED) *(v4u*)&L.sc[4 * lane] = R.rsc;
        *(v4u*)&L.mk[4 * lane] = R.rmk;
        if (has_ts) *(v4u*)&L.ts[4 * lane] = R.rts;
    }
    wave_sync();
    return rinv;
}

// conservative integer form of "raw * row_scale >= thr" for a whole chunk (thr > 0 only)
__device__ __forceinline__ int int_bound(float thr, float rinv)
{
    float x = thr * rinv;
    return (thr > 0.0f) ? ((x >= 2.0e9f) ? INT_MAX : (int)x) : INT_MIN;
}

// Stages A-C for the four items x one query a lane holds after the matrix product.
//   A: cheap test on the maximum of the four accumulators (exact for float / raw int,
//      conservative through `tint` for scaled int8);  B: exact ranking values against
//      the query's bound;  C: attribute predicate of the survivors, key append.
template <int VK, int CH, typename acc_t>
__device__ __forceinline__ void tile_epilogue(const acc_t& acc, float thr_f, int thr_int, uint32_t qi, int ib, u64 item0,
                                              const WaveLds& L, const linr_scan_args& A, uint32_t slot, bool has_ts,
                                              bool& need_compact)
{
    bool hot;
    if constexpr (VK == LINR_VK_FLOAT) {
        float mx = fmaxf(fmaxf(acc[0], acc[1]), fmaxf(acc[2], acc[3]));
        hot = mx >= thr_f;
    } else {
        int mx = max(max(acc[0], acc[1]), max(acc[2], acc[3]));
        hot = mx >= thr_int;
    }
    if (!wave_any(hot)) return;

    uint32_t surv = 0;
    uint32_t hi[4];
    if constexpr (VK == LINR_VK_I8_SCALED) {
        v4f sc4 = *(const v4f*)&L.sc[ib];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float s = (float)acc[r] * sc4[r];
            if (s >= thr_f) surv |= 1u << r;
            hi[r] = ord_f32(s);
        }
    } else if constexpr (VK == LINR_VK_FLOAT) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (acc[r] >= thr_f) surv |= 1u << r;
            hi[r] = ord_f32(acc[r]);
        }
    } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (acc[r] >= thr_int) surv |= 1u << r;
            hi[r] = ord_i32(acc[r]);
        }
    }
    if (qi >= A.B) surv = 0;
    if (!wave_any(surv != 0)) return;

    v4u mk4 = *(const v4u*)&L.mk[ib];
    v4u ts4 = {0, 0, 0, 0};
    if (has_ts) ts4 = *(const v4u*)&L.ts[ib];
    if (surv) {
        const linr_filter F = A.filters[qi];
        uint32_t* cnt_p = A.cnt + (u64)qi * A.nslots + slot;
        u64* seg_p = A.seg + ((u64)slot * A.B + qi) * A.cap;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            u64 item = item0 + ib + r;
            if (((surv >> r) & 1u) && item < A.n && filter_pass(F, mk4[r], has_ts, ts4[r])) {
                u64 key = ((u64)hi[r] << 32) | (u64)(uint32_t)~(uint32_t)item;
                uint32_t pos = atomicAdd(cnt_p, 1u);
                if (pos < A.cap) seg_p[pos] = key;
                if (pos + 1 + CH > A.cap) need_compact = true;
            }
        }
    }
}

// Rare: some segment of this wave (queries q_first .. q_first+nq) is nearly full.
template <int CH>
__device__ __forceinline__ void compact_full_segments(const linr_scan_args& A, uint32_t slot, uint32_t q_first, uint32_t nq,
                                                   uint32_t* hist, int lane)
{
    __threadfence();
    for (uint32_t q0 = 0; q0 < nq; q0 += 64) {
        uint32_t qi = q_first + q0 + lane;
        uint32_t c = 0;
        if (q0 + lane < nq && qi < A.B) c = aload32(A.cnt + (u64)qi * A.nslots + slot);
        u64 todo = __ballot(c + CH > A.cap);
        while (todo) {
            int src = __ffsll((long long)todo) - 1;
            todo &= todo - 1;
            uint32_t qsel = q_first + q0 + src;
            uint32_t csel = __shfl(c, src);
            if (csel > A.cap) csel = A.cap;
            wave_compact_segment(A.seg + ((u64)slot * A.B + qsel) * A.cap, A.cnt + (u64)qsel * A.nslots + slot,
                                 A.tau + qsel, csel, A.k, hist, lane);
        }
    }
}

__device__ __forceinline__ void bound_of(const u64* tau, uint32_t qi, uint32_t B, float& tf, int& ti)
{
    if (qi < B) {
        u64 t = aload64(tau + qi);
        uint32_t hi = (uint32_t)(t >> 32);
        tf = t ? unord_f32(hi) : -INFINITY;
        ti = t ? unord_i32(hi) : INT_MIN;
    } else {
        tf = INFINITY;
        ti = INT_MAX;
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
template <int DT, int VK, int KS, int M, int QG>
__global__ void __launch_bounds__(64 * WPB) scan_kernel(linr_scan_args A)
{
    constexpr int TPC = 8 / KS;
    constexpr int CH = 16 * TPC;
    using acc_t = typename AccOf<DT>::type;

    __shared__ WaveLds lds_all[WPB];
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    WaveLds& L = lds_all[wib];
    const int row = lane & 15, g4 = lane >> 4;
    const uint32_t gw = blockIdx.x * WPB + wib;
    const uint32_t split = gw % A.nsplit, slot = gw / A.nsplit;
    if (slot >= A.nslots) return;
    const uint32_t sg0 = split * QG;
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

    // ---- per-query lower bounds (lane l tracks query row l%16 of each group)
    float thr_f[QG];
    int thr_i[QG];
#pragma unroll
    for (int i = 0; i < QG; ++i) bound_of(A.tau, (sg0 + i) * 16 + row, A.B, thr_f[i], thr_i[i]);

    ChunkRegs<VK, KS> R;
    R.rsc = (v4u){0, 0, 0, 0}; R.rmk = (v4u){0, 0, 0, 0}; R.rts = (v4u){0, 0, 0, 0};
    bool need_compact = false;
    uint32_t since_refresh = 0;
    u64 lc = slot;
    if (lc < A.n_level_chunks) issue_chunk<VK, KS>(R, A, lc, lane, has_ts);

    while (lc < A.n_level_chunks) {
        const u64 item0 = lc * A.stride * CH;
        const float rinv = stage_chunk<VK, KS>(R, L, lane, has_ts);
        int tcmp[QG];
#pragma unroll
        for (int i = 0; i < QG; ++i) tcmp[i] = (VK == LINR_VK_I8_SCALED) ? int_bound(thr_f[i], rinv) : thr_i[i];

        const u64 nlc = lc + A.nslots;
        if (nlc < A.n_level_chunks) issue_chunk<VK, KS>(R, A, nlc, lane, has_ts);     // in flight while scoring

#pragma unroll 1
        for (int t = 0; t < TPC; ++t) {
            v4i a[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) a[ks] = L.a[t * KS + ks][lane];
            const int ib = t * 16 + 4 * g4;              // first of this lane's four items in the chunk
#pragma unroll
            for (int i = 0; i < QG; ++i) {
                acc_t acc;
#pragma unroll
                for (int e = 0; e < M; ++e) {
                    acc_t tmp = {0, 0, 0, 0};
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) tmp = mfma_kstep<DT>(a[ks], q[i][e][ks], tmp);
                    if (e == 0) acc = tmp;
                    else {
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[r] = acc[r] > tmp[r] ? acc[r] : tmp[r];
                    }
                }
                tile_epilogue<VK, CH>(acc, thr_f[i], tcmp[i], (sg0 + i) * 16 + row, ib, item0, L, A, slot, has_ts, need_compact);
            }
        }
        wave_sync();

        if (wave_any(need_compact)) {
            compact_full_segments<CH>(A, slot, sg0 * 16, QG * 16, (uint32_t*)&L.a[0][0], lane);
            need_compact = false;
            since_refresh = 16;
        }
        if (++since_refresh >= 16) {
#pragma unroll
            for (int i = 0; i < QG; ++i) bound_of(A.tau, (sg0 + i) * 16 + row, A.B, thr_f[i], thr_i[i]);
            since_refresh = 0;
        }
        lc = nlc;
    }
}

// ---------------------------------------------------------------------------
// scan kernel, query fragments and bounds streamed from LDS: any m, any number of
// query groups (up to the LDS budget the host plans for); one chunk-slot per wave.
// Dynamic LDS: [n_frag][64] v4i fragments, then [nsg*16] float and int bounds.
// ---------------------------------------------------------------------------
template <int DT, int VK, int KS>
__global__ void __launch_bounds__(64 * WPB) scan_kernel_lds(linr_scan_args A)
{
    constexpr int TPC = 8 / KS;
    constexpr int CH = 16 * TPC;
    using acc_t = typename AccOf<DT>::type;

    __shared__ WaveLds lds_all[WPB];
    extern __shared__ v4i dyn_lds[];
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    WaveLds& L = lds_all[wib];
    const int row = lane & 15, g4 = lane >> 4;
    const uint32_t slot = blockIdx.x * WPB + wib;
    const bool has_ts = A.ts != nullptr;
    const uint32_t rb = A.row_bytes;
    const uint32_t nsg = (A.B + 15) / 16, m = A.m;
    const uint32_t nfrag = nsg * m * KS;
    v4i* qf = dyn_lds;
    float* bf = (float*)(dyn_lds + (size_t)nfrag * 64);
    int* bi = (int*)(bf + nsg * 16);

    for (uint32_t f = wib; f < nfrag; f += WPB) {
        uint32_t ks = f % KS, e = (f / KS) % m, sg = f / (KS * m);
        uint32_t qi = sg * 16 + row, off = ks * 64 + g4 * 16;
        v4i z = {0, 0, 0, 0};
        if (qi < A.B && off < rb) z = *(const v4i*)((const char*)A.Q + ((u64)qi * m + e) * rb + off);
        qf[(size_t)f * 64 + lane] = z;
    }
    for (uint32_t qi = threadIdx.x; qi < nsg * 16; qi += 64 * WPB) bound_of(A.tau, qi, A.B, bf[qi], bi[qi]);
    __syncthreads();
    if (slot >= A.nslots) return;

    ChunkRegs<VK, KS> R;
    R.rsc = (v4u){0, 0, 0, 0}; R.rmk = (v4u){0, 0, 0, 0}; R.rts = (v4u){0, 0, 0, 0};
    bool need_compact = false;
    u64 lc = slot;
    if (lc < A.n_level_chunks) issue_chunk<VK, KS>(R, A, lc, lane, has_ts);

    while (lc < A.n_level_chunks) {
        const u64 item0 = lc * A.stride * CH;
        const float rinv = stage_chunk<VK, KS>(R, L, lane, has_ts);
        const u64 nlc = lc + A.nslots;
        if (nlc < A.n_level_chunks) issue_chunk<VK, KS>(R, A, nlc, lane, has_ts);

#pragma unroll 1
        for (int t = 0; t < TPC; ++t) {
            v4i a[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) a[ks] = L.a[t * KS + ks][lane];
            const int ib = t * 16 + 4 * g4;
#pragma unroll 1
            for (uint32_t sg = 0; sg < nsg; ++sg) {
                acc_t acc;
#pragma unroll 1
                for (uint32_t e = 0; e < m; ++e) {
                    acc_t tmp = {0, 0, 0, 0};
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
                const float tf = bf[qi];
                const int tc = (VK == LINR_VK_I8_SCALED) ? int_bound(tf, rinv) : bi[qi];
                tile_epilogue<VK, CH>(acc, tf, tc, qi, ib, item0, L, A, slot, has_ts, need_compact);
            }
        }
        wave_sync();

        if (wave_any(need_compact)) {
            compact_full_segments<CH>(A, slot, 0, nsg * 16, (uint32_t*)&L.a[0][0], lane);
            need_compact = false;
            // publish the raised bounds to the workgroup (monotone, so a racing reader is only conservative)
            for (uint32_t qi = lane; qi < nsg * 16; qi += 64) bound_of(A.tau, qi, A.B, bf[qi], bi[qi]);
            wave_sync();
        }
        lc = nlc;
    }
}

// ---------------------------------------------------------------------------
// init: no bound yet, all segments empty
// ---------------------------------------------------------------------------
__global__ void init_kernel(u64* tau, uint32_t* cnt, u64 n_cnt, uint32_t B)
{
    u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    u64 stride = (u64)gridDim.x * blockDim.x;
    for (u64 j = i; j < n_cnt; j += stride) cnt[j] = 0;
    for (u64 j = i; j < B; j += stride) tau[j] = 0;
}

// ---------------------------------------------------------------------------
// merge kernel: one workgroup of 1024 lanes per query
// ---------------------------------------------------------------------------
#define MT 1024
struct MergeLds {
    uint32_t pre[LINR_MAX_SLOTS + 1];     // exclusive prefix of segment counts
    uint32_t part[MT];
    uint32_t hist[256];
    u64 win[LINR_MAX_K];
    uint32_t nwin, bsel, above, done;
};

__device__ __forceinline__ u64 merge_fetch(const linr_merge_args& A, const MergeLds& S, uint32_t b, uint32_t f)
{
    // segment s with pre[s] <= f < pre[s+1]
    uint32_t lo = 0, hi = A.nslots;
    while (hi - lo > 1) {
        uint32_t mid = (lo + hi) >> 1;
        if (S.pre[mid] <= f) lo = mid; else hi = mid;
    }
    return A.seg[((u64)lo * A.B + b) * A.cap + (f - S.pre[lo])];
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

    // 1. segment counts -> exclusive prefix
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
        if (s < ns) { S.pre[s] = run; uint32_t c = cnt[s]; run += c < A.cap ? c : A.cap; }
    }
    if (tid == MT - 1) S.pre[ns] = S.part[MT - 1];
    __syncthreads();
    const uint32_t Mtot = S.pre[ns];

    // 2. k-th largest key (all keys distinct).  Once the remaining bucket is taken whole the
    //    low bits of the bound may stay zero: the selected set is already fixed.  A bound that
    //    seeds the next sweep is resolved down to the full score word first.
    u64 kth = 0;
    if (Mtot >= A.k) {
        u64 prefix = 0;
        uint32_t need = A.k;
        for (int shift = 56; shift >= 0; shift -= 8) {
            if (tid < 256) S.hist[tid] = 0;
            __syncthreads();
            for (uint32_t f0 = tid; f0 < Mtot; f0 += 4 * MT) {
                u64 key[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    uint32_t f = f0 + u * MT;
                    key[u] = f < Mtot ? merge_fetch(A, S, b, f) : 0ull;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    uint32_t f = f0 + u * MT;
                    bool match = f < Mtot && ((shift == 56) || ((key[u] >> (shift + 8)) == (prefix >> (shift + 8))));
                    if (match) atomicAdd(&S.hist[(uint32_t)(key[u] >> shift) & 255u], 1u);
                }
            }
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

    if (!A.final_level) {
        if (tid == 0 && Mtot >= A.k) {
            u64 cur = A.tau[b];
            if (kth > cur) A.tau[b] = kth;
        }
    } else {
        // 3. gather the winners, sort them, write the outputs
        if (tid == 0) S.nwin = 0;
        __syncthreads();
        for (uint32_t f = tid; f < Mtot; f += MT) {
            u64 key = merge_fetch(A, S, b, f);
            if (key >= kth) {
                uint32_t p = atomicAdd(&S.nwin, 1u);
                if (p < LINR_MAX_K) S.win[p] = key;
            }
        }
        __syncthreads();
        uint32_t nwin = S.nwin < A.k ? S.nwin : A.k;
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
    __syncthreads();
    // 4. leave the segments empty for the next sweep
    for (uint32_t s = tid; s < ns; s += MT) cnt[s] = 0;
}

// ---------------------------------------------------------------------------
// host launchers
// ---------------------------------------------------------------------------
hipError_t linr_launch_init(unsigned long long* tau, uint32_t* cnt, uint64_t n_cnt, uint32_t B, hipStream_t s)
{
    uint64_t want = (n_cnt + 255) / 256;
    uint32_t grid = (uint32_t)(want < 1 ? 1 : (want > 2048 ? 2048 : want));
    hipLaunchKernelGGL(init_kernel, dim3(grid), dim3(256), 0, s, (u64*)tau, cnt, (u64)n_cnt, B);
    return hipGetLastError();
}

hipError_t linr_launch_merge(const linr_merge_args& a, hipStream_t s)
{
    if (a.nslots > LINR_MAX_SLOTS || a.k > LINR_MAX_K) return hipErrorInvalidValue;
    hipLaunchKernelGGL(merge_kernel, dim3(a.B), dim3(MT), 0, s, a);
    return hipGetLastError();
}

#define SCAN_CASE(DT, VK, KS_, M_, QG_)                                                           \
    if (dtype == DT && p.vk == VK && p.ks == KS_ && a.m == M_ && p.qg == QG_) {                   \
        if (!launch) return hipSuccess;                                                           \
        hipLaunchKernelGGL((scan_kernel<DT, VK, KS_, M_, QG_>), dim3(p.grid), dim3(64 * WPB), 0, s, a); \
        return hipGetLastError();                                                                 \
    }

static hipError_t scan_dispatch(const linr_plan& p, int dtype, const linr_scan_args& a, hipStream_t s, bool launch)
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

int linr_fast_variant_exists(int dtype, int vk, uint32_t ks, uint32_t m, uint32_t qg)
{
    linr_plan p{}; p.vk = vk; p.ks = ks; p.qg = qg;
    linr_scan_args a{}; a.m = m;
    return scan_dispatch(p, dtype, a, nullptr, false) == hipSuccess;
}

uint32_t linr_lds_scan_dynamic_bytes(uint32_t B, uint32_t m, uint32_t ks)
{
    uint32_t nsg = (B + 15) / 16;
    return nsg * m * ks * 1024u + nsg * 16u * 8u;
}

#define LDS_CASE(DT, VK, KS_)                                                                      \
    if (dtype == DT && p.vk == VK && p.ks == KS_) {                                                \
        auto kern = scan_kernel_lds<DT, VK, KS_>;                                                  \
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn); \
        if (e != hipSuccess) return e;                                                             \
        hipLaunchKernelGGL(kern, dim3(p.grid), dim3(64 * WPB), dyn, s, a);                         \
        return hipGetLastError();                                                                  \
    }

static hipError_t lds_dispatch(const linr_plan& p, int dtype, const linr_scan_args& a, hipStream_t s)
{
    const uint32_t dyn = linr_lds_scan_dynamic_bytes(a.B, a.m, p.ks);
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

hipError_t linr_launch_scan(const linr_plan& p, int dtype, const linr_scan_args& a, hipStream_t s)
{
    if (p.generic) return lds_dispatch(p, dtype, a, s);
    return scan_dispatch(p, dtype, a, s, true);
}
