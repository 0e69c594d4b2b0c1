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
#include "linr_device.h"
#include <mutex>


#include "linr_scan_common.h"

// ---------------------------------------------------------------------------
// scan kernel, queries register resident
//   DT element type, VK ranking-value kind, KS 64-byte K-steps per row,
//   M embeddings per query (max-aggregated), QG 16-query groups per wave.
// Work split: wave `gw` belongs to chunk-slot gw / nsplit and owns query groups
// [split*QG, split*QG+QG); slot s visits level chunks s, s+nslots, ...  No block
// barrier is used, so waves are fully independent.
// ---------------------------------------------------------------------------

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
        // an empty window matches nothing -- where there is a timestamp column (without one, windows are not evaluated)
        if (A.ts != nullptr && W.tsmax[i * 16 + row] < W.tsmin[i * 16 + row]) { f_all[i] = 0xFFFFFFFFu; f_none[i] = 0u; }
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
                                                      q_first + i * 16 + row, ib, item0, [&] { return *(const v4f*)&L.sc[ib]; },
                                                      [&] { return *(const v4u*)&L.ts[ib]; }, A, slot, has_ts, need_compact);
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
                                                          q_first + i * 16 + row, ib, item0, [&] { return *(const v4f*)&C.sc[ib]; },
                                                          [&] { return *(const v4u*)&C.ts[ib]; }, A, slot, has_ts, need_compact);
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
// scan kernel for large int8 batches (m = 1): 32-item x 32-query tiles, K = 32 per step
// (v_mfma_i32_32x32x32_i8).  Same workgroup-cooperative staging as above; wave w owns QW
// groups of 32 queries, so a workgroup answers 128 * QW queries per pass; a chunk is 256 / KS items
// (16 KB of rows), twice that of the other kernels, to halve the per-chunk bookkeeping.  After the
// product a lane holds 16 items of ONE query, so the first test is a 16-way integer
// maximum against one bound per query: 9 vector instructions per 32x32 block instead of
// 16 with 16x16 tiles -- the vector ALU, not the matrix pipe, limits this loop.
//
// Scaled int8 (ranking value raw * scale_i): an item matters iff raw >= thr / scale_i, a
// bound that differs from item to item.  With r_i = 1 / scale_i, rmin = min r_i and
// E_i = floor(127 (r_i - rmin) / (rmax - rmin)) in [0, 127],
//     thr * r_i >= thr * rmin + E_i * G,      G = floor(thr * (rmax - rmin) / 127),
// so "raw - E_i * G >= floor(thr * rmin)" never misses such an item, and its right side
// depends on the query only.  The subtraction is one more K step of the same matrix
// instruction: the item side carries E_i in all 32 slots, the query side the digits of -G
// (slot s holds -clamp(G - 127 s, 0, 127)).  One extra product per block buys a test that
// is tight to under 1 % of the bound whatever the spread of the row scales inside a tile.
// A (tile, group) that fires is narrowed to runs of 4 consecutive items per lane, the raw
// values are restored (+ E_i * G) and handed to the same survivor path as in the 16x16
// kernels.  Two to four waves per SIMD overlap one wave's tests with another's products.
//   lane l of a product: query column l%32, item rows 8*(r/4) + 4*(l/32) + r%4, r<16.
// ---------------------------------------------------------------------------
typedef int v16i __attribute__((ext_vector_type(16)));
#define LINR_WIDE_GMAX (32 * 127)

__device__ __forceinline__ int max16(const v16i& a)
{
    int m = max(max(a[0], a[1]), a[2]);
    m = max(max(m, a[3]), a[4]);
    m = max(max(m, a[5]), a[6]);
    m = max(max(m, a[7]), a[8]);
    m = max(max(m, a[9]), a[10]);
    m = max(max(m, a[11]), a[12]);
    m = max(max(m, a[13]), a[14]);
    return max(m, a[15]);
}

// floor(x) clamped to the int range (x may be +-inf)
__device__ __forceinline__ int floor_to_int(float x)
{
    return (int)fminf(fmaxf(floorf(x), -2147483520.0f), 2147483520.0f);
}

// reciprocal of a row scale, rounded down by more than the error of the hardware reciprocal
__device__ __forceinline__ float rcp_down(float scale)
{
    return __builtin_amdgcn_rcpf(scale) * 0.999999f;
}

// One K = 32-byte step of a 32x32 product block.  The accumulators are kept as 32-bit patterns for both element
// types: float products are only ever compared, and for a positive bound "some value >= bound" is the same
// statement about the bit patterns read as signed integers (negative floats are negative integers).
typedef float v16f __attribute__((ext_vector_type(16)));
template <int DT>
__device__ __forceinline__ v16i wide_mfma(const v4i& a, const v4i& b, const v16i& c)
{
    if constexpr (DT == LINR_I8) {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
    } else {
        const v16f r = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b),
                                                                __builtin_bit_cast(v16f, c), 0, 0, 0);
        return __builtin_bit_cast(v16i, r);
    }
}
// bound of the bit patterns for a float threshold (no usable bound unless it is positive)
__device__ __forceinline__ int float_bound_bits(float thr)
{
    return thr > 0.0f ? __float_as_int(thr) : INT_MIN;
}

// One stage of the chunk ring in LDS, filled by direct global -> LDS loads (no registers in between, so
// several chunks can be in flight per workgroup).  Such a load writes the 64 lanes' data to consecutive
// LDS addresses, so block f of `a` (1 KB) holds a 16-row x 64-byte piece of the chunk as
// [16-byte column g][row], exactly as the lanes fetched it (lane: row l%16, column l/16).
struct WideStage {
    v4i a[1024];               // 16 KB of rows: a chunk of this kernel is 256 / KS items
    uint32_t mk[256];
    float sc[256];
    uint32_t ts[256];
    uint32_t ec[64];           // scaled int8: E_i, one byte per item
};

#define LINR_WIDE_DMA_PER_WAVE 8   // direct loads every wave issues per chunk (always this many)

// The stages are read with hand-placed LDS instructions: for a read the compiler can see, it waits until every
// outstanding direct load has landed (it cannot know which stage a load fills), which would empty the ring at
// every step.  Each helper issues its reads and waits for them itself; that a stage's loads have landed is
// established by the step protocol of the kernel (counted wait + workgroup barrier).
__device__ __forceinline__ uint32_t lds_addr(const void* p)
{
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}
template <int NK>
__device__ __forceinline__ void lds_read_tile(uint32_t addr_a, uint32_t addr_e, v4i (&a)[NK], uint32_t& e)
{
    static_assert(NK == 2 || NK == 4 || NK == 8, "K = 32 steps per row");
    if constexpr (NK == 2)
        asm volatile("ds_read_b128 %0, %3\n\tds_read_b128 %1, %3 offset:512\n\tds_read_u8 %2, %4\n\ts_waitcnt lgkmcnt(0)"
                     : "=&v"(a[0]), "=&v"(a[1]), "=&v"(e) : "v"(addr_a), "v"(addr_e) : "memory");
    else if constexpr (NK == 4)
        asm volatile("ds_read_b128 %0, %5\n\tds_read_b128 %1, %5 offset:512\n\tds_read_b128 %2, %5 offset:1024\n\t"
                     "ds_read_b128 %3, %5 offset:1536\n\tds_read_u8 %4, %6\n\ts_waitcnt lgkmcnt(0)"
                     : "=&v"(a[0]), "=&v"(a[1]), "=&v"(a[2]), "=&v"(a[3]), "=&v"(e) : "v"(addr_a), "v"(addr_e) : "memory");
    else
        asm volatile("ds_read_b128 %0, %9\n\tds_read_b128 %1, %9 offset:512\n\tds_read_b128 %2, %9 offset:1024\n\t"
                     "ds_read_b128 %3, %9 offset:1536\n\tds_read_b128 %4, %9 offset:2048\n\tds_read_b128 %5, %9 offset:2560\n\t"
                     "ds_read_b128 %6, %9 offset:3072\n\tds_read_b128 %7, %9 offset:3584\n\tds_read_u8 %8, %10\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=&v"(a[0]), "=&v"(a[1]), "=&v"(a[2]), "=&v"(a[3]), "=&v"(a[4]), "=&v"(a[5]), "=&v"(a[6]), "=&v"(a[7]), "=&v"(e)
                     : "v"(addr_a), "v"(addr_e) : "memory");
}
// side columns of four consecutive items (mask, scale, timestamp: 16 bytes each; codes: 4 bytes)
__device__ __forceinline__ void lds_read_side(uint32_t addr_mk, uint32_t addr_sc, uint32_t addr_ts, uint32_t addr_ec, v4u& mk4, v4f& sc4,
                                              v4u& ts4, uint32_t& e4)
{
    asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %5\n\tds_read_b128 %2, %6\n\tds_read_b32 %3, %7\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(mk4), "=&v"(sc4), "=&v"(ts4), "=&v"(e4) : "v"(addr_mk), "v"(addr_sc), "v"(addr_ts), "v"(addr_ec) : "memory");
}

// s_waitcnt immediate that waits for the vector-memory counter only (gfx9 encoding)
#define LINR_WAIT_VM(n) (((n) & 15) | (((n) >> 4) << 14) | 0x0F70)

// Byte offsets of what a lane fetches, relative to the start of a chunk's rows / side columns; they do not change
// from chunk to chunk, so a full chunk costs no per-lane address arithmetic (uniform base + 32-bit lane offset).
struct WideLaneOff {
    uint32_t emb[4];
    uint32_t side;
    uint32_t ec;
};

template <int KS>
__device__ __forceinline__ WideLaneOff wide_lane_offsets(int lane, int wib)
{
    constexpr int CH = 256 / KS;
    const int row = lane & 15, g4 = lane >> 4;
    WideLaneOff o;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int f = wib * 4 + j, t16 = f / KS, ks = f % KS;
        o.emb[j] = (uint32_t)((t16 * 16 + row) * (KS * 64) + ks * 64 + g4 * 16);
    }
    o.side = ((uint32_t)(wib * 64 + lane) % (uint32_t)CH) * 4u;
    o.ec = ((uint32_t)lane % (uint32_t)(CH / 4)) * 4u;
    return o;
}

// Every wave issues the same eight loads per chunk: four 1 KB blocks of rows, its 64 items' worth of each side
// column (repeating items when the chunk has fewer than 256) and the codes; what a short chunk or a missing
// column leaves over is loaded from a valid address anyway and never read.
template <int VK, int KS>
__device__ __forceinline__ void issue_wide(WideStage& S, const linr_scan_args& A, u64 item0, int lane, int wib, bool has_ts,
                                           const WideLaneOff& off)
{
    typedef const __attribute__((address_space(1))) void* gptr;
    typedef __attribute__((address_space(3))) void* lptr;
    constexpr int CH = 256 / KS;
    constexpr uint32_t RB = KS * 64;
    const char* p_emb[4];
    const char *p_mk, *p_ts, *p_sc, *p_ec;
    if (item0 + CH <= A.n) {                            // uniform; all chunks but possibly the last one
        const char* eb = (const char*)A.emb + item0 * RB;
#pragma unroll
        for (int j = 0; j < 4; ++j) p_emb[j] = eb + off.emb[j];
        p_mk = (const char*)A.mask + item0 * 4 + off.side;
        p_ts = (const char*)(has_ts ? A.ts : A.mask) + item0 * 4 + off.side;
        p_sc = (const char*)(VK == LINR_VK_I8_SCALED ? (const void*)A.row_scale : (const void*)A.mask) + item0 * 4 + off.side;
    } else {                                            // ragged end: items past the last one repeat it
        const u64 last = A.n - 1;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            u64 it = item0 + off.emb[j] / RB;
            it = it < last ? it : last;
            p_emb[j] = (const char*)A.emb + it * RB + off.emb[j] % RB;
        }
        u64 it = item0 + off.side / 4;
        it = it < last ? it : last;
        p_mk = (const char*)A.mask + it * 4;
        p_ts = (const char*)(has_ts ? A.ts : A.mask) + it * 4;
        p_sc = (const char*)(VK == LINR_VK_I8_SCALED ? (const void*)A.row_scale : (const void*)A.mask) + it * 4;
    }
    // CH bytes of codes = CH/4 words; the column is padded so that a whole chunk can always be read
    p_ec = VK == LINR_VK_I8_SCALED ? (const char*)A.scale_code + item0 + off.ec : p_mk;
#pragma unroll
    for (int j = 0; j < 4; ++j) __builtin_amdgcn_global_load_lds((gptr)p_emb[j], (lptr)&S.a[(wib * 4 + j) * 64], 16, 0, 0);
    __builtin_amdgcn_global_load_lds((gptr)p_mk, (lptr)&S.mk[wib * 64], 4, 0, 0);
    __builtin_amdgcn_global_load_lds((gptr)p_ts, (lptr)&S.ts[wib * 64], 4, 0, 0);
    __builtin_amdgcn_global_load_lds((gptr)p_sc, (lptr)&S.sc[wib * 64], 4, 0, 0);
    __builtin_amdgcn_global_load_lds((gptr)p_ec, (lptr)&S.ec[0], 4, 0, 0);
}

// Query side of the scale correction for the query this lane tracks (column l%32): the bound of the
// corrected value, G, and the 16 digit bytes of -G this lane supplies (slots 16 (l/32) .. +15).
__device__ __forceinline__ void wide_query_bound(float thr, float rmin, float r_per_e, int h2, int& base, int& G, v4i& digits)
{
    const float tl = lowered_pos(thr);                                  // -inf: no usable bound yet
    base = floor_to_int(tl * rmin);
    int g = floor_to_int(fmaxf(tl, 0.0f) * r_per_e);                    // +inf (unused query slot) clamps below
    g = g < 0 ? 0 : (g > LINR_WIDE_GMAX ? LINR_WIDE_GMAX : g);
    G = g;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        uint32_t word = 0;
#pragma unroll
        for (int byte = 0; byte < 4; ++byte) {
            const int slot = 16 * h2 + 4 * w + byte;
            int dgt = g - 127 * slot;
            dgt = dgt < 0 ? 0 : (dgt > 127 ? 127 : dgt);
            word |= ((uint32_t)(-dgt) & 0xFFu) << (8 * byte);
        }
        digits[w] = (int)word;
    }
}

template <int DT, int VK, int KS, int QW>
__global__ void __launch_bounds__(64 * WPB, 2) scan_kernel_wide(linr_scan_args A)
{
    constexpr int CH = 256 / KS;
    constexpr int TW = CH / 32;
    constexpr int NK = 2 * KS;
    constexpr int NQ = QW * 32;
    constexpr int NST = 3;                               // ring stages: NST - 1 chunks (16 KB each) are in flight per workgroup
    constexpr bool SCALED = (VK == LINR_VK_I8_SCALED);
    constexpr bool FLOATS = (VK == LINR_VK_FLOAT);
    static_assert(KS == 1 || KS == 2 || KS == 4, "rows of 64, 128 or 256 bytes");
    static_assert((DT == LINR_I8 && !FLOATS) || (DT == LINR_BF16 && FLOATS), "int8 and bf16 only");

    constexpr int QCAP = LINR_WIDE_QCAP;
    constexpr int SCRATCH_WORDS = 2 * QCAP + QCAP / 4 + 4;   // keys, query numbers, count (last word)
    static_assert(SCRATCH_WORDS - 4 >= 2 * NQ + 1 && SCRATCH_WORDS - 4 >= 256, "scratch is shared with compaction and the final flush");

    __shared__ WideStage ring[NST];
    __shared__ WaveQ<QW * 2> wq_all[WPB];
    __shared__ __attribute__((aligned(8))) uint32_t scratch_all[WPB][SCRATCH_WORDS];
    const int lane = threadIdx.x & 63, wib = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    u64* const qkey = (u64*)&scratch_all[wib][0];
    uint8_t* const qql = (uint8_t*)&scratch_all[wib][2 * QCAP];
    uint32_t* const qcount = &scratch_all[wib][SCRATCH_WORDS - 1];
    WaveQ<QW * 2>& W = wq_all[wib];
    const QSide qs = {W.cnt, W.thr_f, W.thr_i, W.fall, W.fnone, W.tsmin, W.tsmax, W.fflag};
    const int col = lane & 31, h2 = lane >> 5;
    const uint32_t slot = blockIdx.x;
    if (slot >= A.nslots) return;                       // uniform for the workgroup
    const uint32_t q_first = wib * NQ;
    const bool active = q_first < A.B;                  // waves past the batch still load and synchronise
    const bool has_ts = A.ts != nullptr;
    float rmin = 0.0f, r_per_e = 0.0f;                  // index-wide statistics of 1 / row scale
    if constexpr (SCALED) { rmin = A.scale_stats[0]; r_per_e = A.scale_stats[2]; }

    v4i q[QW][NK];
#pragma unroll
    for (int i = 0; i < QW; ++i) {
        const uint32_t qi = q_first + i * 32 + col;
#pragma unroll
        for (int s = 0; s < NK; ++s) {
            v4i z = {0, 0, 0, 0};
            if (qi < A.B) z = *(const v4i*)((const char*)A.Q + (u64)qi * (KS * 64) + (s * 32 + h2 * 16));
            q[i][s] = z;
        }
    }
    for (uint32_t ql = lane; ql < (uint32_t)NQ; ql += 64) {
        W.cnt[ql] = 0;
        load_query_side(qs, ql, q_first + ql, A, true);
    }
    if (lane == 0) *qcount = 0;
    wave_sync();
    int bound[QW];            // lane l tracks query column l%32 of each group
    v4i qe[QW];               // digits of -G (scaled int8)
    auto refresh_bounds = [&]() {
#pragma unroll
        for (int i = 0; i < QW; ++i) {
            if constexpr (SCALED) {
                int G;
                wide_query_bound(W.thr_f[i * 32 + col], rmin, r_per_e, h2, bound[i], G, qe[i]);
                if (h2 == 0) W.thr_i[i * 32 + col] = G;  // (thr_i is not used otherwise for this ranking kind)
            } else {
                bound[i] = FLOATS ? float_bound_bits(W.thr_f[i * 32 + col]) : W.thr_i[i * 32 + col];
                qe[i] = (v4i){0, 0, 0, 0};
            }
        }
        wave_sync();
    };
    refresh_bounds();

    // Fragment (T, s) of a stage: lane l needs bytes [32 s + 16 (l/32), +16) of item row 32 T + l%32.  That is
    // 16-byte column 2 s + l/32 of the row, which sits in block (2 T + (l%32)/16) * KS + (2 s + l/32) / 4 at
    // [column % 4][row % 16]: byte offset frag0 + 2048 KS T + 512 s.
    const uint32_t frag0 = (uint32_t)(((col >> 4) * KS * 64 + h2 * 16 + (col & 15)) * 16);

    uint32_t need_compact = 0u;
    uint32_t since_refresh = 0;
    // Candidate keys wait in the wave's LDS queue and are written out in bulk.  Loads and stores may complete out
    // of order with respect to each other, which would spoil the counting of outstanding direct loads, so every
    // path that stores to global memory ends by waiting for all of the wave's memory operations.
    auto flush_queue = [&]() {
        wave_sync();
        const uint32_t nqd = *qcount;
        for (uint32_t t = lane; t < nqd; t += 64) {
            const u64 key = qkey[t];
            const uint32_t ql = qql[t];
            const uint32_t pos = atomicAdd(&W.cnt[ql], 1u);
            if (pos < A.cap) A.seg[((u64)slot * A.B + q_first + ql) * A.cap + pos] = key;
            if (pos + 1 + QCAP > A.cap) need_compact = 1u;
        }
        wave_sync();
        if (lane == 0) *qcount = 0;
        wave_sync();
        __builtin_amdgcn_s_waitcnt(LINR_WAIT_VM(0));
    };
    const v16i zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    const WideLaneOff lane_off = wide_lane_offsets<KS>(lane, wib);
    // One walker runs NST - 1 chunks ahead of the consumer and hands it the first item of each chunk through a
    // small queue indexed by ring stage; `n_mine` chunks belong to this workgroup.
    SweepWalk ahead;
    ahead.init(slot, A);
    const uint32_t n_dense32 = (uint32_t)A.n_dense;
    const uint32_t n_mine = slot < n_dense32 ? (n_dense32 - slot + A.nslots - 1) / A.nslots : 0u;
    u64 item0_q[NST];
    u64 item0_last = 0;

    // Every wave always issues the same number of direct loads per step (past the end of the sweep it reloads
    // the last valid chunk), so "at most (NST-2) * LINR_WIDE_DMA_PER_WAVE loads outstanding" means: the chunk
    // about to be consumed has landed.
    auto issue_next = [&](int rf) {
        if (ahead.valid()) item0_last = ahead.lc() * A.stride * CH;
#pragma unroll
        for (int t = 0; t < NST; ++t)
            if (t == rf) item0_q[t] = item0_last;
        issue_wide<VK, KS>(ring[rf], A, item0_last, lane, wib, has_ts, lane_off);
        ahead.advance();
    };

    auto consume = [&](int st) {
        WideStage& C = ring[st];
        u64 item0 = item0_q[0];
#pragma unroll
        for (int t = 1; t < NST; ++t)
            if (t == st) item0 = item0_q[t];
        const uint32_t base_a = lds_addr(&C.a[0]) + frag0, base_e = lds_addr(&C.ec[0]) + col;
        const uint32_t base_mk = lds_addr(&C.mk[0]), base_sc = lds_addr(&C.sc[0]), base_ts = lds_addr(&C.ts[0]);
#pragma unroll 1
        for (int T = 0; T < TW; ++T) {
            v16i acc[QW];
            {
                v4i a[NK];
                uint32_t ecode;
                lds_read_tile<NK>(base_a + T * (2048 * KS), base_e + T * 32, a, ecode);
#pragma unroll
                for (int s = 0; s < NK; ++s)
#pragma unroll
                    for (int i = 0; i < QW; ++i)
                        acc[i] = wide_mfma<DT>(a[s], q[i][s], s == 0 ? zero16 : acc[i]);
                if constexpr (SCALED) {
                    const int rep = (int)(ecode * 0x01010101u);
                    const v4i ae = {rep, rep, rep, rep};
#pragma unroll
                    for (int i = 0; i < QW; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ae, qe[i], acc[i], 0, 0, 0);
                }
            }
            uint32_t pend = 0;                       // groups of this tile whose test fired (uniform)
#pragma unroll
            for (int i = 0; i < QW; ++i) pend |= wave_any(max16(acc[i]) >= bound[i]) ? (1u << i) : 0u;
            while (pend) {
                const int i = __ffs((int)pend) - 1;
                pend &= pend - 1;
                v16i hv = acc[0];
#pragma unroll
                for (int c = 1; c < QW; ++c)
                    if (i == c) hv = acc[c];
                const uint32_t ql = i * 32 + col;
                int bi, G = 0;
                if constexpr (SCALED) {
                    G = W.thr_i[ql];
                    bi = floor_to_int(lowered_pos(W.thr_f[ql]) * rmin);
                } else {
                    bi = FLOATS ? float_bound_bits(W.thr_f[ql]) : W.thr_i[ql];
                }
                const uint32_t fa = W.fall[ql], fn = W.fnone[ql];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int ib = T * 32 + 8 * j + 4 * h2;
                    v4i acc4 = {hv[4 * j], hv[4 * j + 1], hv[4 * j + 2], hv[4 * j + 3]};
                    const bool lane_hot = max(max(acc4[0], acc4[1]), max(acc4[2], acc4[3])) >= bi;
                    if (!wave_any(lane_hot)) continue;
                    v4u mk4, ts4;
                    v4f sc4;
                    uint32_t e4;
                    lds_read_side(base_mk + ib * 4, base_sc + ib * 4, base_ts + ib * 4, base_e - col + ib, mk4, sc4, ts4, e4);
                    if constexpr (SCALED) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc4[r] += (int)((e4 >> (8 * r)) & 0xFFu) * G;
                    }
                    if (*qcount + 256u > (uint32_t)QCAP) {             // uniform: one call appends at most 4 keys per lane
                        flush_queue();
                        if (wave_any(need_compact != 0u)) {
                            compact_full_segments<QCAP>(A, qs, slot, q_first, NQ, scratch_all[wib], lane);
                            __builtin_amdgcn_s_waitcnt(LINR_WAIT_VM(0));
                            need_compact = 0u;
                            since_refresh = 64;                       // bounds moved: reload them after this chunk
                        }
                    }
                    if constexpr (FLOATS) {
                        const v4f accf = {__int_as_float(acc4[0]), __int_as_float(acc4[1]), __int_as_float(acc4[2]),
                                          __int_as_float(acc4[3])};
                        tile_survivors<VK, false, CH, true>(accf, lane_hot, mk4, fa, fn, qs, ql, q_first + ql, ib, item0,
                                                            [&] { return sc4; }, [&] { return ts4; }, A, slot, has_ts,
                                                            need_compact, qcount, qkey, qql);
                    } else {
                        tile_survivors<VK, false, CH, true>(acc4, lane_hot, mk4, fa, fn, qs, ql, q_first + ql, ib, item0,
                                                            [&] { return sc4; }, [&] { return ts4; }, A, slot, has_ts,
                                                            need_compact, qcount, qkey, qql);
                    }
                }
            }
        }
        // (an ordinary load returns after all direct loads issued before it, so each refresh empties the ring: keep it rare)
        const bool refresh = ++since_refresh >= 64;
        if (refresh) {
            for (uint32_t ql = lane; ql < (uint32_t)NQ; ql += 64) load_query_side(qs, ql, q_first + ql, A, false);
            wave_sync();
            refresh_bounds();
            since_refresh = 0;
        }
    };

    // One step: wait until the chunk in stage `cur` has landed for every wave, refill the stage consumed one
    // step ago with the chunk NST - 1 steps ahead, then consume `cur`.
    if (n_mine) {
        // prologue: NST - 1 chunks in flight
        for (int st = 0; st < NST - 1; ++st) issue_next(st);
        int st = 0;                                      // stage that holds the chunk to consume
        // One step: wait until the chunk in stage `st` has landed for every wave, refill the stage consumed one
        // step ago with the chunk NST - 1 steps ahead, then consume `st`.
        for (uint32_t c = 0; c < n_mine; ++c) {
            __builtin_amdgcn_s_waitcnt(LINR_WAIT_VM((NST - 2) * LINR_WIDE_DMA_PER_WAVE));
            __builtin_amdgcn_s_barrier();
            issue_next(st == 0 ? NST - 1 : st - 1);
            if (active) consume(st);
            st = st + 1 == NST ? 0 : st + 1;
        }
        // nothing of this workgroup may still be on its way to LDS when its waves end
        __builtin_amdgcn_s_waitcnt(LINR_WAIT_VM(0));
    }
    if (active) {
        flush_queue();
        own_stores_done();
        flush_segments(A, qs, slot, q_first, NQ, lane, scratch_all[wib]);
    }
}

// Index-wide statistics of r = 1 / row scale for the kernel above and the per-item codes E_i.
// out[3] = 1 / (mean row scale) (0 if unusable); out[0] = min r; out[1] = 127 / span and out[2] = span / 127, both rounded down, where span =
// min(max r - min r, 2 (mean r - min r)) so that a few extreme rows do not cost the bulk its resolution
// (rows beyond the span get E = 127, a valid if loose correction).  All zero if the scales are unusable.
// Three launches: per-block partials, one block reduces them, then the codes.
__device__ __forceinline__ float block_reduce(float v, float* sh, int op)    // op 0 min, 1 max, 2 sum
{
    sh[threadIdx.x] = v;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) {
            const float x = sh[threadIdx.x], y = sh[threadIdx.x + o];
            sh[threadIdx.x] = op == 0 ? fminf(x, y) : op == 1 ? fmaxf(x, y) : x + y;
        }
        __syncthreads();
    }
    const float r = sh[0];
    __syncthreads();
    return r;
}

__global__ void __launch_bounds__(256) scale_stats_partial(const float* row_scale, u64 n, float* part)
{
    __shared__ float sh[256];
    float mn = INFINITY, mx = 0.0f, sum = 0.0f, sum_s = 0.0f;
    for (u64 i = (u64)blockIdx.x * 256 + threadIdx.x; i < n; i += (u64)gridDim.x * 256) {
        const float sc = row_scale[i];
        const float r = rcp_down(sc);
        if (r == r) { mn = fminf(mn, r); mx = fmaxf(mx, r); sum += fminf(r, 3.0e30f); }
        if (sc > 0.0f) sum_s += fminf(sc, 3.0e30f);
    }
    mn = block_reduce(mn, sh, 0); mx = block_reduce(mx, sh, 1); sum = block_reduce(sum, sh, 2); sum_s = block_reduce(sum_s, sh, 2);
    if (threadIdx.x == 0) {
        part[4 * blockIdx.x] = mn; part[4 * blockIdx.x + 1] = mx; part[4 * blockIdx.x + 2] = sum; part[4 * blockIdx.x + 3] = sum_s;
    }
}

__global__ void __launch_bounds__(256) scale_stats_final(const float* part, uint32_t nparts, u64 n, float* out)
{
    __shared__ float sh[256];
    float mn = INFINITY, mx = 0.0f, sum = 0.0f, sum_s = 0.0f;
    for (uint32_t i = threadIdx.x; i < nparts; i += 256) {
        mn = fminf(mn, part[4 * i]); mx = fmaxf(mx, part[4 * i + 1]); sum += part[4 * i + 2]; sum_s += part[4 * i + 3];
    }
    mn = block_reduce(mn, sh, 0); mx = block_reduce(mx, sh, 1); sum = block_reduce(sum, sh, 2); sum_s = block_reduce(sum_s, sh, 2);
    if (threadIdx.x == 0) {
        const float mean = sum / (float)n;
        float span = fminf(mx - mn, 2.0f * (mean - mn));
        const bool ok = mn > 0.0f && mn < 3.0e38f;
        const bool usable = ok && span > 0.0f && span < 3.0e38f;
        out[0] = ok ? mn : 0.0f;                               // 0: the bound degenerates to "everything may matter"
        out[1] = usable ? (127.0f / span) * 0.99999f : 0.0f;
        out[2] = usable ? (span / 127.0f) * 0.99999f : 0.0f;
        // reference 1 / row scale of the large-batch kernel: 1 / (mean positive scale).  The mean scale is set by the
        // rows with large scales, the ones whose scores reach the top; zero scales and outliers of 1 / scale do not move it.
        const float ref = (float)n / sum_s;
        out[3] = (sum_s > 0.0f && ref > 0.0f && ref < 3.0e38f) ? ref : 0.0f;
    }
}

__global__ void __launch_bounds__(256) scale_code_kernel(const float* row_scale, u64 n, u64 n_pad, const float* stats, uint8_t* out)
{
    const float rmin = stats[0], e_per_r = stats[1];
    for (u64 i = (u64)blockIdx.x * 256 + threadIdx.x; i < n_pad; i += (u64)gridDim.x * 256) {
        float ef = 0.0f;
        if (i < n) ef = fminf(fmaxf((rcp_down(row_scale[i]) - rmin) * e_per_r, 0.0f), 127.0f);    // NaN -> 0
        out[i] = (uint8_t)ef;
    }
}

// ---------------------------------------------------------------------------
// quantised search (LiNR Sec. 3.2): scan over 1-bit Sign-OPORP codes
//   similarity = number of equal bits = k_bits - popcount(code ^ query code).
// A wave is a chunk-slot of its own (no barrier); a lane holds 4 items of the 256-item
// chunk (their W code words, mask, timestamp) in registers and walks over the batch's
// queries, whose codes and bounds sit in LDS (uniform reads).  Per (item, query): W xor,
// 2 W bit counts, one compare; the predicate and the key append run only for the lanes
// that beat the query's bound.  The same candidate segments, bounds, sweeps and merges
// as the exact scan are used, with the match count as an integer ranking value.
// HBM-bound for a few queries (8 W + 4 bytes per item), vector-ALU-bound for many.
// ---------------------------------------------------------------------------
#define LINR_BITS_NQ 64            // queries per pass
#define LINR_BITS_CH 256           // items per chunk

template <int W>
struct BitsRegs {
    u64 x[4][W];
    uint32_t mk[4], ts[4];
};

template <int W>
__device__ __forceinline__ void issue_bits(BitsRegs<W>& R, const linr_scan_args& A, u64 lc, int lane, bool has_ts)
{
    const u64 item0 = lc * A.stride * LINR_BITS_CH;
    const u64 last = A.n - 1;
    const u64* bits = (const u64*)A.emb;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        u64 it = item0 + u * 64 + lane;
        it = it < last ? it : last;
#pragma unroll
        // (codes of several words: a lane's loads touch each 64-byte sector several times in a row; only an allocating
        // load lets the first-level cache serve the repeats)
        for (int w = 0; w < W; ++w) R.x[u][w] = W >= 2 ? bits[it * W + w] : __builtin_nontemporal_load(bits + it * W + w);
        R.mk[u] = __builtin_nontemporal_load(A.mask + it);
        R.ts[u] = has_ts ? __builtin_nontemporal_load(A.ts + it) : 0u;
    }
}

// one query as the bit-matching loop reads it: its code and the offset that turns the bound test into a sign test
template <int W>
struct __attribute__((aligned(8))) BitsQ {
    u64 code[W];
    uint32_t bias, pad;
};

// acc + number of set bits of x (one instruction; the accumulate operand carries the bound offset)
__device__ __forceinline__ uint32_t bcnt_acc(uint32_t x, uint32_t acc)
{
    uint32_t r;
    asm("v_bcnt_u32_b32 %0, %1, %2" : "=v"(r) : "v"(x), "v"(acc));
    return r;
}

template <int W>
__global__ void __launch_bounds__(64 * WPB, W <= 2 ? 4 : 2) scan_kernel_bits(linr_scan_args A)
{
    constexpr int NQ = LINR_BITS_NQ;
    __shared__ WaveQ<NQ / 16> wq_all[WPB];
    __shared__ uint32_t hist_all[WPB][256];
    __shared__ BitsQ<W> qrec_all[WPB][NQ + 2];           // per wave (the offsets follow the wave's own bounds); +2: read-ahead
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    WaveQ<NQ / 16>& Wq = wq_all[wib];
    BitsQ<W>* qrec = qrec_all[wib];
    const QSide qs = {Wq.cnt, Wq.thr_f, Wq.thr_i, Wq.fall, Wq.fnone, Wq.tsmin, Wq.tsmax, Wq.fflag};
    const uint32_t slot = blockIdx.x * WPB + wib;
    const bool has_ts = A.ts != nullptr;
    const int kb = (int)A.k_bits;                        // bits per code
    if (slot >= A.nslots) return;                        // no workgroup-wide barrier below
    for (uint32_t ql = lane; ql < (uint32_t)NQ; ql += 64) {
#pragma unroll
        for (int w = 0; w < W; ++w) qrec[ql].code[w] = ql < A.B ? ((const u64*)A.Q)[(u64)ql * W + w] : 0ull;
        Wq.cnt[ql] = 0;
        load_query_side(qs, ql, ql, A, true);
    }
    wave_sync();
    // matches >= bound  <=>  differing bits - (k_bits - bound + 1) < 0: the bit counts accumulate onto that
    // offset, so the sign of the sum is the test.  No bound yet (INT_MIN): the saturating add keeps INT_MIN,
    // and every sum stays negative.
    auto set_bias = [&]() {
        for (uint32_t ql = lane; ql < (uint32_t)NQ; ql += 64)
            qrec[ql].bias = (uint32_t)__builtin_elementwise_add_sat(Wq.thr_i[ql], -(kb + 1));
        wave_sync();
    };
    set_bias();

    // The chunk being matched and the chunks in flight live in register sets whose roles rotate (no copies: a copy
    // of a set with loads pending would wait for them).  64-bit codes keep two chunks in flight, wider codes one.
    constexpr bool DEEP = W == 1;
    uint32_t need_compact = 0u, since_refresh = 0u;
    SweepWalk walk;
    walk.init(slot, A);
    u64 lcA = walk.lc(), lcB = 0;
    bool vA = walk.valid(), vB = false;
    BitsRegs<W> S0, S1, S2;
    if (vA) issue_bits<W>(S0, A, lcA, lane, has_ts);
    if constexpr (DEEP) {
        walk.advance();
        lcB = walk.lc(); vB = walk.valid();
        if (vB) issue_bits<W>(S1, A, lcB, lane, has_ts);
    }
    auto step = [&](BitsRegs<W>& cur, BitsRegs<W>& fre) -> bool {
        if (!vA) return false;
        const u64 item0 = lcA * A.stride * LINR_BITS_CH;
        walk.advance();
        const u64 lcC = walk.lc();
        const bool vC = walk.valid();
        if (vC) issue_bits<W>(fre, A, lcC, lane, has_ts);

        bool live[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) live[u] = item0 + u * 64 + lane < A.n;
        // survivors of one query: predicate, key, append (rare).  The query index goes through an opaque copy so
        // that the addresses below are formed here and not carried as induction variables of the hot loop.
        auto survivors = [&](uint32_t bq, const BitsQ<W>& q, const uint32_t (&r)[4]) {
            asm volatile("" : "+s"(bq));
            const linr_filter* F = A.filters + bq;
            const uint32_t fa = Wq.fall[bq], fn = Wq.fnone[bq];
            const bool complex = (Wq.fflag[bq] & 1u) != 0u;
            u64* seg_p = A.seg + ((u64)slot * A.B + bq) * A.cap;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int matches = kb - (int)(r[u] - q.bias);
                bool ok = live[u] & ((int)r[u] < 0) & ((cur.mk[u] & fn) == fa);
                if (has_ts) ok = ok & (cur.ts[u] >= Wq.tsmin[bq]) & (cur.ts[u] <= Wq.tsmax[bq]);
                if (ok && complex) ok = filter_pass(*F, cur.mk[u], has_ts, cur.ts[u]);
                if (ok) {
                    const u64 item = item0 + u * 64 + lane;
                    const u64 key = ((u64)ord_i32(matches) << 32) | (u64)(uint32_t)~(uint32_t)item;
                    const uint32_t pos = atomicAdd(&Wq.cnt[bq], 1u);
                    if (pos < A.cap) seg_p[pos] = key;
                    if (pos + 1 + LINR_BITS_CH > A.cap) need_compact = 1u;
                }
            }
        };
        auto match4 = [&](const BitsQ<W>& q, uint32_t (&r)[4]) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                uint32_t acc = q.bias;
#pragma unroll
                for (int w = 0; w < W; ++w) {
                    const u64 x = cur.x[u][w] ^ q.code[w];
                    acc = bcnt_acc((uint32_t)x, acc);
                    acc = bcnt_acc((uint32_t)(x >> 32), acc);
                }
                r[u] = acc;
            }
        };
        // two queries per trip (the record after an odd batch's last query has a bound nothing reaches); the next
        // two records are read ahead (entries up to NQ + 1 exist)
        BitsQ<W> qn0 = qrec[0], qn1 = qrec[1];
#pragma unroll 1
        for (uint32_t b = 0; b < A.B; b += 2) {
            const BitsQ<W> q0 = qn0, q1 = qn1;
            qn0 = qrec[b + 2];
            qn1 = qrec[b + 3];
            uint32_t r0[4], r1[4];
            match4(q0, r0);
            match4(q1, r1);
            const uint32_t h0 = r0[0] | r0[1] | r0[2] | r0[3], h1 = r1[0] | r1[1] | r1[2] | r1[3];
            if (!wave_any((int)(h0 | h1) < 0)) continue;
            if (wave_any((int)h0 < 0)) survivors(b, q0, r0);
            if (wave_any((int)h1 < 0)) survivors(b + 1, q1, r1);
        }
        bool refresh = ++since_refresh >= 16;
        if (wave_any(need_compact != 0u)) {
            compact_full_segments<LINR_BITS_CH>(A, qs, slot, 0, NQ, hist_all[wib], lane);
            need_compact = 0u;
            refresh = true;
        }
        if (refresh) {
            for (uint32_t ql = lane; ql < (uint32_t)NQ; ql += 64) load_query_side(qs, ql, ql, A, false);
            wave_sync();
            set_bias();
            since_refresh = 0;
        }
        if constexpr (DEEP) { lcA = lcB; vA = vB; lcB = lcC; vB = vC; }
        else { lcA = lcC; vA = vC; }
        return true;
    };
    if constexpr (DEEP) {
        while (true) {
            if (!step(S0, S2)) break;
            if (!step(S1, S0)) break;
            if (!step(S2, S1)) break;
        }
    } else {
        while (true) {
            if (!step(S0, S1)) break;
            if (!step(S1, S0)) break;
        }
    }
    own_stores_done();
    flush_segments(A, qs, slot, 0, NQ, lane, hist_all[wib]);
}

// ---------------------------------------------------------------------------
// quantised search for many queries: bit matching on the matrix cores.
//   With item bits a in {0, 1} and query bits q mapped to {-1, +1}, sum_j a_j q_j = (#bits both 1) - (#item 1, query 0)
//   and the number of equal bits is that sum + (number of 0 bits in the query's code): a 16-item x 16-query tile of
//   match counts is ONE int8 matrix instruction per 64 code bits whose accumulator starts at the query's constant.
//   A lane expands its 16 bits of an item's code word to 16 bytes of 0 / 1 in registers (the code stays 8 bytes per
//   item in HBM); the queries' +-1 bytes are built once per wave.  Everything after the product -- bound test,
//   predicate, candidate segments, compaction, flush -- is the exact scan's (tile_survivors etc.) with the match
//   count as a raw integer ranking value.  Waves are independent chunk-slots; a chunk is 128 items.
// ---------------------------------------------------------------------------
#define LINR_BITSM_CH 128

// 16 bits -> 16 bytes of 0 / 1 (four registers; byte j of the result = bit j)
__device__ __forceinline__ v4i expand16(uint32_t bits16)
{
    v4i r;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        r[j] = (int)((((bits16 >> (4 * j)) & 0xFu) * 0x00204081u) & 0x01010101u);
    return r;
}

template <int W, int QG>
__global__ void __launch_bounds__(64 * WPB, (QG * W <= 4 ? 3 : 2)) scan_kernel_bits_mfma(linr_scan_args A)
{
    constexpr int CH = LINR_BITSM_CH, TPC = 8, NQ = QG * 16;
    // per-wave scratch: 256 words for the compaction's histogram; the final flush needs 2 * NQ + 1 words
    constexpr int SCRATCH = 2 * NQ + 1 > 256 ? 2 * NQ + 8 : 256;
    __shared__ WaveQ<QG> wq_all[WPB];
    __shared__ uint32_t hist_all[WPB][SCRATCH];
    __shared__ u64 stage_all[WPB][CH * W];
    __shared__ __attribute__((aligned(16))) uint32_t stage_side[WPB][2][CH];     // masks, timestamps of the chunk
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    WaveQ<QG>& Wq = wq_all[wib];
    const QSide qs = {Wq.cnt, Wq.thr_f, Wq.thr_i, Wq.fall, Wq.fnone, Wq.tsmin, Wq.tsmax, Wq.fflag};
    const int row = lane & 15, g4 = lane >> 4;
    const uint32_t gw = blockIdx.x * WPB + wib;
    const uint32_t split = gw % A.nsplit, slot = gw / A.nsplit;
    if (slot >= A.nslots) return;
    const uint32_t q_first = split * NQ;
    const bool has_ts = A.ts != nullptr;
    const int sh = 16 * (g4 & 1);                        // this lane's 16 bits of a word: half g4 / 2, shifted by sh
    const bool hi_half = g4 >= 2;

    // ---- query operand: bits -> +1 / -1 bytes; accumulator start = number of 0 bits of the code
    v4i q[QG][W];
    v4i cinit[QG];
    int zeros_q[QG];
#pragma unroll
    for (int i = 0; i < QG; ++i) {
        const uint32_t qi = q_first + i * 16 + row;
        int zeros = 0;
#pragma unroll
        for (int w = 0; w < W; ++w) {
            const u64 code = qi < A.B ? ((const u64*)A.Q)[(u64)qi * W + w] : 0ull;
            const uint32_t half = hi_half ? (uint32_t)(code >> 32) : (uint32_t)code;
            const v4i e = expand16((half >> sh) & 0xFFFFu);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t ff = (uint32_t)e[j] * 255u;                 // 0xFF where the bit is 1
                q[i][w][j] = qi < A.B ? (int)(0xFFFFFFFFu ^ (ff & 0xFEFEFEFEu)) : 0;   // 0x01 for 1, 0xFF (-1) for 0
            }
            zeros += 64 - __popcll(code);
        }
        zeros_q[i] = zeros - (64 * W - (int)A.k_bits);                      // bits beyond k_bits are 0 in every code
    }

    for (uint32_t ql = lane; ql < (uint32_t)NQ; ql += 64) {
        Wq.cnt[ql] = 0;
        load_query_side(qs, ql, q_first + ql, A, true);
    }
    wave_sync();
    int thr_i[QG];
    uint32_t f_all[QG], f_none[QG];
    // The accumulators start at (zero bits of the query) - (the query's bound), so that they hold matches - bound and
    // "some item of the tile reaches some query's bound" is one running maximum over all groups against 0: two vector
    // instructions per matrix instruction.  No bound yet: a start value that keeps everything non-negative.
    auto set_start = [&]() {
#pragma unroll
        for (int i = 0; i < QG; ++i) {
            thr_i[i] = Wq.thr_i[i * 16 + row];
            const int c = zeros_q[i] + (thr_i[i] == INT_MIN ? (1 << 30) : -thr_i[i]);
            cinit[i] = (v4i){c, c, c, c};
        }
    };
    set_start();
#pragma unroll
    for (int i = 0; i < QG; ++i) { f_all[i] = Wq.fall[i * 16 + row]; f_none[i] = Wq.fnone[i * 16 + row]; }

    // ---- items: a chunk's code words travel through registers (next chunk in flight, two items per lane) into the
    // wave's LDS area, from which a lane picks the word of its tile row (keeps the tile loop rolled)
    const u64* codes = (const u64*)A.emb;
    const u64 last = A.n - 1;
    u64* stage = stage_all[wib];
    uint32_t* stage_mk = stage_side[wib][0];
    uint32_t* stage_ts = stage_side[wib][1];
    u64 nxt[2][W];
    uint32_t nxt_mk[2], nxt_ts[2] = {0u, 0u};
    auto issue = [&](u64 lc) {
        const u64 item0 = lc * A.stride * CH;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            u64 it = item0 + h * 64 + lane;
            it = it < last ? it : last;
#pragma unroll
            for (int w = 0; w < W; ++w) nxt[h][w] = __builtin_nontemporal_load(codes + it * W + w);
            nxt_mk[h] = __builtin_nontemporal_load(A.mask + it);
            if (has_ts) nxt_ts[h] = __builtin_nontemporal_load(A.ts + it);
        }
    };
    uint32_t need_compact = 0u, since_refresh = 0u;
    SweepWalk walk;
    walk.init(slot, A);
    u64 lc = walk.lc();
    if (walk.valid()) issue(lc);
    while (walk.valid()) {
        const u64 item0 = lc * A.stride * CH;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int w = 0; w < W; ++w) stage[(h * 64 + lane) * W + w] = nxt[h][w];
#pragma unroll
        for (int h = 0; h < 2; ++h) { stage_mk[h * 64 + lane] = nxt_mk[h]; stage_ts[h * 64 + lane] = nxt_ts[h]; }
        wave_sync();
        walk.advance();
        const u64 nlc = walk.lc();
        if (walk.valid()) issue(nlc);

        u64 code_next[W];                                 // the next tile's words are read one tile ahead
#pragma unroll
        for (int w = 0; w < W; ++w) code_next[w] = stage[row * W + w];
#pragma unroll 1
        for (int t = 0; t < TPC; ++t) {
            v4i a[W];
#pragma unroll
            for (int w = 0; w < W; ++w) {
                const u64 code = code_next[w];
                code_next[w] = stage[(((t + 1) & (TPC - 1)) * 16 + row) * W + w];
                const uint32_t half = hi_half ? (uint32_t)(code >> 32) : (uint32_t)code;
                a[w] = expand16((half >> sh) & 0xFFFFu);
            }
            const int ib = t * 16 + 4 * g4;               // first of this lane's four items (output rows) in the chunk
            v4i acc[QG];
            int best = INT_MIN;
#pragma unroll
            for (int i = 0; i < QG; ++i) {
                v4i c = cinit[i];
#pragma unroll
                for (int w = 0; w < W; ++w) c = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[w], q[i][w], c, 0, 0, 0);
                acc[i] = c;
                best = max(max(best, c[0]), c[1]);
                best = max(max(best, c[2]), c[3]);
            }
            if (wave_any(best >= 0)) {
                u64 hot[QG];
#pragma unroll
                for (int i = 0; i < QG; ++i) {
                    hot[i] = wave_ballot(max(max(acc[i][0], acc[i][1]), max(acc[i][2], acc[i][3])) >= 0);
                    const int back = thr_i[i] == INT_MIN ? -(1 << 30) : thr_i[i];      // back to match counts
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[i][r] += back;
                }
                // masks and timestamps of the lane's four items, staged with the codes
                const v4u mk4 = *(const v4u*)&stage_mk[ib];
                const v4u ts4 = *(const v4u*)&stage_ts[ib];
#pragma unroll
                for (int i = 0; i < QG; ++i)
                    if (hot[i])
                        tile_survivors<LINR_VK_I8_RAW, false, CH>(acc[i], (hot[i] >> lane) & 1ull, mk4, f_all[i], f_none[i], qs,
                                                                  i * 16 + row, q_first + i * 16 + row, ib, item0,
                                                                  [&] { return (v4f){0, 0, 0, 0}; }, [&] { return ts4; }, A, slot,
                                                                  has_ts, need_compact);
            }
        }
        wave_sync();
        bool refresh = ++since_refresh >= 16;
        if (wave_any(need_compact != 0u)) {
            compact_full_segments<CH>(A, qs, slot, q_first, NQ, hist_all[wib], lane);
            need_compact = 0u;
            refresh = true;
        }
        if (refresh) {
            for (uint32_t ql = lane; ql < (uint32_t)NQ; ql += 64) load_query_side(qs, ql, q_first + ql, A, false);
            wave_sync();
            set_start();
            since_refresh = 0;
        }
        lc = nlc;
    }
    own_stores_done();
    flush_segments(A, qs, slot, q_first, NQ, lane, hist_all[wib]);
}

// Sign-OPORP codes of n rows: thread (row, word) sums its 64 bins in double precision, t ascending, and
// sets bit j%64 of word j/64 for a strictly positive bin sum (Sec. 3.2; construction in the header).  Codes of
// more bits than one pass over the coordinates gives (Sec. 5.3.1: 512 bits for d = 128) are `reps` independent
// draws one after the other: bit r * k1 + j comes from bin j of draw r (perm / signs are [reps][d], k1 = k_bits / reps).
__global__ void __launch_bounds__(256) sign_oporp_kernel(int dtype, const void* x, u64 n, uint32_t d, const uint32_t* perm,
                                                         const int8_t* signs, uint32_t k_bits, uint32_t reps, u64* out,
                                                         const uint32_t* scatter)
{
    const uint32_t Wn = (k_bits + 63) / 64, k1 = k_bits / reps, L = d / k1;
    const u64 t = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n * Wn) return;
    const u64 row = t / Wn;
    const uint32_t w = (uint32_t)(t % Wn);
    u64 word = 0;
    for (uint32_t jj = 0; jj < 64; ++jj) {
        const uint32_t j = w * 64 + jj;
        if (j >= k_bits) break;
        const uint32_t base = (j / k1) * d + (j % k1) * L;       // draw j / k1, bin j % k1
        double sum = 0.0;
        for (uint32_t q = 0; q < L; ++q) {
            const uint32_t col = perm[base + q];
            double v;
            if (dtype == LINR_F32) v = (double)((const float*)x)[row * d + col];
            else v = (double)__uint_as_float((uint32_t)((const uint16_t*)x)[row * d + col] << 16);
            sum = sum + (signs[base + q] > 0 ? v : -v);
        }
        if (sum > 0.0) word |= 1ull << jj;
    }
    out[scatter ? (u64)scatter[row] * Wn + w : t] = word;
}

// The same codes for a FEW rows (the queries of a search): one wave per (row, word), lane jj sums bin 64 w + jj in the
// same order and precision, the word is the ballot of the signs.  A thread per word would walk its 64 bins one after
// the other, which for a batch of 16 queries of 512 bits is 60 us of latency in front of every search.
__global__ void __launch_bounds__(256) sign_oporp_rows_kernel(int dtype, const void* x, u64 n, uint32_t d, const uint32_t* perm,
                                                              const int8_t* signs, uint32_t k_bits, uint32_t reps, u64* out,
                                                              const uint32_t* scatter)
{
    const uint32_t Wn = (k_bits + 63) / 64, k1 = k_bits / reps, L = d / k1;
    const u64 t = ((u64)blockIdx.x * blockDim.x + threadIdx.x) >> 6;       // (uniform over the wave)
    if (t >= n * Wn) return;
    const u64 row = t / Wn;
    const uint32_t w = (uint32_t)(t % Wn), j = w * 64 + (threadIdx.x & 63u);
    bool on = false;
    if (j < k_bits) {
        const uint32_t base = (j / k1) * d + (j % k1) * L;
        double sum = 0.0;
        for (uint32_t q = 0; q < L; ++q) {
            const uint32_t col = perm[base + q];
            double v;
            if (dtype == LINR_F32) v = (double)((const float*)x)[row * d + col];
            else v = (double)__uint_as_float((uint32_t)((const uint16_t*)x)[row * d + col] << 16);
            sum = sum + (signs[base + q] > 0 ? v : -v);
        }
        on = sum > 0.0;
    }
    const u64 word = wave_ballot(on);
    if ((threadIdx.x & 63u) == 0u) out[scatter ? (u64)scatter[row] * Wn + w : t] = word;
}

// ---------------------------------------------------------------------------
// attribute matching over clause lists (LiNR Sec. 3.1.1; 64-bit attributes as in the benchmark of Sec. 5.3)
//   One thread per item.  The item's lists sit back to back in its row of the values matrix, their lengths in
//   the count matrix; the lists of up to 32 queries are staged in LDS.  For every clause each attribute of the
//   item is read once and compared with the clause's list of every query (uniform LDS reads); bit b of the
//   result says that the item satisfies all clauses of query b.  A clause for which a query lists nothing does
//   not constrain that query; a reverse clause is satisfied by "no attribute matches".
// ---------------------------------------------------------------------------
#define LINR_CLAUSE_MAX_C 8
#define LINR_CLAUSE_MAX_QW 64
#define LINR_CLAUSE_MAX_ENT (32 * LINR_CLAUSE_MAX_QW)

// The group's query lists, regrouped by clause: entry e of clause c (start[c] <= e < start[c + 1]) is one attribute
// some query lists for c, with that query's bit.  Written once per group by one small workgroup; the item pass then
// walks a clause's entries with uniform (scalar) reads.
struct ClauseEntries {
    u64 val[LINR_CLAUSE_MAX_ENT];
    uint32_t bit[LINR_CLAUSE_MAX_ENT];
    uint32_t start[LINR_CLAUSE_MAX_C + 1];
    uint32_t constrained[LINR_CLAUSE_MAX_C];          // bit b: query b lists something for this clause
};

__global__ void __launch_bounds__(256) clause_entries_kernel(linr_clause_args A, ClauseEntries* E)
{
    __shared__ uint32_t len[32][LINR_CLAUSE_MAX_C], qoff[32][LINR_CLAUSE_MAX_C], tot[LINR_CLAUSE_MAX_C + 1];
    const uint32_t C = A.n_clauses, nq = A.nq, t = threadIdx.x;
    if (t < nq) {
        uint32_t off = 0;
        for (uint32_t c = 0; c < C; ++c) {
            uint32_t l = A.q_counts[t * C + c];
            if (off + l > A.q_width) l = A.q_width - off;       // counts that overrun the query's row are cut
            len[t][c] = l; qoff[t][c] = off;
            off += l;
        }
    }
    __syncthreads();
    if (t == 0) {
        uint32_t run = 0;
        for (uint32_t c = 0; c < C; ++c) {
            tot[c] = run;
            uint32_t cons = 0;
            for (uint32_t b = 0; b < nq; ++b) { run += len[b][c]; if (len[b][c]) cons |= 1u << b; }
            E->constrained[c] = cons;
        }
        tot[C] = run;
        for (uint32_t c = 0; c <= C; ++c) E->start[c] = tot[c];
    }
    __syncthreads();
    if (t < nq * C) {
        const uint32_t c = t / nq, b = t % nq;
        uint32_t pos = tot[c];
        for (uint32_t b2 = 0; b2 < b; ++b2) pos += len[b2][c];
        for (uint32_t j = 0; j < len[b][c]; ++j) {
            E->val[pos + j] = (u64)A.q_values[(u64)b * A.q_width + qoff[b][c] + j];
            E->bit[pos + j] = 1u << b;
        }
    }
}

__global__ void __launch_bounds__(256) clause_words_kernel(linr_clause_args A, const ClauseEntries* __restrict__ E)
{
    const uint32_t C = A.n_clauses, nq = A.nq;
    const uint32_t all = nq >= 32 ? 0xFFFFFFFFu : ((1u << nq) - 1u);
    for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < A.n; i += (u64)gridDim.x * blockDim.x) {
        const u64* row = (const u64*)A.values + i * A.width;
        const uint8_t* cnt = A.counts + i * C;
        uint32_t ok = all, io = 0;
        for (uint32_t c = 0; c < C; ++c) {
            const uint32_t len = cnt[c];
            const uint32_t e0 = E->start[c], e1 = E->start[c + 1];
            uint32_t match = 0u;
            for (uint32_t a = 0; a < len && io + a < A.width; ++a) {
                const u64 v = row[io + a];
                uint32_t e = e0;
                for (; e + 4 <= e1; e += 4) {                   // four entries per trip: their scalar reads overlap
                    const u64 v0 = E->val[e], v1 = E->val[e + 1], v2 = E->val[e + 2], v3 = E->val[e + 3];
                    const uint32_t b0 = E->bit[e], b1 = E->bit[e + 1], b2 = E->bit[e + 2], b3 = E->bit[e + 3];
                    match |= (b0 & (0u - (uint32_t)(v0 == v))) | (b1 & (0u - (uint32_t)(v1 == v))) |
                             (b2 & (0u - (uint32_t)(v2 == v))) | (b3 & (0u - (uint32_t)(v3 == v)));
                }
                for (; e < e1; ++e) match |= E->bit[e] & (0u - (uint32_t)(E->val[e] == v));
            }
            const uint32_t sat = ((A.reverse >> c) & 1u) ? ~match : match;
            ok &= sat | ~E->constrained[c];
            io += len;
        }
        if (A.dead_bit && (A.mask[i] & A.dead_bit)) ok = 0u;
        A.out[i] = ok;
    }
}

__global__ void __launch_bounds__(64) bit_filters_kernel(linr_filter* f, uint32_t nq)
{
    const uint32_t b = threadIdx.x;
    if (b >= nq) return;
    linr_filter F;
    F.all_bits = 1u << b; F.none_bits = 0u;
    for (int g = 0; g < LINR_MAX_ANY; ++g) F.any_bits[g] = 0u;
    F.n_any = 0u; F.ts_min = 0u; F.ts_max = 0xFFFFFFFFu; F._pad = 0u;
    f[b] = F;
}

// ---------------------------------------------------------------------------
// explicit pre-filtering (LiNR Sec. 3.1.2): the feasibility words are scanned, only feasible (item, query) pairs
// are scored -- one lane per pair, rows read with 16-byte loads -- and their keys are appended where the merge
// looks for candidates.  Pays off when few items are feasible; the scan kernels above serve the other case.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int dot_i8_row(const int8_t* q, const int8_t* x, uint32_t d);      // (defined with the merge)

__device__ __forceinline__ float dot_f32_row(const float* q, const float* x, uint32_t d)
{
    float s = 0.0f;
    for (uint32_t j = 0; j < d; j += 4) {
        const float4 a = *(const float4*)(q + j), b = *(const float4*)(x + j);
        s += a.x * b.x; s += a.y * b.y; s += a.z * b.z; s += a.w * b.w;
    }
    return s;
}

__device__ __forceinline__ float dot_bf16_row(const uint16_t* q, const uint16_t* x, uint32_t d)
{
    float s = 0.0f;
    for (uint32_t j = 0; j < d; j += 8) {
        const v4i a = *(const v4i*)(q + j), b = *(const v4i*)(x + j);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            s += __uint_as_float((uint32_t)a[w] << 16) * __uint_as_float((uint32_t)b[w] << 16);
            s += __uint_as_float((uint32_t)a[w] & 0xFFFF0000u) * __uint_as_float((uint32_t)b[w] & 0xFFFF0000u);
        }
    }
    return s;
}

// sixteen bytes of a row against sixteen bytes of a query, already in registers
__device__ __forceinline__ int dot16_i8(v4i a, v4i b)
{
    int s = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) s = __builtin_amdgcn_sdot4(a[w], b[w], s, false);
    return s;
}
__device__ __forceinline__ float dot16_bf16(v4i a, v4i b)
{
    float s = 0.0f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        s += __uint_as_float((uint32_t)a[w] << 16) * __uint_as_float((uint32_t)b[w] << 16);
        s += __uint_as_float((uint32_t)a[w] & 0xFFFF0000u) * __uint_as_float((uint32_t)b[w] & 0xFFFF0000u);
    }
    return s;
}
__device__ __forceinline__ float dot16_f32(v4i a, v4i b)
{
    float s = 0.0f;
#pragma unroll
    for (int w = 0; w < 4; ++w) s += __int_as_float(a[w]) * __int_as_float(b[w]);
    return s;
}

#define LINR_VCNT_STRIDE 32            // words between two queries' counters (a 128-byte line each: no false sharing)
#define LINR_PREFILTER_RUN 8           // 64-item groups a wave takes at a time: 512 items, a lane holds 2 x 4 neighbours

// before the first phase: the counters and the sticky "too many" flags (later phases: the counts kernel re-zeroes)
__global__ void __launch_bounds__(64) prefilter_zero_kernel(uint32_t* vcnt)
{
    if (threadIdx.x < 32) {
        vcnt[threadIdx.x * LINR_VCNT_STRIDE] = 0u;
        vcnt[threadIdx.x * LINR_VCNT_STRIDE + 1] = 0u;
    }
}

#define LINR_PREFILTER_QCAP 512        // (item, query) pairs a wave collects before it scores and places them

// w <- 2 w + (the lane's bit of `cond`): one instruction appends a query's verdict to the lane's feasibility word
__device__ __forceinline__ uint32_t shift_in(uint32_t w, u64 cond)
{
    uint32_t r;
    asm("v_addc_co_u32 %0, vcc, %1, %1, %2" : "=v"(r) : "v"(w), "s"(cond) : "vcc");
    return r;
}

// MODE 0: one feasibility word per item is given; 1: bitmask filters; 2: bitmask filters and timestamp windows;
// 3: a list of candidate ids per query is given (a "run" is then 64 slots of one query's list, one per lane: every
// candidate costs a gather, so short runs spread them over many waves)
template <int MODE>
__global__ void __launch_bounds__(256, 4) prefilter_score_kernel(linr_prefilter_args A)
{
    constexpr int R = LINR_PREFILTER_RUN, QCAP = LINR_PREFILTER_QCAP;
    constexpr bool from_filters = MODE == 1 || MODE == 2;
    constexpr bool has_ts = MODE == 2;
    constexpr bool from_lists = MODE == 3;
    // per wave: the feasible (item, query) pairs found so far (item id, query), their keys, and per query a count / a
    // position.  Pairs of many runs share one flush, so a sparse predicate costs few counter updates.
    __shared__ uint32_t queue_all[256 / 64][QCAP];
    __shared__ uint8_t qb_all[256 / 64][QCAP];
    __shared__ u64 keys_all[256 / 64][QCAP];
    __shared__ uint32_t hist_all[256 / 64][32], base_all[256 / 64][32];
    __shared__ u64 bound_all[256 / 64][32];
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    uint32_t* queue = queue_all[wib];
    uint8_t* qb = qb_all[wib];
    u64* keys = keys_all[wib];
    uint32_t* hist = hist_all[wib];
    uint32_t* base = base_all[wib];
    u64* bound = bound_all[wib];
    // (run numbers fit 32 bits: item ids do)
    const uint32_t wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, n_waves = (gridDim.x * blockDim.x) >> 6;
    const uint32_t rpq = from_lists ? (uint32_t)((A.cand_T + 63) / 64) : 1u;                    // runs per query's list
    const uint32_t n_runs = from_lists ? A.nq * rpq : (uint32_t)((A.n + 64 * R - 1) / (64 * R));
    // this phase's runs: those whose number modulo `mod` lies in [lo, hi)
    const uint32_t per = A.hi - A.lo, rem = n_runs % A.mod;
    const uint32_t n_sel = (n_runs / A.mod) * per + (rem > A.lo ? (rem - A.lo < per ? rem - A.lo : per) : 0u);
    // bitmask / timestamp filters (no feasibility words given): the queries' filters in the compact form the scans use
    __shared__ uint32_t f_must[32], f_care[32], f_t0[32], f_span[32];
    __shared__ uint32_t f_any;                 // bit b: query b also has "any of" groups (checked apart, after the loop)
    if (threadIdx.x == 0) f_any = 0u;
    __syncthreads();
    if (from_filters && threadIdx.x < 32) {
        const uint32_t b = threadIdx.x;
        linr_filter F;
        if (b < A.nq) F = A.filters[b];
        else { F.all_bits = 0xFFFFFFFFu; F.none_bits = 0xFFFFFFFFu; F.n_any = 0; F.ts_min = 1; F.ts_max = 0; }
        const uint32_t none = F.none_bits | A.dead_bit;
        const bool impossible = (F.all_bits & none) != 0u || (A.ts != nullptr && F.ts_min > F.ts_max);   // (windows count only with a timestamp column)
        f_must[b] = impossible ? 0xFFFFFFFFu : F.all_bits;
        f_care[b] = impossible ? 0u : (F.all_bits | none);
        f_t0[b] = F.ts_min; f_span[b] = F.ts_max - F.ts_min;
        if (F.n_any && !impossible) atomicOr(&f_any, 1u << b);
    }
    if (lane < 32) bound[lane] = (A.tau && (uint32_t)lane < A.nq) ? A.tau[lane] : 0ull;     // the phase's bounds do not move
    __syncthreads();
    // Many queries: the all / none clauses of ALL of them at once.  (mask & care) == must holds iff it holds byte by byte,
    // so table[p][v] keeps, for byte p of a mask having the value v, the queries whose clauses on that byte are met: an
    // item's feasibility word is the AND of four table entries, whatever the number of queries (three vector
    // instructions per item and QUERY otherwise).  Timestamp windows and any-of groups are checked afterwards, only
    // for the queries that are still feasible somewhere in the run.
    __shared__ uint32_t table[4][256];
    const bool use_table = from_filters && A.table_min != 0u && A.nq >= A.table_min;
    if (use_table) {
        for (uint32_t e = threadIdx.x; e < 1024u; e += blockDim.x) {
            const uint32_t p8 = 8u * (e >> 8), v = e & 255u;
            uint32_t bits = 0u;
            for (uint32_t b = 0; b < 32u; ++b)
                if ((v & ((f_care[b] >> p8) & 255u)) == ((f_must[b] >> p8) & 255u)) bits |= 1u << b;
            table[e >> 8][v] = bits;
        }
        __syncthreads();
    }

    // Scores the `qn` queued pairs (4, 8 or 16 lanes per pair, by the length of a row: each reads 16 bytes of every
    // stretch, two to four exchanges for the sum; all loads of the loop are independent), drops keys below the query's
    // bound, then places the rest: one LDS count per query, ONE round of counter updates (lane b for query b), one
    // store per key.
    const int lpp_log = A.row_bytes >= 256 ? 4 : A.row_bytes >= 128 ? 3 : 2;
    auto flush = [&](uint32_t qn) {
        const int lpp = 1 << lpp_log, ppt = 64 >> lpp_log;
        const int grp = lane >> lpp_log, sub = lane & (lpp - 1);
        // rows of exactly one 16-byte piece per lane (64, 128 or 256 bytes), one embedding per query: two trips' loads
        // are issued before the first product, so twice as many gathers are in flight
        uint32_t j_from = 0;
        if (A.m == 1 && A.row_bytes == (uint32_t)lpp * 16) {
            constexpr int U = 2;
            for (; j_from < qn; j_from += (uint32_t)(U * ppt)) {
                v4i xv[U], qv[U];
                float sc[U];
                uint32_t jj[U], ii[U], bb[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    jj[u] = j_from + (uint32_t)(u * ppt + grp);
                    const bool valid = jj[u] < qn;
                    bb[u] = valid ? qb[jj[u]] : 0u;
                    ii[u] = valid ? queue[jj[u]] : 0u;           // (item 0 exists: its row is read and dropped)
                    xv[u] = *(const v4i*)((const char*)A.emb + (u64)ii[u] * A.row_bytes + sub * 16);
                    sc[u] = A.vk == LINR_VK_I8_SCALED ? A.row_scale[ii[u]] : 1.0f;
                }
#pragma unroll
                for (int u = 0; u < U; ++u) qv[u] = *(const v4i*)((const char*)A.Q + (u64)bb[u] * A.row_bytes + sub * 16);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    uint32_t hi;
                    if (A.dtype == LINR_I8) {
                        int part = dot16_i8(qv[u], xv[u]);
                        if (lpp_log > 3) part += __shfl_xor(part, 8);
                        if (lpp_log > 2) part += __shfl_xor(part, 4);
                        part += __shfl_xor(part, 2); part += __shfl_xor(part, 1);
                        hi = A.vk == LINR_VK_I8_SCALED ? ord_f32((float)part * sc[u]) : ord_i32(part);
                    } else {
                        float part = A.dtype == LINR_F32 ? dot16_f32(qv[u], xv[u]) : dot16_bf16(qv[u], xv[u]);
                        if (lpp_log > 3) part += __shfl_xor(part, 8);
                        if (lpp_log > 2) part += __shfl_xor(part, 4);
                        part += __shfl_xor(part, 2); part += __shfl_xor(part, 1);
                        hi = ord_f32(part);
                    }
                    if (jj[u] < qn && sub == 0) {
                        const u64 key = ((u64)hi << 32) | (u64)(uint32_t)~ii[u];
                        keys[jj[u]] = key < bound[bb[u]] ? 0ull : key;     // below the k-th key found so far: cannot matter
                    }
                }
            }
        }
        for (uint32_t j0 = j_from; j0 < qn; j0 += (uint32_t)ppt) {
            const uint32_t j = j0 + (uint32_t)grp;
            const bool valid = j < qn;
            const uint32_t b = valid ? qb[j] : 0u;
            const u64 i = valid ? queue[j] : 0u;
            const char* x = (const char*)A.emb + i * A.row_bytes;
            uint32_t hi;
            if (A.dtype == LINR_I8) {
                int best = INT_MIN;
                for (uint32_t e = 0; e < A.m; ++e) {
                    const char* q = (const char*)A.Q + ((u64)b * A.m + e) * A.row_bytes;
                    int part = 0;
                    if (valid)
                        for (uint32_t off = (uint32_t)sub * 16; off < A.row_bytes; off += (uint32_t)lpp * 16)
                            part += dot_i8_row((const int8_t*)(q + off), (const int8_t*)(x + off), 16);
                    if (lpp_log > 3) part += __shfl_xor(part, 8);
                    if (lpp_log > 2) part += __shfl_xor(part, 4);
                    part += __shfl_xor(part, 2); part += __shfl_xor(part, 1);
                    best = part > best ? part : best;
                }
                hi = A.vk == LINR_VK_I8_SCALED ? ord_f32((float)best * (valid ? A.row_scale[i] : 0.0f)) : ord_i32(best);
            } else {
                float best = -INFINITY;
                for (uint32_t e = 0; e < A.m; ++e) {
                    const char* q = (const char*)A.Q + ((u64)b * A.m + e) * A.row_bytes;
                    float part = 0.0f;
                    if (valid)
                        for (uint32_t off = (uint32_t)sub * 16; off < A.row_bytes; off += (uint32_t)lpp * 16)
                            part += A.dtype == LINR_F32 ? dot_f32_row((const float*)(q + off), (const float*)(x + off), 4)
                                                        : dot_bf16_row((const uint16_t*)(q + off), (const uint16_t*)(x + off), 8);
                    if (lpp_log > 3) part += __shfl_xor(part, 8);
                    if (lpp_log > 2) part += __shfl_xor(part, 4);
                    part += __shfl_xor(part, 2); part += __shfl_xor(part, 1);
                    best = fmaxf(best, part);
                }
                hi = ord_f32(best);
            }
            if (valid && sub == 0) {
                const u64 key = ((u64)hi << 32) | (u64)(uint32_t)~(uint32_t)i;
                keys[j] = key < bound[b] ? 0ull : key;         // below the k-th key found so far: cannot matter any more
            }
        }
        if (lane < 32) hist[lane] = 0u;
        wave_sync();
        uint32_t rank[QCAP / 64];
#pragma unroll
        for (int t = 0; t < QCAP / 64; ++t) {
            const uint32_t j = (uint32_t)t * 64 + lane;
            rank[t] = (j < qn && keys[j] != 0ull) ? atomicAdd(&hist[qb[j]], 1u) : 0xFFFFFFFFu;
        }
        wave_sync();
        if (lane < 32) base[lane] = hist[lane] ? atomicAdd(&A.vcnt[lane * LINR_VCNT_STRIDE], hist[lane]) : 0u;
        wave_sync();
#pragma unroll
        for (int t = 0; t < QCAP / 64; ++t) {
            const uint32_t j = (uint32_t)t * 64 + lane;
            if (rank[t] == 0xFFFFFFFFu) continue;
            const uint32_t b = qb[j];
            const uint32_t pos = base[b] + rank[t];
            const u64 key = keys[j];
            if (pos < A.flat_cap) {
                const uint32_t rcap = A.flat_cap / LINR_FLAT_REGIONS;
                A.flat[(u64)b * A.flat_cap + (u64)(pos % LINR_FLAT_REGIONS) * rcap + pos / LINR_FLAT_REGIONS] = key;
            } else {
                const u64 q2 = pos - A.flat_cap;
                const u64 slot = q2 / A.cap;
                if (slot < A.nslots) A.seg[(slot * A.B + b) * A.cap + q2 % A.cap] = key;
            }
        }
        wave_sync();
    };

    // word r = 4 h + c of a lane is item run0 + 256 h + 4 lane + c; `a` = feasibility words or masks, `t` = timestamps
    auto run_of = [&](uint32_t rr) { return (rr / per) * A.mod + A.lo + rr % per; };
    auto load_run = [&](uint32_t rr, uint32_t (&a)[R], uint32_t (&t)[R]) {
        if constexpr (from_lists) {                   // a = candidate id (0xFFFFFFFF: beyond the list), t = its query
            const uint32_t run = run_of(rr), b = run / rpq, c = run % rpq;
            const u64 have = A.cand_counts[b] < A.cand_T ? A.cand_counts[b] : A.cand_T;
            const u64 j = (u64)c * 64 + lane;
#pragma unroll
            for (int r = 0; r < R; ++r) { a[r] = 0xFFFFFFFFu; t[r] = b; }
            if (j < have) a[0] = A.cand[(u64)b * A.cand_T + j];
            return;
        }
        const u64 run0 = (u64)run_of(rr) * (64 * R);
        const uint32_t* src = from_filters ? A.mask : A.words;
        if (run0 + 64 * R <= A.n && A.vec16) {
#pragma unroll
            for (int h = 0; h < R / 4; ++h) {
                const v4i x = __builtin_nontemporal_load((const v4i*)(src + run0 + 256 * h + 4 * lane));
                a[4 * h] = (uint32_t)x[0]; a[4 * h + 1] = (uint32_t)x[1]; a[4 * h + 2] = (uint32_t)x[2]; a[4 * h + 3] = (uint32_t)x[3];
                if (has_ts) {
                    const v4i u = __builtin_nontemporal_load((const v4i*)(A.ts + run0 + 256 * h + 4 * lane));
                    t[4 * h] = (uint32_t)u[0]; t[4 * h + 1] = (uint32_t)u[1]; t[4 * h + 2] = (uint32_t)u[2]; t[4 * h + 3] = (uint32_t)u[3];
                }
            }
        } else {                  // the index's last run, unaligned columns: item by item (what lies beyond is dropped below)
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const u64 i = run0 + 256 * (r / 4) + 4 * lane + (r % 4);
                const u64 ic = i < A.n ? i : A.n - 1;
                a[r] = src[ic];
                if (has_ts) t[r] = A.ts[ic];
            }
        }
        if (!has_ts) {
#pragma unroll
            for (int r = 0; r < R; ++r) t[r] = 0u;
        }
    };

    uint32_t qn = 0;
    uint32_t cur_a[R], cur_t[R];
    if (wave < n_sel) load_run(wave, cur_a, cur_t);
    for (uint32_t rr = wave; rr < n_sel; rr += n_waves) {
        const u64 run0 = (u64)run_of(rr) * (64 * R);
        const bool full = from_lists || run0 + 64 * R <= A.n;
        // the next run's words are on their way while this one is looked at
        uint32_t nxt_a[R], nxt_t[R];
        const bool more = rr + n_waves < n_sel && rr + n_waves > rr;
        if (more) load_run(rr + n_waves, nxt_a, nxt_t);
        uint32_t w[R];
        if constexpr (from_lists) {
#pragma unroll
            for (int r = 0; r < R; ++r) w[r] = cur_a[r] != 0xFFFFFFFFu ? 1u << cur_t[r] : 0u;
        } else if constexpr (!from_filters) {
#pragma unroll
            for (int r = 0; r < R; ++r) w[r] = cur_a[r];
        } else {
            // query by query (its filter constants are uniform) over the eight items, last query first: each verdict is
            // shifted into the word from below
            if (use_table) {
#pragma unroll
                for (int r = 0; r < R; ++r)
                    w[r] = table[0][cur_a[r] & 255u] & table[1][(cur_a[r] >> 8) & 255u] & table[2][(cur_a[r] >> 16) & 255u] &
                           table[3][cur_a[r] >> 24];
                if (has_ts) {                              // windows: only the queries some item of the run still passes for
                    uint32_t live = 0u;
#pragma unroll
                    for (int r = 0; r < R; ++r) live |= w[r];
#pragma unroll
                    for (int o = 32; o > 0; o >>= 1) live |= (uint32_t)__shfl_xor((int)live, o);
                    for (uint32_t cx = (uint32_t)__builtin_amdgcn_readfirstlane((int)live); cx != 0u; cx &= cx - 1u) {
                        const uint32_t b = (uint32_t)__builtin_ctz(cx), t0 = f_t0[b], span = f_span[b];
#pragma unroll
                        for (int r = 0; r < R; ++r)
                            if (cur_t[r] - t0 > span) w[r] &= ~(1u << b);
                    }
                }
            } else {
#pragma unroll
                for (int r = 0; r < R; ++r) w[r] = 0u;
                for (uint32_t b = A.nq; b-- > 0;) {
                    const uint32_t care = f_care[b], must = f_must[b], t0 = has_ts ? f_t0[b] : 0u, span = has_ts ? f_span[b] : 0u;
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        bool ok = (cur_a[r] & care) == must;
                        if (has_ts) ok = ok & (cur_t[r] - t0 <= span);       // t0 <= ts <= t1 (t0 <= t1 here)
                        w[r] = shift_in(w[r], wave_ballot(ok));
                    }
                }
            }
            for (uint32_t cx = f_any; cx != 0u; cx &= cx - 1u) {
                const uint32_t b = (uint32_t)__builtin_ctz(cx);
#pragma unroll
                for (int r = 0; r < R; ++r)
                    if (((w[r] >> b) & 1u) && !filter_pass(A.filters[b], cur_a[r], has_ts, cur_t[r])) w[r] &= ~(1u << b);
            }
        }
        if (!full) {
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (run0 + 256 * (r / 4) + 4 * lane + (r % 4) >= A.n) w[r] = 0u;
        }
        uint32_t any = 0u;
#pragma unroll
        for (int r = 0; r < R; ++r) any |= w[r];
        if (wave_any(any != 0u)) {
            // queue the run's feasible pairs: one pair per lane and trip, lowest query first; a full queue is flushed
#pragma unroll
            for (int r = 0; r < R; ++r) {
                uint32_t word = w[r];
                while (true) {
                    const u64 bal = wave_ballot(word != 0u);
                    if (bal == 0ull) break;
                    if (qn + 64 > (uint32_t)QCAP) { wave_sync(); flush(qn); qn = 0; }
                    if (word) {
                        const uint32_t b = (uint32_t)__builtin_ctz(word);
                        word &= word - 1u;
                        const uint32_t at = qn + (uint32_t)__popcll(bal & ((1ull << lane) - 1ull));
                        queue[at] = from_lists ? cur_a[r] : (uint32_t)run0 + (uint32_t)(256 * (r / 4) + 4 * lane + (r % 4));
                        qb[at] = (uint8_t)b;
                    }
                    qn += (uint32_t)__popcll(bal);
                }
            }
        }
        if (more) {
#pragma unroll
            for (int r = 0; r < R; ++r) { cur_a[r] = nxt_a[r]; cur_t[r] = nxt_t[r]; }
        }
    }
    wave_sync();
    if (qn) flush(qn);
}

// tells the merge where the keys are: per flat region the number of keys, per slot the size of its segment
__global__ void __launch_bounds__(256) prefilter_counts_kernel(linr_prefilter_args A)
{
    const uint32_t b = blockIdx.x;
    const uint32_t total = A.vcnt[b * LINR_VCNT_STRIDE];
    __syncthreads();
    if (threadIdx.x == 0) {
        if ((u64)total > (u64)A.flat_cap + (u64)A.nslots * A.cap) A.vcnt[b * LINR_VCNT_STRIDE + 1] = 1u;
        A.vcnt[b * LINR_VCNT_STRIDE] = 0u;                        // the next phase counts from zero
    }
    const uint32_t in_flat = total < A.flat_cap ? total : A.flat_cap;
    for (uint32_t r = threadIdx.x; r < LINR_FLAT_REGIONS; r += blockDim.x) {
        const u64 ci = ((u64)b * LINR_FLAT_REGIONS + r) * LINR_COUNTER_STRIDE;
        const uint32_t c = in_flat / LINR_FLAT_REGIONS + (r < in_flat % LINR_FLAT_REGIONS ? 1u : 0u);
        A.gcnt[ci] = c;
        A.fvalid[ci] = total > A.flat_cap ? c : 0xFFFFFFFFu;      // "look into the segments too"
    }
    const u64 rest = total - in_flat;
    for (uint32_t s2 = threadIdx.x; s2 < A.nslots; s2 += blockDim.x) {
        const u64 lo = (u64)s2 * A.cap;
        A.cnt[(u64)b * A.nslots + s2] = rest > lo ? (uint32_t)(rest - lo < A.cap ? rest - lo : A.cap) : 0u;
    }
}

// a query with more feasible items than the candidate arrays hold cannot be answered this way: say so in its count
__global__ void __launch_bounds__(64) prefilter_overflow_kernel(const uint32_t* vcnt, uint64_t capacity, uint32_t* out_counts,
                                                                uint32_t nq)
{
    (void)capacity;
    if (threadIdx.x < nq && vcnt[threadIdx.x * LINR_VCNT_STRIDE + 1] != 0u) out_counts[threadIdx.x] = 0xFFFFFFFFu;
}

// ---------------------------------------------------------------------------
// live updates (LiNR Sec. 4 "Model Live Update"): rows and side columns of `count` slots, 8 bytes per thread
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) upsert_kernel(linr_upsert_args A)
{
    const uint32_t pieces = A.row_bytes / 8;
    const u64 t = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (u64)A.count * pieces) return;
    const uint32_t e = (uint32_t)(t / pieces), piece = (uint32_t)(t % pieces);
    const u64 slot = A.slots[e];
    ((u64*)A.emb)[slot * pieces + piece] = ((const u64*)A.src_emb)[(u64)e * pieces + piece];
    if (piece == 0) {
        if (A.row_scale) A.row_scale[slot] = A.src_scale[e];
        if (A.ts) A.ts[slot] = A.src_ts[e];
    }
}

// ... and, in a launch of its own behind the rows (and their codes), the masks: the word that makes a slot visible
__global__ void __launch_bounds__(256) upsert_mask_kernel(linr_upsert_args A)
{
    const uint32_t e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < A.count) A.mask[A.slots[e]] = A.src_mask[e] & ~A.dead_bit;
}

__global__ void __launch_bounds__(256) upsert_clauses_kernel(const uint32_t* slots, uint32_t count, const u64* src_values,
                                                             const uint8_t* src_counts, u64* values, uint8_t* counts, uint32_t width,
                                                             uint32_t n_clauses)
{
    const u64 t = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (u64)count * width) return;
    const uint32_t e = (uint32_t)(t / width), j = (uint32_t)(t % width);
    const u64 slot = slots[e];
    values[slot * width + j] = src_values[(u64)e * width + j];
    if (j < n_clauses) counts[slot * n_clauses + j] = src_counts[(u64)e * n_clauses + j];
    if (j == 0)
        for (uint32_t c = width; c < n_clauses; ++c) counts[slot * n_clauses + c] = src_counts[(u64)e * n_clauses + c];
}

__global__ void __launch_bounds__(256) tombstone_kernel(uint32_t* mask, const uint32_t* slots, uint32_t count, uint32_t dead_bit)
{
    const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < count) atomicOr(mask + slots[t], dead_bit);
}

__global__ void __launch_bounds__(256) fill_u32_kernel(uint32_t* dst, u64 n, uint32_t value)
{
    for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (u64)gridDim.x * blockDim.x) dst[i] = value;
}

__global__ void __launch_bounds__(256) mask_or_kernel(const uint32_t* mask, u64 n, uint32_t* out)
{
    uint32_t acc = 0;
    for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (u64)gridDim.x * blockDim.x) acc |= mask[i];
    if (acc) atomicOr(out, acc);
}

// Second stage of the two-stage search: one workgroup per query scores its T candidates with the
// full-precision embeddings (fp32 accumulation), sorts them by (score desc, id asc) and writes the first k.
#define RESCORE_T 1024
__global__ void __launch_bounds__(RESCORE_T) rescore_kernel(linr_rescore_args A)
{
    __shared__ u64 keys[LINR_MAX_K];
    const uint32_t b = blockIdx.x, tid = threadIdx.x;
    uint32_t c = A.cand_counts[b];
    if (c > A.T) c = A.T;
    uint32_t P = 1;
    while (P < c) P <<= 1;
    // sixteen lanes per candidate: each reads 16 bytes of every 256-byte stretch of the row, four exchanges for the sum
    const uint32_t grp = tid >> 4, sub = tid & 15;
    const char* q = (const char*)A.Q + (u64)b * A.row_bytes;
    for (uint32_t j0 = 0; j0 < P; j0 += RESCORE_T / 16) {
        const uint32_t j = j0 + grp;
        const bool valid = j < c;
        const uint32_t id = valid ? A.cand_ids[(u64)b * A.T + j] : 0u;
        const char* x = (const char*)A.emb + (u64)id * A.row_bytes;
        float part = 0.0f;
        if (valid)
            for (uint32_t off = sub * 16; off < A.row_bytes; off += 256)
                part += A.dtype == LINR_F32 ? dot_f32_row((const float*)(q + off), (const float*)(x + off), 4)
                                            : dot_bf16_row((const uint16_t*)(q + off), (const uint16_t*)(x + off), 8);
        part += __shfl_xor(part, 8); part += __shfl_xor(part, 4); part += __shfl_xor(part, 2); part += __shfl_xor(part, 1);
        if (sub == 0 && j < P) keys[j] = valid ? (((u64)ord_f32(part) << 32) | (u64)(uint32_t)~id) : 0ull;
    }
    __syncthreads();
    for (uint32_t size = 2; size <= P; size <<= 1)
        for (uint32_t str = size >> 1; str > 0; str >>= 1) {
            for (uint32_t j = tid; j < P; j += RESCORE_T) {
                const uint32_t o = j ^ str;
                if (o > j) {
                    const u64 xk = keys[j], yk = keys[o];
                    const bool desc = (j & size) == 0;
                    if (desc ? (xk < yk) : (xk > yk)) { keys[j] = yk; keys[o] = xk; }
                }
            }
            __syncthreads();
        }
    const uint32_t nout = c < A.k ? c : A.k;
    for (uint32_t j = tid; j < A.k; j += RESCORE_T) {
        const u64 o = (u64)b * A.k + j;
        if (j < nout) {
            A.out_ids[o] = ~(uint32_t)keys[j];
            A.out_scores[o] = unord_f32((uint32_t)(keys[j] >> 32));
        } else {
            A.out_ids[o] = LINR_NO_ID;
            A.out_scores[o] = -INFINITY;
        }
    }
    if (tid == 0) A.out_counts[b] = nout;
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
                    tile_survivors<VK, MAGIC, CH>(acc, lane_hot, mk4, qs.fall[qi], qs.fnone[qi], qs, qi, qi, ib, item0,
                                                  [&] { return *(const v4f*)&L.sc[ib]; }, [&] { return *(const v4u*)&L.ts[ib]; }, A,
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
#define NPIECE (LINR_FLAT_REGIONS + 1)
// LDS of a merge workgroup, for k up to KMAX: the winners (KMAX keys) and, when all candidates fit and nothing was
// spilled, the candidates themselves -- 112 KB of the 160 KB a workgroup may use for k <= 2048, 80 KB above that
template <int KMAX>
struct MergeLdsT {
    static constexpr uint32_t LDS_KEYS = KMAX <= 2048 ? 14336u : 10240u;
    union {
        u64 keys[LDS_KEYS];                       // all candidates, when they fit and nothing was spilled
        uint32_t pre[LINR_MAX_SLOTS + 1];         // exclusive prefix of segment counts (spilled case)
    } u;
    u64 win[KMAX];
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

// f(key, j) for keys j = first, first + step, ... < c of src, U loads in flight at a time (a merge workgroup is
// alone on its compute unit and waits for every load it depends on: the latency of a walk is what its time is)
template <int U, typename F>
__device__ __forceinline__ void walk_keys(const u64* src, uint32_t c, uint32_t first, uint32_t step, F f)
{
    for (uint32_t j0 = first; j0 < c; j0 += step * U) {
        u64 kk[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t j = j0 + (uint32_t)u * step;
            kk[u] = j < c ? src[j] : 0ull;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t j = j0 + (uint32_t)u * step;
            if (j < c) f(kk[u], j);
        }
    }
}

// The keys of the carry and of the flat regions of query b, f(key, piece, j) once each: the carried keys by all 1024
// lanes, region r by the 16 lanes 16 r .. 16 r + 15 (a region holds at most flat_cap / 64 keys, usually far fewer).
template <typename LDS, typename F>
__device__ __forceinline__ void walk_flat(const linr_merge_args& A, const LDS& S, uint32_t b, uint32_t tid, F f)
{
    walk_keys<4>(piece_ptr(A, b, 0), S.ppre[1] - S.ppre[0], tid, MT, [&](u64 key, uint32_t j) { f(key, 0u, j); });
    static_assert(MT / 16 == LINR_FLAT_REGIONS, "sixteen lanes per region");
    const uint32_t p = 1u + (tid >> 4);
    walk_keys<8>(piece_ptr(A, b, p), S.ppre[p + 1] - S.ppre[p], tid & 15u, 16u, [&](u64 key, uint32_t j) { f(key, p, j); });
}

// Calls f(key) once for every candidate of the query, by the whole workgroup.  From LDS when they were
// staged there; else from the carry and the flat regions; the per-slot segments (spilled case only) are
// located through the prefix array.
template <typename LDS, typename F>
__device__ __forceinline__ void for_each_candidate(const linr_merge_args& A, const LDS& S, int mode, uint32_t m_flat,
                                                   uint32_t b, uint32_t tid, F f)
{
    if (mode == MERGE_FROM_LDS) {
        for (uint32_t i = tid; i < m_flat; i += MT) f(S.u.keys[i]);
        return;
    }
    const uint32_t wave = tid >> 6, lane = tid & 63;
    walk_flat(A, S, b, tid, [&](u64 key, uint32_t, uint32_t) { f(key); });
    if (mode == MERGE_FROM_ALL) {                      // wave w walks the segments of slots w, w + 16, ...
        const uint32_t* cnt = A.cnt + (u64)b * A.nslots;
        for (uint32_t sl = wave; sl < A.nslots; sl += MT / 64) {
            uint32_t c = cnt[sl];
            if (c > A.cap) c = A.cap;
            const u64* src = A.seg + ((u64)sl * A.B + b) * A.cap;
            for (uint32_t j = lane; j < c; j += 64) f(src[j]);
        }
    }
}

// int32 dot product of two int8 rows (16-byte aligned, d a multiple of 16), 16 bytes per load, four bytes per
// instruction (v_dot4_i32_i8: exact, like the matrix instruction's integer accumulation)
__device__ __forceinline__ int dot_i8_row(const int8_t* q, const int8_t* x, uint32_t d)
{
    int s = 0;
    for (uint32_t j = 0; j < d; j += 16) {
        const v4i a = *(const v4i*)(q + j), b = *(const v4i*)(x + j);
#pragma unroll
        for (int w = 0; w < 4; ++w) s = __builtin_amdgcn_sdot4(a[w], b[w], s, false);
    }
    return s;
}

template <int KMAX>
__global__ void __launch_bounds__(MT) merge_kernel(linr_merge_args A)
{
    __shared__ MergeLdsT<KMAX> S;
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
    } else if (m_flat <= MergeLdsT<KMAX>::LDS_KEYS) {
        // stage everything in LDS
        walk_flat(A, S, b, tid, [&](u64 key, uint32_t p, uint32_t j) { S.u.keys[S.ppre[p] + j] = key; });
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
            for_each_candidate(A, S, mode, m_flat, b, tid, [&](u64 key) {
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
    for_each_candidate(A, S, mode, m_flat, b, tid, [&](u64 key) {
        if (key >= kth) {
            uint32_t p = atomicAdd(&S.nwin, 1u);
            if (p < (uint32_t)KMAX) S.win[p] = key;
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
        // sort them (descending), write the outputs.  Bitonic network over P = 1024 E keys, key e * 1024 + tid in register
        // e of lane tid: partners less than 64 apart are exchanged by lane shuffles, those 1024 or more apart sit in
        // the same lane, and only the strides 64 .. 512 go through LDS and the workgroup barrier.
        constexpr int EMAX = KMAX / MT;
        uint32_t P = MT;
        while (P < nwin) P <<= 1;
        const int E = (int)(P / MT);
        u64 key_e[EMAX];
#pragma unroll
        for (int e = 0; e < EMAX; ++e) {
            const uint32_t idx = (uint32_t)e * MT + tid;
            key_e[e] = (e < E && idx < nwin) ? S.win[idx] : 0ull;
        }
        __syncthreads();
        for (uint32_t size = 2; size <= P; size <<= 1)
            for (uint32_t str = size >> 1; str > 0; str >>= 1) {
                if (str >= MT) {                           // partner in the same lane
                    const int se = (int)(str / MT);
#pragma unroll
                    for (int e = 0; e < EMAX; ++e) {
                        if (e < E && (e & se) == 0) {
                            const uint32_t idx = (uint32_t)e * MT + tid;
                            const bool desc = (idx & size) == 0;
#pragma unroll
                            for (int e2 = 0; e2 < EMAX; ++e2)
                                if (e2 == (e | se)) {
                                    const u64 x = key_e[e], y = key_e[e2];
                                    if (desc ? (x < y) : (x > y)) { key_e[e] = y; key_e[e2] = x; }
                                }
                        }
                    }
                } else if (str >= 64) {                    // through LDS
#pragma unroll
                    for (int e = 0; e < EMAX; ++e)
                        if (e < E) S.win[(uint32_t)e * MT + tid] = key_e[e];
                    __syncthreads();
#pragma unroll
                    for (int e = 0; e < EMAX; ++e)
                        if (e < E) {
                            const uint32_t idx = (uint32_t)e * MT + tid;
                            const u64 y = S.win[idx ^ str];
                            const bool keep_max = ((idx & str) == 0) == ((idx & size) == 0);
                            const u64 x = key_e[e];
                            key_e[e] = keep_max ? (x > y ? x : y) : (x < y ? x : y);
                        }
                    __syncthreads();
                } else {                                   // inside the wave
#pragma unroll
                    for (int e = 0; e < EMAX; ++e)
                        if (e < E) {
                            const uint32_t idx = (uint32_t)e * MT + tid;
                            const u64 x = key_e[e];
                            const uint32_t ylo = (uint32_t)__shfl_xor((int)(uint32_t)x, (int)str);
                            const uint32_t yhi = (uint32_t)__shfl_xor((int)(uint32_t)(x >> 32), (int)str);
                            const u64 y = ((u64)yhi << 32) | ylo;
                            const bool keep_max = ((idx & str) == 0) == ((idx & size) == 0);
                            key_e[e] = keep_max ? (x > y ? x : y) : (x < y ? x : y);
                        }
                }
            }
#pragma unroll
        for (int e = 0; e < EMAX; ++e)
            if (e < E) S.win[(uint32_t)e * MT + tid] = key_e[e];
        __syncthreads();
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
                } else if (A.dtype == LINR_BITS) {
                    const int matches = unord_i32(hi);
                    A.out_scores[o] = (float)matches;
                    if (A.out_raw) A.out_raw[o] = matches;
                } else {
                    A.out_scores[o] = unord_f32(hi);
                }
            } else {
                A.out_ids[o] = LINR_NO_ID;
                A.out_scores[o] = -INFINITY;
                if (A.out_raw && (A.dtype == LINR_I8 || A.dtype == LINR_BITS)) A.out_raw[o] = INT_MIN;
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
// Fixed scratch memory of linr_search_filtered_noalloc: the search workspace of callers that cannot allocate.
// Every GPU the library runs on holds its own copy of the array at its own address; in host code the name is
// only a handle for hipGetSymbolAddress, never an address to hand to a kernel or a copy.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[LINR_NOALLOC_SCRATCH_BYTES];

#define LINR_MAX_DEVICES 64
hipError_t linr_static_scratch(int device, void** ptr)
{
    static std::mutex mu;
    static void* per_device[LINR_MAX_DEVICES];          // device address of `scratch` on each GPU, looked up once
    if (!ptr || device < 0 || device >= LINR_MAX_DEVICES) return hipErrorInvalidValue;
    std::lock_guard<std::mutex> g(mu);
    if (!per_device[device]) {
        int cur = -1;
        hipError_t e = hipGetDevice(&cur);
        if (e != hipSuccess) return e;
        if (cur != device) return hipErrorInvalidDevice;    // the symbol is resolved for the current GPU
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p || (((uintptr_t)p) & 255u)) return hipErrorInvalidSymbol;
        per_device[device] = p;
    }
    *ptr = per_device[device];
    return hipSuccess;
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
    if (a.k <= 2048) hipLaunchKernelGGL(merge_kernel<2048>, dim3(a.B), dim3(MT), 0, s, a);
    else hipLaunchKernelGGL(merge_kernel<LINR_MAX_K>, dim3(a.B), dim3(MT), 0, s, a);
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

#define WIDE_CASE(DT, VK, KS_, QW_)                                                               \
    if (dtype == DT && vk == VK && ks == KS_ && m == 1 && qw == QW_)                              \
        return scan_act(scan_kernel_wide<DT, VK, KS_, QW_>, act);

static hipError_t wide_dispatch(int dtype, int vk, uint32_t ks, uint32_t m, uint32_t qw, ScanAct& act)
{
    WIDE_CASE(LINR_I8, LINR_VK_I8_SCALED, 1, 1) WIDE_CASE(LINR_I8, LINR_VK_I8_SCALED, 1, 2)
    WIDE_CASE(LINR_I8, LINR_VK_I8_RAW, 1, 1)    WIDE_CASE(LINR_I8, LINR_VK_I8_RAW, 1, 2)
    WIDE_CASE(LINR_I8, LINR_VK_I8_SCALED, 2, 1) WIDE_CASE(LINR_I8, LINR_VK_I8_SCALED, 2, 2)
    WIDE_CASE(LINR_I8, LINR_VK_I8_RAW, 2, 1)    WIDE_CASE(LINR_I8, LINR_VK_I8_RAW, 2, 2)
    WIDE_CASE(LINR_I8, LINR_VK_I8_SCALED, 4, 1) WIDE_CASE(LINR_I8, LINR_VK_I8_SCALED, 4, 2)
    WIDE_CASE(LINR_I8, LINR_VK_I8_RAW, 4, 1)    WIDE_CASE(LINR_I8, LINR_VK_I8_RAW, 4, 2)
    WIDE_CASE(LINR_BF16, LINR_VK_FLOAT, 1, 1)   WIDE_CASE(LINR_BF16, LINR_VK_FLOAT, 1, 2)
    WIDE_CASE(LINR_BF16, LINR_VK_FLOAT, 2, 1)   WIDE_CASE(LINR_BF16, LINR_VK_FLOAT, 2, 2)
    WIDE_CASE(LINR_BF16, LINR_VK_FLOAT, 4, 1)   WIDE_CASE(LINR_BF16, LINR_VK_FLOAT, 4, 2)
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

int linr_wide_variant_exists(int dtype, int vk, uint32_t ks, uint32_t m, uint32_t qw)
{
    ScanAct act{}; act.what = ACT_EXISTS;
    return wide_dispatch(dtype, vk, ks, m, qw, act) == hipSuccess;
}

// Per-bit population counts of the mask column over an evenly spaced sample (planner input: how selective is a filter).
__global__ void __launch_bounds__(256) mask_bit_count_kernel(const uint32_t* mask, u64 n, u64 step, unsigned long long* out)
{
    const int lane = threadIdx.x & 63;
    const u64 n_sample = (n + step - 1) / step;
    uint32_t mine = 0;                                   // lane b < 32 accumulates bit b, lane 32 the number of items
    for (u64 j0 = ((u64)blockIdx.x * 256 + (threadIdx.x & ~63u)); j0 < n_sample; j0 += (u64)gridDim.x * 256) {
        const u64 j = j0 + lane;
        const bool in = j < n_sample;
        const uint32_t mk = in ? mask[j * step] : 0u;
#pragma unroll
        for (int b = 0; b < 32; ++b) {
            const uint32_t c = (uint32_t)__popcll(wave_ballot(in && ((mk >> b) & 1u)));
            if (lane == b) mine += c;
        }
        const uint32_t c = (uint32_t)__popcll(wave_ballot(in));
        if (lane == 32) mine += c;
    }
    if (lane <= 32 && mine) atomicAdd(out + lane, (unsigned long long)mine);
}

hipError_t linr_launch_mask_bit_counts(const uint32_t* mask, uint64_t n, uint64_t step, unsigned long long* out, hipStream_t s)
{
    if (n == 0 || step == 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(mask_bit_count_kernel, dim3(1024), dim3(256), 0, s, mask, (u64)n, (u64)step, out);
    return hipGetLastError();
}

hipError_t linr_launch_scale_stats(const float* row_scale, uint64_t n, uint64_t n_pad, float* part, float* out, uint8_t* codes,
                                   hipStream_t s)
{
    hipLaunchKernelGGL(scale_stats_partial, dim3(LINR_SCALE_STAT_BLOCKS), dim3(256), 0, s, row_scale, (u64)n, part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(scale_stats_final, dim3(1), dim3(256), 0, s, (const float*)part, (uint32_t)LINR_SCALE_STAT_BLOCKS, (u64)n, out);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(scale_code_kernel, dim3(4096), dim3(256), 0, s, row_scale, (u64)n, (u64)n_pad, (const float*)out, codes);
    return hipGetLastError();
}

uint32_t linr_lds_scan_dynamic_bytes(uint32_t B, uint32_t m, uint32_t ks)
{
    uint32_t nsg = (B + 15) / 16;
    return nsg * m * ks * 1024u + nsg * 16u * 4u * (7u + WPB);
}

#define BITSM_CASE(W_, QG_) if (words == W_ && qg == QG_) return scan_act(scan_kernel_bits_mfma<W_, QG_>, act);
static hipError_t bits_mfma_dispatch(uint32_t words, uint32_t qg, ScanAct& act)
{
    BITSM_CASE(1, 1) BITSM_CASE(1, 2) BITSM_CASE(1, 4) BITSM_CASE(1, 8)
    BITSM_CASE(2, 1) BITSM_CASE(2, 2) BITSM_CASE(2, 4) BITSM_CASE(2, 8)
    return hipErrorInvalidDeviceFunction;
}
int linr_bits_mfma_variant_exists(uint32_t words, uint32_t qg)
{
    ScanAct act{}; act.what = ACT_EXISTS;
    return bits_mfma_dispatch(words, qg, act) == hipSuccess;
}

static hipError_t bits_dispatch(uint32_t words, ScanAct& act)
{
    if (words == 1) return scan_act(scan_kernel_bits<1>, act);
    if (words == 2) return scan_act(scan_kernel_bits<2>, act);
    if (words == 3) return scan_act(scan_kernel_bits<3>, act);
    if (words == 4) return scan_act(scan_kernel_bits<4>, act);
    if (words == 6) return scan_act(scan_kernel_bits<6>, act);
    if (words == 8) return scan_act(scan_kernel_bits<8>, act);
    return hipErrorInvalidDeviceFunction;
}

hipError_t linr_launch_sign_oporp_scatter(int dtype, const void* x, uint64_t n, uint32_t d, const uint32_t* perm,
                                          const int8_t* signs, uint32_t k_bits, uint32_t reps, uint64_t* out,
                                          const uint32_t* scatter, hipStream_t s)
{
    if (reps == 0 || k_bits == 0 || k_bits % reps != 0 || d % (k_bits / reps) != 0) return hipErrorInvalidValue;
    const uint64_t threads = n * ((k_bits + 63) / 64);
    if (threads == 0) return hipSuccess;
    if (threads <= 16384)                               // few rows (queries): a wave per word
        hipLaunchKernelGGL(sign_oporp_rows_kernel, dim3((uint32_t)((threads + 3) / 4)), dim3(256), 0, s, dtype, x, (u64)n, d, perm,
                           signs, k_bits, reps, (u64*)out, scatter);
    else
        hipLaunchKernelGGL(sign_oporp_kernel, dim3((uint32_t)((threads + 255) / 256)), dim3(256), 0, s, dtype, x, (u64)n, d, perm, signs,
                           k_bits, reps, (u64*)out, scatter);
    return hipGetLastError();
}

hipError_t linr_launch_sign_oporp(int dtype, const void* x, uint64_t n, uint32_t d, const uint32_t* perm, const int8_t* signs,
                                  uint32_t k_bits, uint32_t reps, uint64_t* out, hipStream_t s)
{
    return linr_launch_sign_oporp_scatter(dtype, x, n, d, perm, signs, k_bits, reps, out, nullptr, s);
}

hipError_t linr_launch_clause_words(const linr_clause_args& a, hipStream_t s)
{
    if (a.n == 0) return hipSuccess;
    if (a.nq == 0 || a.nq > 32 || a.n_clauses == 0 || a.n_clauses > LINR_CLAUSE_MAX_C || a.q_width == 0 ||
        a.q_width > LINR_CLAUSE_MAX_QW || a.width == 0 || !a.entries || (((uintptr_t)a.entries) & 7u))
        return hipErrorInvalidValue;
    ClauseEntries* E = (ClauseEntries*)a.entries;
    hipLaunchKernelGGL(clause_entries_kernel, dim3(1), dim3(256), 0, s, a, E);
    const uint64_t blocks = (a.n + 255) / 256;
    hipLaunchKernelGGL(clause_words_kernel, dim3((uint32_t)(blocks < 8192 ? blocks : 8192)), dim3(256), 0, s, a, E);
    return hipGetLastError();
}

uint32_t linr_clause_entries_bytes(void) { return (uint32_t)sizeof(ClauseEntries); }

hipError_t linr_launch_bit_filters(linr_filter* filters, uint32_t nq, hipStream_t s)
{
    if (nq == 0 || nq > 32) return hipErrorInvalidValue;
    hipLaunchKernelGGL(bit_filters_kernel, dim3(1), dim3(64), 0, s, filters, nq);
    return hipGetLastError();
}

hipError_t linr_launch_prefilter(const linr_prefilter_args& a_in, hipStream_t s)
{
    linr_prefilter_args a = a_in;
    if (a.nq == 0 || a.nq > 32 || a.nq > a.B || a.flat_cap % LINR_FLAT_REGIONS != 0 || a.cap == 0 || a.nslots == 0 ||
        a.row_bytes % 16 != 0 || a.mod == 0 || a.lo >= a.hi || a.hi > a.mod)
        return hipErrorInvalidValue;
    // four neighbours' words with one 16-byte load where the columns allow it (borrowed columns need not be aligned)
    a.vec16 = ((((uintptr_t)a.words) | ((uintptr_t)a.mask) | ((uintptr_t)a.ts)) & 15u) == 0 ? 1u : 0u;
    static int per_cu = 0, cus = 0;
    if (per_cu == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess) return hipGetLastError();
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&v, prefilter_score_kernel<2>, 256, 0) != hipSuccess || v <= 0) v = 4;
        per_cu = v;
    }
    if (a.lo == 0) hipLaunchKernelGGL(prefilter_zero_kernel, dim3(1), dim3(64), 0, s, a.vcnt);
    // as many workgroups as are resident at once; a wave keeps its queue across its runs
    const uint64_t runs = a.cand ? (uint64_t)a.nq * ((a.cand_T + 63) / 64)
                                 : (a.n + 64 * LINR_PREFILTER_RUN - 1) / (64 * LINR_PREFILTER_RUN);
    const uint64_t sel = (runs / a.mod + 1) * (a.hi - a.lo);
    const uint64_t blocks = (sel + 3) / 4, most = (uint64_t)cus * per_cu;
    const dim3 grid((uint32_t)(blocks < most ? blocks : most));
    if (a.cand) hipLaunchKernelGGL(prefilter_score_kernel<3>, grid, dim3(256), 0, s, a);
    else if (a.words) hipLaunchKernelGGL(prefilter_score_kernel<0>, grid, dim3(256), 0, s, a);
    else if (!a.ts) hipLaunchKernelGGL(prefilter_score_kernel<1>, grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL(prefilter_score_kernel<2>, grid, dim3(256), 0, s, a);
    hipLaunchKernelGGL(prefilter_counts_kernel, dim3(a.nq), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t linr_launch_prefilter_overflow(const uint32_t* vcnt, uint64_t capacity, uint32_t* out_counts, uint32_t nq, hipStream_t s)
{
    hipLaunchKernelGGL(prefilter_overflow_kernel, dim3(1), dim3(64), 0, s, vcnt, capacity, out_counts, nq);
    return hipGetLastError();
}

hipError_t linr_launch_upsert(const linr_upsert_args& a, hipStream_t s)
{
    if (a.count == 0) return hipSuccess;
    if (a.row_bytes == 0 || a.row_bytes % 8 != 0) return hipErrorInvalidValue;
    const uint64_t threads = (uint64_t)a.count * (a.row_bytes / 8);
    hipLaunchKernelGGL(upsert_kernel, dim3((uint32_t)((threads + 255) / 256)), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t linr_launch_upsert_masks(const linr_upsert_args& a, hipStream_t s)
{
    if (a.count == 0) return hipSuccess;
    hipLaunchKernelGGL(upsert_mask_kernel, dim3((a.count + 255) / 256), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t linr_launch_upsert_clauses(const uint32_t* slots, uint32_t count, const uint64_t* src_values, const uint8_t* src_counts,
                                      uint64_t* values, uint8_t* counts, uint32_t width, uint32_t n_clauses, hipStream_t s)
{
    if (count == 0) return hipSuccess;
    const uint64_t threads = (uint64_t)count * width;
    hipLaunchKernelGGL(upsert_clauses_kernel, dim3((uint32_t)((threads + 255) / 256)), dim3(256), 0, s, slots, count,
                       (const u64*)src_values, src_counts, (u64*)values, counts, width, n_clauses);
    return hipGetLastError();
}

hipError_t linr_launch_tombstone(uint32_t* mask, const uint32_t* slots, uint32_t count, uint32_t dead_bit, hipStream_t s)
{
    if (count == 0) return hipSuccess;
    hipLaunchKernelGGL(tombstone_kernel, dim3((count + 255) / 256), dim3(256), 0, s, mask, slots, count, dead_bit);
    return hipGetLastError();
}

hipError_t linr_launch_fill_u32(uint32_t* dst, uint64_t n, uint32_t value, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    const uint64_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((uint32_t)(blocks < 4096 ? blocks : 4096)), dim3(256), 0, s, dst, (u64)n, value);
    return hipGetLastError();
}

hipError_t linr_launch_mask_or(const uint32_t* mask, uint64_t n, uint32_t* out, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    const uint64_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(mask_or_kernel, dim3((uint32_t)(blocks < 4096 ? blocks : 4096)), dim3(256), 0, s, mask, (u64)n, out);
    return hipGetLastError();
}

hipError_t linr_launch_rescore(const linr_rescore_args& a, hipStream_t s)
{
    if (a.T > LINR_MAX_K || a.k > a.T) return hipErrorInvalidValue;
    hipLaunchKernelGGL(rescore_kernel, dim3(a.B), dim3(RESCORE_T), 0, s, a);
    return hipGetLastError();
}

static hipError_t plan_dispatch(const linr_plan& p, int dtype, uint32_t B, uint32_t m, bool ts, ScanAct& act)
{
    if (p.bits == 2) { act.dyn = 0; return bits_mfma_dispatch(p.ks, p.qg, act); }
    if (p.bits) { act.dyn = 0; return bits_dispatch(p.ks, act); }
    if (p.generic) {
        act.dyn = linr_lds_scan_dynamic_bytes(B, m, p.ks);
        return lds_dispatch(dtype, p.vk, p.ks, act);
    }
    act.dyn = 0;
    if (p.dense && dtype == LINR_BF16)
        return linr_dense_bf16_dispatch(act.what == ACT_EXISTS ? 0 : act.what == ACT_OCCUPANCY ? 1 : 2, p.ks, p.qg, m, ts, act.grid, act.s,
                                        act.a, &act.blocks_per_cu);
    if (p.dense)
        return linr_dense_dispatch(act.what == ACT_EXISTS ? 0 : act.what == ACT_OCCUPANCY ? 1 : 2, p.vk, p.qg, ts, act.grid, act.s,
                                   act.a, &act.blocks_per_cu);
    if (p.wide) return wide_dispatch(dtype, p.vk, p.ks, m, p.qg, act);
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
