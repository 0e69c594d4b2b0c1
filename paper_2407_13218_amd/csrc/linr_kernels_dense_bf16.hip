// Scan kernel for large bf16 batches (rows of 256 bytes: d = 128, the shape of the benchmark in LiNR, arXiv 2407.13218,
// Sec. 5.3, m = 1; and rows of 128 bytes with m = 8 embeddings per query, the multi-embedding score of Sec. 3.1.1):
// the large-batch design of linr_kernels_dense.hip for a float ranking value.
//
// Same ideas, simpler arithmetic (no row scales):
//   * queries are the ROW operand, so after the products of a group a lane holds 4 queries x ONE item;
//   * the bound of each query enters through the accumulator input: acc = <q, x> - thr_q', thr_q' the query's bound
//     lowered by the rounding slack.  "Some query wants this item" is max_q(acc) >= 0: two v_max3_f32 per group of
//     16 queries (four v_mfma_f32_16x16x32_bf16 each), one compare per tile;
//   * a quarter (64 queries) of a tile that fired is finished at once, its accumulators still in registers: every lane
//     finishes its pairs one per round: all / none clauses, timestamp window, ranking value s = acc + thr_q' against the bound
//     itself, any-of clauses; keys are queued in LDS and written out in bulk.  (s differs from a sum accumulated from
//     zero by a rounding of the bound's magnitude at most; every comparison of the search -- candidate test, bound
//     of later sweeps, final order -- is made on these same values.  A query without a bound yet enters with 0.)
//   * every wave is autonomous: a private ring of steps of ONE tile (16 items: 4 KB of rows + masks), direct global ->
//     LDS loads, a counted wait per step, hand-placed LDS reads, no workgroup barrier per step;
//   * a wave keeps up to 8 query groups (128 queries: 128 registers of fragments + 32 of bounds); the four waves of a
//     workgroup hold up to four query sets (512 queries per stream of the index) or walk different chunks;
//   * m = 8: the eight embeddings of a query are the rows 4 (l / 16) .. + 3 of two neighbouring groups, so that ONE lane
//     holds all eight values of a (query, item) pair; they share the query's bound as accumulator input, the tile's test
//     is the same maximum, and the pair's ranking value is the maximum of the lane's eight accumulators.  A wave keeps
//     16 groups = 32 queries, a workgroup up to 128.
// Matrix work dominates here (32 products of 16 clocks per tile against 16 + a few vector instructions).
#include "linr_dense.h"

#define DENSEF_STEP 16                 // items per step of a wave: one tile

template <int KS, int NG, int M, bool TS>
__global__ void __launch_bounds__(64 * WPB, 2) scan_kernel_dense_bf16(linr_scan_args A)
{
    static_assert(M == 1 || M == 8, "one embedding per query, or eight");
    constexpr int NQW = NG * 16 / M;                     // query positions per wave
    constexpr int NQT = NG / 4;                          // quarters (four groups: 64 / M queries) per wave
    constexpr int QPQ = 64 / M;                          // queries per quarter
    constexpr int NC = M == 8 ? NG / 2 : NG;             // accumulator inputs kept per lane (m = 8: one per pair of groups)
    constexpr int RB = KS * 64;                          // bytes per row
    constexpr int ROWS = KS * 1024;                      // bytes of a tile's rows
    constexpr int STG = ROWS + 256 + (TS ? 256 : 0);     // bytes of a ring stage: rows, masks, timestamps
    constexpr int NST = KS >= 4 ? 3 : 5;                 // ring stages per wave: NST - 1 steps in flight
    constexpr int DMA = KS + 1 + (TS ? 1 : 0);           // direct loads per step (always this many)
    static_assert(NG % 4 == 0 && NG * KS <= 32, "query fragments must fit the register file");
    static_assert((NST - 2) * DMA <= 63, "the load counter has six bits");
    static_assert(DENSE_SCRATCH_WORDS >= 2 * NQW + 1 + 3 && DENSE_SCRATCH_WORDS >= 2 * DENSE_QCAP + DENSE_QCAP / 4 + 4, "scratch");

    __shared__ __attribute__((aligned(16))) unsigned char ring_all[WPB][NST * STG];
    __shared__ DenseQ<NQW, TS> QS;
    __shared__ uint32_t cnt_all[WPB][NQW];
    __shared__ __attribute__((aligned(8))) uint32_t scratch_all[WPB][DENSE_SCRATCH_WORDS];

    const int lane = threadIdx.x & 63, wib = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = lane & 15, g4 = lane >> 4;
    const uint32_t nsets = A.nsplit;                     // query sets per workgroup: 1, 2 or 4
    const uint32_t wps = WPB / nsets;                    // waves per query set; each walks its own chunks
    const uint32_t qset = (uint32_t)wib % nsets, tlane = (uint32_t)wib / nsets;
    const uint32_t slot = blockIdx.x * wps + tlane;      // this wave's private candidate segments
    const uint32_t per_set = ((A.B + nsets - 1) / nsets + (uint32_t)QPQ - 1u) / (uint32_t)QPQ * (uint32_t)QPQ;
    const uint32_t pos_first = qset * per_set;           // first position of the batch's order this wave serves
    const uint32_t nq_mine = pos_first < A.B ? (A.B - pos_first < per_set ? A.B - pos_first : per_set) : 0u;
    const int nqt = (int)((nq_mine + QPQ - 1) / QPQ);
    const bool has_ts = TS && A.ts != nullptr;
    uint32_t* const cnt = cnt_all[wib];
    u64* const qkey = (u64*)&scratch_all[wib][0];
    uint8_t* const qql = (uint8_t*)&scratch_all[wib][2 * DENSE_QCAP];
    const QSide qs = {cnt, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};   // (the shared helpers use cnt only)
    float* const s_thr = QS.thr + wib * NQW;             // the bounds themselves
    float* const s_low = (float*)(QS.T + wib * NQW);     // the lowered bounds that entered the accumulators
    const uint32_t set0 = qset * NQW;
    const uint32_t* const s_fa = QS.fa + set0;
    const uint32_t* const s_fn = QS.fn + set0;
    const uint8_t* const s_flag = QS.flag + set0;
    const uint16_t* const s_qi = QS.qi + set0;

    if (tlane == 0) {
        for (uint32_t ql = lane; ql < (uint32_t)NQW; ql += 64) {
            const uint32_t pos = pos_first + ql;
            uint32_t qi = 0xFFFFu;
            if (ql < nq_mine) qi = A.qorder ? A.qorder[pos] : pos;
            QS.qi[set0 + ql] = (uint16_t)qi;
            linr_filter F;
            if (qi < A.B) F = A.filters[qi];
            else { F.all_bits = 0xFFFFFFFFu; F.none_bits = 0xFFFFFFFFu; F.n_any = 0; F.ts_min = 1; F.ts_max = 0; }
            const uint32_t none = F.none_bits | A.dead_bit;
            const bool impossible = (F.all_bits & none) != 0u;
            QS.fa[set0 + ql] = impossible ? 0xFFFFFFFFu : F.all_bits;
            QS.fn[set0 + ql] = impossible ? 0u : (F.all_bits | none);
            QS.flag[set0 + ql] = F.n_any ? 1 : 0;
            if constexpr (TS) { QS.t0[set0 + ql] = F.ts_min; QS.t1[set0 + ql] = F.ts_max; }
        }
    }
    __syncthreads();
    // ---- query fragments (row operand): for each 64-byte K-step, lane l supplies bytes [16 (l/16), +16) of row l%16.
    //      m = 1: row r of group g is query position 16 g + r; m = 8: embedding 4 (g % 2) + r % 4 of position 4 (g / 2) + r / 4
    v4i q[NG][KS];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const uint32_t qpos = M == 8 ? (uint32_t)(4 * (g / 2) + col / 4) : (uint32_t)(g * 16 + col);
        const uint32_t emb_e = M == 8 ? (uint32_t)(4 * (g % 2) + (col & 3)) : 0u;
        const uint32_t qi = s_qi[qpos];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            v4i z = {0, 0, 0, 0};
            if (qi < A.B) z = *(const v4i*)((const char*)A.Q + ((u64)qi * M + emb_e) * RB + ks * 64 + g4 * 16);
            q[g][ks] = z;
        }
    }
    // (they must have arrived before the loop: a wait at their first use inside it would empty the ring every time)
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) pin(q[g][ks]);
    for (uint32_t ql = lane; ql < (uint32_t)NQW; ql += 64) cnt[ql] = 0;

    v4f c[NC];                                           // accumulator inputs: -(lowered bound) of the lane's four queries of each group
    bool any_free = false;                               // (uniform) some query of this wave has no bound yet: every tile matters
    auto load_bounds = [&]() __attribute__((always_inline)) {
        bool fr = false;
        for (uint32_t ql = lane; ql < (uint32_t)NQW; ql += 64) {
            const uint32_t qi = s_qi[ql];
            float tf = INFINITY;                         // no query here: never a candidate
            if (qi < A.B) {
                const u64 t = aload64(A.tau + qi);
                tf = t ? unord_f32((uint32_t)(t >> 32)) : -INFINITY;        // (no bound yet: always a candidate)
            }
            s_thr[ql] = tf;
            // what enters the accumulator: the lowered bound; 0 for a query without one (its values are then the dot
            // products themselves; while the wave has such a query, every pair of every tile goes through the slow path)
            s_low[ql] = tf == -INFINITY ? 0.0f : lowered(tf);
            fr = fr || tf == -INFINITY;
        }
        any_free = wave_any(fr);
        wave_sync();
        if constexpr (M == 8) {                          // (all eight rows of a pair of groups belong to one query per lane)
#pragma unroll
            for (int j = 0; j < NC; ++j) {
                const float t = -s_low[4 * j + g4];
                c[j] = (v4f){t, t, t, t};
            }
        } else {
#pragma unroll
            for (int g = 0; g < NC; ++g) {
                const v4f t4 = *(const v4f*)&s_low[g * 16 + 4 * g4];
                c[g] = (v4f){-t4[0], -t4[1], -t4[2], -t4[3]};
            }
        }
    };
    load_bounds();

    uint32_t need_compact = 0u, direct = 0u;
    uint32_t since_refresh = 0;
    uint32_t queued = 0;                                 // keys in the queue (uniform)
    auto flush_queue = [&]() __attribute__((always_inline)) {
        wave_sync();
        const uint32_t nqd = queued;
        for (uint32_t t = lane; t < nqd; t += 64) {
            const u64 key = qkey[t];
            const uint32_t ql = qql[t];
            const uint32_t pos = atomicAdd(&cnt[ql], 1u);
            if (pos < A.cap) A.seg[((u64)slot * A.B + s_qi[ql]) * A.cap + pos] = key;
            if (pos + 1 + DENSE_SLACK > A.cap) need_compact = 1u;
        }
        wave_sync();
        queued = 0;
        __builtin_amdgcn_s_waitcnt(DENSE_WAIT_VM(0));
    };

    // ---- the wave's private ring of steps (one tile each)
    typedef const __attribute__((address_space(1))) void* gptr;
    typedef __attribute__((address_space(3))) void* lptr;
    unsigned char* const ring = ring_all[wib];
    const uint32_t ring_lds = dense_lds_addr(ring);
    const uint32_t nwalk = gridDim.x * wps;
    // (a sweep with few chunks is dealt out by steps instead of chunks: see linr_kernels_dense.hip)
    constexpr uint32_t SPC = DENSE_CH / DENSEF_STEP;     // steps per chunk
    const uint32_t n_dense32 = (uint32_t)A.n_dense, slot_first = blockIdx.x * wps;
    const bool fine = nwalk % SPC == 0u && n_dense32 < nwalk;
    const uint32_t walker = fine ? slot / SPC : slot, walker_first = fine ? slot_first / SPC : slot_first;
    const uint32_t nwalkers = fine ? nwalk / SPC : nwalk;
    const uint32_t sub_fixed = fine ? slot % SPC : 0u;
    SweepWalk ahead;
    ahead.init_strided(walker, nwalkers, A);
    const uint32_t n_wg = walker_first < n_dense32 ? (n_dense32 - walker_first + nwalkers - 1) / nwalkers : 0u;
    const uint32_t nsteps = fine ? n_wg : n_wg * SPC;    // (the same for every wave of the workgroup)
    const uint32_t off_row = (uint32_t)(col * RB + g4 * 16);
    const char* const mask_base = (const char*)(A.mask + col);
    const char* const ts_base = has_ts ? (const char*)(A.ts + col) : (const char*)(A.mask + col);
    u64 f_item = 0;
    uint32_t f_sub = 0;
    bool f_valid = false;
    uint32_t stage_info = 0;                             // lane s: first item / 16 of the step in stage s, bit 31: consume it
    auto fetch = [&](uint32_t stage) __attribute__((always_inline)) {
        if (f_sub == 0) {
            f_valid = ahead.valid();
            if (f_valid) f_item = ahead.lc() * A.stride * DENSE_CH + sub_fixed * DENSEF_STEP;
            ahead.advance();
        }
        const u64 item = f_item + f_sub * DENSEF_STEP;
        f_sub = fine ? 0u : (f_sub + 1) & (SPC - 1);
        if ((uint32_t)lane == stage) stage_info = (uint32_t)(item >> 4) | (f_valid ? 0x80000000u : 0u);
        unsigned char* const dst = ring + stage * STG;
        if (item + DENSEF_STEP <= A.n) {                 // uniform; all steps but those at the end of the index
            const char* eb = (const char*)A.emb + item * RB + off_row;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                __builtin_amdgcn_global_load_lds((gptr)(eb + ks * 64), (lptr)(dst + ks * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((gptr)(mask_base + item * 4), (lptr)(dst + ROWS), 4, 0, 0);
            if constexpr (TS) __builtin_amdgcn_global_load_lds((gptr)(ts_base + item * 4), (lptr)(dst + ROWS + 256), 4, 0, 0);
        } else {                                         // items past the last one repeat it (discarded later by `item < n`)
            const u64 last = A.n - 1;
            u64 it = item + (u64)col;
            it = it < last ? it : last;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                __builtin_amdgcn_global_load_lds((gptr)((const char*)A.emb + it * RB + ks * 64 + g4 * 16), (lptr)(dst + ks * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((gptr)(A.mask + it), (lptr)(dst + ROWS), 4, 0, 0);
            if constexpr (TS) __builtin_amdgcn_global_load_lds((gptr)((has_ts ? A.ts : A.mask) + it), (lptr)(dst + ROWS + 256), 4, 0, 0);
        }
    };

    // products of quarter QT (four groups, KS K-steps each; the four chains are interleaved) of the tile `bb`
    auto products = [&](v4f (&R)[4], auto QT, const v4i (&bb)[KS]) __attribute__((always_inline)) {
        constexpr int qt = decltype(QT)::value;
        if constexpr (qt < NQT) {
#pragma unroll
            for (int i = 0; i < 4; ++i) R[i] = mfma_kstep<LINR_BF16>(q[4 * qt + i][0], bb[0], c[M == 8 ? (4 * qt + i) / 2 : 4 * qt + i]);
#pragma unroll
            for (int ks = 1; ks < KS; ++ks)
#pragma unroll
                for (int i = 0; i < 4; ++i) R[i] = mfma_kstep<LINR_BF16>(q[4 * qt + i][ks], bb[ks], R[i]);
        }
    };

    const uint32_t lds_fa = dense_lds_addr(s_fa), lds_fn = dense_lds_addr(s_fn), lds_low = dense_lds_addr(s_low);
    const uint32_t lds_thr = dense_lds_addr(s_thr), lds_flag = dense_lds_addr(s_flag);
    const uint32_t lds_t0 = dense_lds_addr(QS.t0 + (TS ? set0 : 0)), lds_t1 = dense_lds_addr(QS.t1 + (TS ? set0 : 0));
    const uint32_t lds_qkey = dense_lds_addr(qkey), lds_qql = dense_lds_addr(qql);

    using Q0 = std::integral_constant<int, 0>; using Q1 = std::integral_constant<int, 1>;
    using Q2 = std::integral_constant<int, 2>; using Q3 = std::integral_constant<int, 3>;
    // ---- a quarter (four groups) of a tile that fired, its accumulators H still in registers: the lane's values that
    //      are >= 0 are marked (m = 1: the sign bits of its 16 values, one instruction each; m = 8: the maxima of its two
    //      queries' eight values), and the lanes that have any finish their (query, item) pairs one per round
    auto quarter_hot = [&](const v4f (&H)[4], int qt, uint32_t mk, uint32_t ts, u64 item) __attribute__((always_inline)) {
        {
            uint32_t bm;
            float v0 = 0.0f, v1 = 0.0f;                  // m = 8: the values of the lane's two queries of this quarter
            if constexpr (M == 8) {
                v0 = fmaxf(fmaxf(H[0][0], H[0][1]), fmaxf(H[0][2], H[0][3]));
                v0 = fmaxf(fmaxf(v0, H[1][0]), H[1][1]); v0 = fmaxf(fmaxf(v0, H[1][2]), H[1][3]);
                v1 = fmaxf(fmaxf(H[2][0], H[2][1]), fmaxf(H[2][2], H[2][3]));
                v1 = fmaxf(fmaxf(v1, H[3][0]), H[3][1]); v1 = fmaxf(fmaxf(v1, H[3][2]), H[3][3]);
                bm = (v0 >= 0.0f ? 1u : 0u) | (v1 >= 0.0f ? 2u : 0u);
                if (any_free) bm = 3u;
            } else {
                uint32_t lt = 0;                         // bit a: value a (group a / 4 of the quarter, query row 4 g4 + a % 4) is negative
#pragma unroll
                for (int a = 15; a >= 0; --a)
                    lt = __builtin_amdgcn_alignbit(lt, (uint32_t)__float_as_int(H[a >> 2][a & 3]), 31);  // (lt << 1) | sign
                bm = ~lt & 0xFFFFu;
                if (any_free) bm = 0xFFFFu;              // queries without a bound take every item: all pairs are looked at
            }
            if (item >= A.n) bm = 0u;                    // (items past the end of the index repeat the last one)
            while (wave_any(bm != 0u)) {
                const bool act = bm != 0u;
                const uint32_t a = (uint32_t)(__ffs((int)bm) - 1) & 15u;
                bm &= bm - 1u;
                const uint32_t ql = M == 8 ? (uint32_t)(qt * 8) + (a & 1u) * 4u + (uint32_t)g4
                                           : (uint32_t)(qt * 4) * 16u + (a >> 2) * 16u + 4u * (uint32_t)g4 + (a & 3u);
                uint32_t fa, fn, flag, t0 = 0u, t1 = 0xFFFFFFFFu;
                float low, thr;
                if constexpr (TS)
                    asm volatile("ds_read_b32 %0, %7\n\tds_read_b32 %1, %8\n\tds_read_b32 %2, %9\n\tds_read_b32 %3, %10\n\t"
                                 "ds_read_u8 %4, %11\n\tds_read_b32 %5, %12\n\tds_read_b32 %6, %13\n\ts_waitcnt lgkmcnt(0)"
                                 : "=&v"(fa), "=&v"(fn), "=&v"(low), "=&v"(thr), "=&v"(flag), "=&v"(t0), "=&v"(t1)
                                 : "v"(lds_fa + 4u * ql), "v"(lds_fn + 4u * ql), "v"(lds_low + 4u * ql), "v"(lds_thr + 4u * ql),
                                   "v"(lds_flag + ql), "v"(lds_t0 + 4u * ql), "v"(lds_t1 + 4u * ql) : "memory");
                else
                    asm volatile("ds_read_b32 %0, %5\n\tds_read_b32 %1, %6\n\tds_read_b32 %2, %7\n\tds_read_b32 %3, %8\n\t"
                                 "ds_read_u8 %4, %9\n\ts_waitcnt lgkmcnt(0)"
                                 : "=&v"(fa), "=&v"(fn), "=&v"(low), "=&v"(thr), "=&v"(flag)
                                 : "v"(lds_fa + 4u * ql), "v"(lds_fn + 4u * ql), "v"(lds_low + 4u * ql), "v"(lds_thr + 4u * ql),
                                   "v"(lds_flag + ql) : "memory");
                bool ok = act && (mk & fn) == fa;
                if constexpr (TS) {
                    if (has_ts) ok = ok && ts >= t0 && ts <= t1;
                }
                // (a round without any survivor of the filter ends here, before the value is selected and scored)
                if (!wave_any(ok)) continue;
                const bool a0 = (a & 1u) != 0u, a1 = (a & 2u) != 0u, a2 = (a & 4u) != 0u, a3 = (a & 8u) != 0u;
                // (the group first, then the row; every select written out and pinned -- as an indexed array the
                // compiler would place the accumulators in scratch memory, whose loads wait for the whole ring)
                int t0v = 0, t1v = 0, t2v = 0, t3v = 0;
                if constexpr (M == 1) {
                    int lo0 = __float_as_int(a2 ? H[1][0] : H[0][0]), hi0 = __float_as_int(a2 ? H[3][0] : H[2][0]);
                    pin(lo0); pin(hi0);
                    t0v = a3 ? hi0 : lo0; pin(t0v);
                    int lo1 = __float_as_int(a2 ? H[1][1] : H[0][1]), hi1 = __float_as_int(a2 ? H[3][1] : H[2][1]);
                    pin(lo1); pin(hi1);
                    t1v = a3 ? hi1 : lo1; pin(t1v);
                    int lo2 = __float_as_int(a2 ? H[1][2] : H[0][2]), hi2 = __float_as_int(a2 ? H[3][2] : H[2][2]);
                    pin(lo2); pin(hi2);
                    t2v = a3 ? hi2 : lo2; pin(t2v);
                    int lo3 = __float_as_int(a2 ? H[1][3] : H[0][3]), hi3 = __float_as_int(a2 ? H[3][3] : H[2][3]);
                    pin(lo3); pin(hi3);
                    t3v = a3 ? hi3 : lo3; pin(t3v);
                }
                const float hv = M == 8 ? (a0 ? v1 : v0) : __int_as_float(a1 ? (a0 ? t3v : t2v) : (a0 ? t1v : t0v));
                const float sv = hv + low;               // ranking value: the accumulator plus what it started from
                ok = ok && sv >= thr;
                if (ok && flag) ok = filter_pass(A.filters[s_qi[ql]], mk, has_ts, ts);
                const u64 okm = wave_ballot(ok);
                if (okm == 0ull) continue;
                const uint32_t nok = (uint32_t)__popcll(okm);
                const u64 key = ((u64)ord_f32(sv) << 32) | (u64)(uint32_t)~(uint32_t)item;
                if (queued + nok <= (uint32_t)DENSE_QCAP) {
                    const uint32_t pos = queued + __builtin_amdgcn_mbcnt_hi((uint32_t)(okm >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)okm, 0u));
                    if (ok)
                        asm volatile("ds_write_b64 %0, %1\n\tds_write_b8 %2, %3"
                                     :: "v"(lds_qkey + 8u * pos), "v"(key), "v"(lds_qql + pos), "v"(ql) : "memory");
                    queued += nok;
                } else {                                  // queue full (rare): straight to the segments
                    if (ok) {
                        const uint32_t p2 = atomicAdd(&cnt[ql], 1u);
                        if (p2 < A.cap) A.seg[((u64)slot * A.B + s_qi[ql]) * A.cap + p2] = key;
                        if (p2 + 1 + DENSE_SLACK > A.cap) need_compact = 1u;
                    }
                    direct = 1u;
                }
            }
        }
    };

    // ---- one step = one tile: fragments and side values read at once; products and maxima of all quarters, branch-free;
    //      ONE compare; if it fires, the quarters are told apart and handed to the slow path
    auto consume = [&](uint32_t stage) __attribute__((always_inline)) {
        const uint32_t info = __builtin_amdgcn_readlane(stage_info, stage);
        if ((info >> 31) == 0u) return;
        const u64 item0 = (u64)(info & 0x7FFFFFFFu) << 4;
        const uint32_t addr_a = ring_lds + stage * STG + (uint32_t)lane * 16u;
        const uint32_t addr_s = ring_lds + stage * STG + (uint32_t)ROWS + (uint32_t)col * 4u;
        v4i b[KS];
        uint32_t mk, ts = 0u;
        static_assert(KS == 4 || KS == 2, "rows of 256 or 128 bytes");
        if constexpr (KS == 4) {
            if constexpr (TS)
                asm volatile("ds_read_b128 %0, %6\n\tds_read_b128 %1, %6 offset:1024\n\tds_read_b128 %2, %6 offset:2048\n\t"
                             "ds_read_b128 %3, %6 offset:3072\n\tds_read_b32 %4, %7\n\tds_read_b32 %5, %7 offset:256\n\ts_waitcnt lgkmcnt(0)"
                             : "=&v"(b[0]), "=&v"(b[1]), "=&v"(b[2]), "=&v"(b[3]), "=&v"(mk), "=&v"(ts) : "v"(addr_a), "v"(addr_s) : "memory");
            else
                asm volatile("ds_read_b128 %0, %5\n\tds_read_b128 %1, %5 offset:1024\n\tds_read_b128 %2, %5 offset:2048\n\t"
                             "ds_read_b128 %3, %5 offset:3072\n\tds_read_b32 %4, %6\n\ts_waitcnt lgkmcnt(0)"
                             : "=&v"(b[0]), "=&v"(b[1]), "=&v"(b[2]), "=&v"(b[3]), "=&v"(mk) : "v"(addr_a), "v"(addr_s) : "memory");
        } else {
            if constexpr (TS)
                asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %4 offset:1024\n\tds_read_b32 %2, %5\n\t"
                             "ds_read_b32 %3, %5 offset:256\n\ts_waitcnt lgkmcnt(0)"
                             : "=&v"(b[0]), "=&v"(b[1]), "=&v"(mk), "=&v"(ts) : "v"(addr_a), "v"(addr_s) : "memory");
            else
                asm volatile("ds_read_b128 %0, %3\n\tds_read_b128 %1, %3 offset:1024\n\tds_read_b32 %2, %4\n\ts_waitcnt lgkmcnt(0)"
                             : "=&v"(b[0]), "=&v"(b[1]), "=&v"(mk) : "v"(addr_a), "v"(addr_s) : "memory");
        }
        // per quarter: products (four interleaved chains of KS), 8 v_max3_f32 over its 16 accumulators, one compare; a
        // quarter that fires is finished at once, while its accumulators are still in registers
        const u64 item = item0 + (uint32_t)col;
        auto quarter = [&](auto QT) __attribute__((always_inline)) {
            constexpr int qt = decltype(QT)::value;
            if constexpr (qt < NQT) {
                v4f X[4];
                products(X, QT, b);
                float m = fmaxf(fmaxf(X[0][0], X[0][1]), fmaxf(X[0][2], X[0][3]));
#pragma unroll
                for (int i = 1; i < 4; ++i) {
                    m = fmaxf(fmaxf(m, X[i][0]), X[i][1]);
                    m = fmaxf(fmaxf(m, X[i][2]), X[i][3]);
                }
                if (__builtin_expect(any_free || wave_any(m >= 0.0f), 0)) quarter_hot(X, qt, mk, ts, item);
            }
        };
        quarter(Q0{}); quarter(Q1{}); quarter(Q2{}); quarter(Q3{});
        // the one place where this wave touches global memory besides its direct loads (each of these waits for
        // everything in flight: they are kept rare)
        ++since_refresh;
        if (queued >= (uint32_t)(DENSE_QCAP / 2) || wave_any(direct != 0u)) {
            flush_queue();
            direct = 0u;
            if (wave_any(need_compact != 0u)) {
                compact_full_segments<DENSE_SLACK>(A, qs, slot, 0, NQW, scratch_all[wib], lane, s_qi);
                need_compact = 0u;
                since_refresh = 1u << 30;                // bounds moved
                __builtin_amdgcn_s_waitcnt(DENSE_WAIT_VM(0));
            }
        }
        if (since_refresh >= 2048u) {
            load_bounds();
            since_refresh = 0;
            __builtin_amdgcn_s_waitcnt(DENSE_WAIT_VM(0));
        }
    };

    // The loop over the steps (see linr_kernels_dense.hip): counted wait, refill of the stage consumed last, consume.
    if (nsteps) {
        for (uint32_t sg = 0; sg + 1 < (uint32_t)NST; ++sg) fetch(sg);
        uint32_t st = 0;
        for (uint32_t i = 0; i < nsteps; ++i) {
            __builtin_amdgcn_s_waitcnt(DENSE_WAIT_VM((NST - 2) * DMA));
            fetch(st == 0 ? (uint32_t)NST - 1 : st - 1);
            if (nqt > 0) consume(st);
            st = st + 1 == (uint32_t)NST ? 0u : st + 1;
            if (nsets > 1 && (i & 31u) == 31u) __builtin_amdgcn_s_barrier();
        }
        __builtin_amdgcn_s_waitcnt(DENSE_WAIT_VM(0));      // nothing may still be on its way to LDS when the wave ends
    }
    if (nqt > 0) {
        flush_queue();
        own_stores_done();
        flush_segments(A, qs, slot, 0, NQW, lane, scratch_all[wib], s_qi);
    }
}

// ---------------------------------------------------------------------------
// host side: which variants exist, their occupancy, their launch
// ---------------------------------------------------------------------------
template <typename K>
static hipError_t densef_act(K kern, int what, uint32_t grid, hipStream_t s, const linr_scan_args* a, int* blocks_per_cu)
{
    if (what == 0) return hipSuccess;
    if (what == 1) return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, kern, 64 * WPB, 0);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * WPB), 0, s, *a);
    return hipGetLastError();
}

#define DENSEF_CASE(KS_, NG_, M_)                                                                                  \
    if (ks == KS_ && ng == NG_ && m == M_)                                                                         \
        return ts ? densef_act(scan_kernel_dense_bf16<KS_, NG_, M_, true>, what, grid, s, a, blocks_per_cu)        \
                  : densef_act(scan_kernel_dense_bf16<KS_, NG_, M_, false>, what, grid, s, a, blocks_per_cu);

// what: 0 = does the variant exist, 1 = workgroups per compute unit, 2 = launch
hipError_t linr_dense_bf16_dispatch(int what, uint32_t ks, uint32_t ng, uint32_t m, bool ts, uint32_t grid, hipStream_t s,
                                    const linr_scan_args* a, int* blocks_per_cu)
{
    DENSEF_CASE(4, 8, 1) DENSEF_CASE(4, 4, 1) DENSEF_CASE(2, 16, 8)
    return hipErrorInvalidDeviceFunction;
}
