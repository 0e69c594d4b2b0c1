// Scan kernel for large int8 batches (rows of exactly 64 bytes, m = 1): the fused masked matrix product of
// LiNR (arXiv 2407.13218) Sec. 6 "Custom filtering kernel" in the regime of Sec. 5.3.2 (batched queries, each
// with its own filter), where the pass is bound by the matrix cores and by instruction issue, not by HBM.
//
// What limits such a pass on gfx950: a 16x16x64 int8 product occupies a SIMD for 16 cycles, and every vector
// instruction issued next to it costs about 3.3 more (measured; matrix and vector instructions of one SIMD barely
// overlap).  So the loop below spends the minimum of vector work per product:
//   * queries are the ROW operand: after a product a lane holds 4 queries x ONE item.  Everything that belongs
//     to the item (its scale, its mask) is then one value per lane, and the running maximum over a quarter of a
//     wave's queries is one register per lane;
//   * the bound of each query enters through the accumulator input: acc = raw - T_q with T_q an integer lower
//     bound of the raw dot product a candidate of query q needs.  "Some query wants this item" is then a test of
//     max_q(acc) that does not depend on q: two v_max3 per product, one compare per 64 queries;
//   * per-row scales (ranking value raw * s_i): with any reference scale s_ref = 1 / rho (the index's typical one)
//     and T_q = floor(thr_q * rho), a candidate of query q at item i has raw >= thr_q / s_i >= T_q / u_i with
//     u_i = s_i * rho, i.e. raw - T_q >= T_q * g_i, g_i = 1 / u_i - 1.  For g_i >= 0 the right side is at least
//     T_min * g_i, for g_i < 0 at least T_max * g_i (T_min, T_max over the 64 queries tested together): a value
//     per item.  "max_q(raw - T_q) >= that" never misses a candidate, is exact for scales equal to s_ref and loose
//     only by (spread of the T_q) x |g_i|.  That spread is kept small by ORDERING the batch: a tiny kernel sorts
//     the queries by their current bounds before every sweep, a wave takes up to 256 neighbours of that order and
//     tests them in quarters of 64 with the quarter's own T_min / T_max (data with dense clusters is unforgiving
//     here: a test that is 10 % loose lets a query's whole cluster through);
//   * a wave keeps up to 16 query groups (256 queries, 64 registers of fragments + 64 of bounds) and the four
//     waves of a workgroup either split a batch of up to 1024 queries between them (every item is read from HBM
//     once per search for ANY batch size up to 1024; the other three waves find it in L2) or, for smaller
//     batches, walk different chunks;
//   * the loop over a tile is branch-free: products, maxima and compares of all quarters, then ONE branch.  A tile
//     that fired recomputes the products of the quarters concerned (the fragments are still in registers) and
//     narrows them to (query, item) pairs by the exact predicate and ranking value;
//   * every wave is autonomous: its items arrive through direct global -> LDS loads into a private ring of
//     steps (no staging registers, no workgroup barrier per step), consumed with hand-placed LDS reads; candidate
//     keys are queued in LDS and written out in bulk.
// The survivors' keys go to the same per-(slot, query) segments, bounds, sweeps and merges as in the other kernels.
#include "linr_dense.h"

template <int VK, int NG, bool TS>
__global__ void __launch_bounds__(64 * WPB, 2) scan_kernel_dense(linr_scan_args A)
{
    constexpr int NQW = NG * 16;                         // query positions per wave
    constexpr int NQT = NG / 4;                          // 64-query quarters per wave
    constexpr bool SCALED = (VK == LINR_VK_I8_SCALED);
    constexpr int STG = 2048 + 256 + (TS ? 256 : 0);     // bytes of a ring stage: rows of two tiles, masks + scales, timestamps
    constexpr int NST = TS ? 4 : 5;                      // ring stages per wave: NST - 1 steps in flight
    constexpr int DMA = TS ? 4 : 3;                      // direct loads per step (always this many)
    static_assert(NG % 4 == 0 && NG <= 16, "query groups per wave come in quarters of four");
    static_assert(DENSE_SCRATCH_WORDS >= 2 * NQW + 1 + 3 && DENSE_SCRATCH_WORDS >= 2 * DENSE_QCAP + DENSE_QCAP / 4 + 4, "scratch");

    __shared__ __attribute__((aligned(16))) unsigned char ring_all[WPB][NST * STG];
    __shared__ DenseQ<NQW, TS> QS;
    __shared__ uint32_t cnt_all[WPB][NQW];
    __shared__ __attribute__((aligned(8))) uint32_t scratch_all[WPB][DENSE_SCRATCH_WORDS];

    const int lane = threadIdx.x & 63, wib = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = lane & 15, g4 = lane >> 4;
    const uint32_t nsets = A.nsplit;                     // query sets per workgroup: 1, 2 or 4
    const uint32_t wps = WPB / nsets;                    // waves that share a query set and split the tiles of a chunk
    const uint32_t qset = (uint32_t)wib % nsets, tlane = (uint32_t)wib / nsets;
    const uint32_t slot = blockIdx.x * wps + tlane;      // this wave's private candidate segments
    // The batch's order (ascending bounds) is dealt to the sets in equal runs of a multiple of 64 positions.
    const uint32_t per_set = ((A.B + nsets - 1) / nsets + 63u) & ~63u;
    const uint32_t pos_first = qset * per_set;           // first position of the order this wave serves
    const uint32_t nq_mine = pos_first < A.B ? (A.B - pos_first < per_set ? A.B - pos_first : per_set) : 0u;
    const int nqt = (int)((nq_mine + 63) / 64);          // quarters of this wave that hold queries
    const bool has_ts = TS && A.ts != nullptr;
    uint32_t* const cnt = cnt_all[wib];
    u64* const qkey = (u64*)&scratch_all[wib][0];
    uint8_t* const qql = (uint8_t*)&scratch_all[wib][2 * DENSE_QCAP];
    const QSide qs = {cnt, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};   // (the shared helpers use cnt only)
    float* const s_thr = QS.thr + wib * NQW;
    int* const s_T = QS.T + wib * NQW;
    const uint32_t set0 = qset * NQW;                    // this set's part of the per-set arrays
    const uint32_t* const s_fa = QS.fa + set0;
    const uint32_t* const s_fn = QS.fn + set0;
    const uint8_t* const s_flag = QS.flag + set0;
    const uint16_t* const s_qi = QS.qi + set0;           // wave-local query number -> query index of the batch

    float rho = 1.0f;                                    // 1 / (reference row scale): any positive number is valid, a typical one is tight
    if constexpr (SCALED) {
        const float ref = A.scale_stats[3];              // 1 / (mean row scale) at load time
        if (ref > 0.0f && ref < 3.0e38f) rho = ref;
    }

    // ---- which queries: position p of the batch's order (the identity if no order is given) is wave-local query
    //      p - pos_first of its set.  The first wave of each set fills the set's arrays.
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
    // ---- query fragments (row operand): lane l supplies bytes [16 (l/16), +16) of query row l%16 of each group
    v4i q[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const uint32_t qi = s_qi[g * 16 + col];
        v4i z = {0, 0, 0, 0};
        if (qi < A.B) z = *(const v4i*)((const char*)A.Q + (u64)qi * 64 + g4 * 16);
        q[g] = z;
    }
    // The fragments must have arrived before the chunk loop: a wait for them at their first use inside it would be
    // repeated on every pass and, waiting for "all loads", would empty the ring of chunks in flight each time.
#pragma unroll
    for (int g = 0; g < NG; ++g) pin(q[g]);
    for (uint32_t ql = lane; ql < (uint32_t)NQW; ql += 64) cnt[ql] = 0;

    v4i c[NG];                                           // accumulator inputs: -T of the lane's four queries of each group
    float tmin_f[NQT], tmax_f[NQT];                      // per quarter: T_min lowered / T_max raised over its queries that have a bound
    float twmin = 0.0f, twmax = 0.0f;                    // the same over all quarters of the wave that hold queries
    // Bounds: every wave reads those of its queries into its own arrays and derives its accumulator inputs from them.
    auto load_bounds = [&]() __attribute__((always_inline)) {
        twmin = 3.0e38f;
        twmax = -3.0e38f;
#pragma unroll
        for (int r = 0; r < NQT; ++r) {                  // iteration r of the lanes covers exactly quarter r
            const uint32_t ql = (uint32_t)(r * 64 + lane);
            const uint32_t qi = s_qi[ql];
            float tf = SCALED ? INFINITY : __int_as_float(INT_MAX);
            int T = DENSE_BIG;                           // no query here: never a candidate
            int tmin = DENSE_BIG, tmax = -DENSE_BIG;
            if (qi < A.B) {
                const u64 t = aload64(A.tau + qi);
                const uint32_t hi = (uint32_t)(t >> 32);
                if constexpr (SCALED) {
                    tf = t ? unord_f32(hi) : -INFINITY;
                    T = tf > 0.0f ? dense_floor_to_int(lowered(tf) * rho) : -DENSE_BIG;     // (no usable bound: always a candidate)
                } else {
                    const int ti = t ? unord_i32(hi) : INT_MIN;
                    tf = __int_as_float(ti);
                    T = ti < -DENSE_BIG ? -DENSE_BIG : (ti > DENSE_BIG ? DENSE_BIG : ti);
                }
                if (T > -DENSE_BIG) { tmin = T; tmax = T; }     // (a query without a bound fires for every item by itself)
            }
            s_thr[ql] = tf;
            s_T[ql] = T;
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) { tmin = min(tmin, __shfl_xor(tmin, o)); tmax = max(tmax, __shfl_xor(tmax, o)); }
            // lowered / raised by 2^-11 relative (rounding of g_i and of the products)
            const bool bounded = tmin <= tmax;
            tmin_f[r] = bounded ? (float)tmin * 0.99951f : 0.0f;
            tmax_f[r] = bounded ? (float)tmax * 1.00049f : 0.0f;
            if (wave_any(qi < A.B)) { twmin = fminf(twmin, tmin_f[r]); twmax = fmaxf(twmax, tmax_f[r]); }
        }
        wave_sync();
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const v4i t4 = *(const v4i*)&s_T[g * 16 + 4 * g4];
            c[g] = (v4i){-t4[0], -t4[1], -t4[2], -t4[3]};
        }
    };
    load_bounds();

    uint32_t need_compact = 0u, direct = 0u;
    uint32_t since_refresh = 0;
    uint32_t queued = 0;                                 // keys in the queue (uniform)
    // Candidate keys wait in the wave's LDS queue and are written out in bulk (an ordinary memory operation returns
    // after all direct loads issued before it, so whatever waits for one empties the ring of chunks in flight).
    auto flush_queue = [&]() __attribute__((always_inline)) {
        wave_sync();
        const uint32_t nqd = queued;                     // (keys that found the queue full went straight to their segments)
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

    // ---- the wave's private ring of steps.  A step is DENSE_SUB = 32 items (two tiles): 2 KB of rows, their masks and
    //      row scales (one load: lanes 0 .. 31 fetch masks, lanes 32 .. 63 scales) and, if the index has them, their
    //      timestamps.  Nothing is shared between waves, so no workgroup barrier is needed per step: a wave waits on its
    //      own load counter only.  Waves that serve different query sets of the same slot fetch the same items, each for
    //      itself (the second to fourth fetch is an L2 hit; a barrier now and then keeps them close enough for that).
    typedef const __attribute__((address_space(1))) void* gptr;
    typedef __attribute__((address_space(3))) void* lptr;
    unsigned char* const ring = ring_all[wib];
    const uint32_t ring_lds = dense_lds_addr(ring);
    const uint32_t nwalk = gridDim.x * wps;              // walkers of the sweep: one per slot
    // A sweep with fewer chunks than slots (the first, small sweeps, where bounds are missing or weak and most pairs go
    // through the slow path) is dealt out by steps instead of chunks: SPC neighbouring slots share a walker and each
    // takes one step of every chunk it visits, so SPC times as many waves have work.
    constexpr uint32_t SPC = DENSE_CH / DENSE_SUB;       // steps per chunk
    const uint32_t n_dense32 = (uint32_t)A.n_dense, slot_first = blockIdx.x * wps;
    const bool fine = nwalk % SPC == 0u && n_dense32 < nwalk;
    const uint32_t walker = fine ? slot / SPC : slot, walker_first = fine ? slot_first / SPC : slot_first;
    const uint32_t nwalkers = fine ? nwalk / SPC : nwalk;
    const uint32_t sub_fixed = fine ? slot % SPC : 0u;
    SweepWalk ahead;
    ahead.init_strided(walker, nwalkers, A);
    // every wave of a workgroup runs the step count of the workgroup's first slot (the largest); steps past the end of
    // a wave's own walk fetch its last chunk once more and consume nothing
    const uint32_t n_wg = walker_first < n_dense32 ? (n_dense32 - walker_first + nwalkers - 1) / nwalkers : 0u;
    const uint32_t nsteps = fine ? n_wg : n_wg * SPC;
    // what this lane fetches, relative to the first item of a step (the same for every step)
    const uint32_t off_row = (uint32_t)(col * 64 + g4 * 16);
    const uint32_t side_lane = (uint32_t)lane & 31u;
    const char* const side_base = (SCALED && lane >= 32) ? (const char*)(A.row_scale + side_lane) : (const char*)(A.mask + side_lane);
    const char* const ts_base = has_ts ? (const char*)(A.ts + side_lane) : (const char*)(A.mask + side_lane);
    u64 f_item = 0;                                      // first item of the chunk being fetched
    uint32_t f_sub = 0;                                  // its next step
    bool f_valid = false;                                // (false: past the end of this wave's walk)
    uint32_t stage_info = 0;                             // lane s: first item / 32 of the step in stage s, bit 31: consume it
    auto fetch = [&](uint32_t stage) __attribute__((always_inline)) {
        if (f_sub == 0) {
            f_valid = ahead.valid();
            if (f_valid) f_item = ahead.lc() * A.stride * DENSE_CH + sub_fixed * DENSE_SUB;
            ahead.advance();
        }
        const u64 item = f_item + f_sub * DENSE_SUB;
        f_sub = fine ? 0u : (f_sub + 1) & (SPC - 1);
        if ((uint32_t)lane == stage) stage_info = (uint32_t)(item >> 5) | (f_valid ? 0x80000000u : 0u);
        unsigned char* const dst = ring + stage * STG;
        if (item + DENSE_SUB <= A.n) {                   // uniform; all steps but those at the end of the index
            const char* eb = (const char*)A.emb + item * 64 + off_row;
            __builtin_amdgcn_global_load_lds((gptr)eb, (lptr)dst, 16, 0, 0);
            __builtin_amdgcn_global_load_lds((gptr)(eb + 1024), (lptr)(dst + 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((gptr)(side_base + item * 4), (lptr)(dst + 2048), 4, 0, 0);
            if constexpr (TS) __builtin_amdgcn_global_load_lds((gptr)(ts_base + item * 4), (lptr)(dst + 2304), 4, 0, 0);
        } else {                                         // items past the last one repeat it (discarded later by `item < n`)
            const u64 last = A.n - 1;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                u64 it = item + (u64)(j * 16 + col);
                it = it < last ? it : last;
                __builtin_amdgcn_global_load_lds((gptr)((const char*)A.emb + it * 64 + g4 * 16), (lptr)(dst + j * 1024), 16, 0, 0);
            }
            u64 it = item + side_lane;
            it = it < last ? it : last;
            __builtin_amdgcn_global_load_lds((gptr)(side_base + (it - side_lane) * 4), (lptr)(dst + 2048), 4, 0, 0);
            if constexpr (TS) __builtin_amdgcn_global_load_lds((gptr)(ts_base + (it - side_lane) * 4), (lptr)(dst + 2304), 4, 0, 0);
        }
    };

    // What the slow path knows about the tile it works on (one item per lane).
    struct TileCtx {
        int dtest[NQT];         // per quarter, the integer right side of the first test: a pair can only matter if raw - T >= dtest
        uint32_t mk, ts;        // the item's mask and timestamp
        float sc;               // its row scale
        u64 item;               // its id
    };

    // products of quarter QT (four groups) of the tile whose item fragments are `bb`
    auto products = [&](v4i (&R)[4], auto QT, const v4i& bb) __attribute__((always_inline)) {
        constexpr int qt = decltype(QT)::value;
        if constexpr (qt < NQT) {
#pragma unroll
            for (int i = 0; i < 4; ++i) R[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(q[4 * qt + i], bb, c[4 * qt + i], 0, 0, 0);
        }
    };

    // LDS addresses of the per-query arrays this wave's slow path reads.  (It reads and writes LDS with hand-placed
    // instructions for the same reason as the ring is: an LDS access the compiler can see waits for every direct
    // load in flight, i.e. for the memory latency of the chunk requested last.)
    const uint32_t lds_fa = dense_lds_addr(s_fa), lds_fn = dense_lds_addr(s_fn), lds_T = dense_lds_addr(s_T);
    const uint32_t lds_thr = dense_lds_addr(s_thr), lds_flag = dense_lds_addr(s_flag);
    const uint32_t lds_t0 = dense_lds_addr(QS.t0 + (TS ? set0 : 0)), lds_t1 = dense_lds_addr(QS.t1 + (TS ? set0 : 0));
    const uint32_t lds_qkey = dense_lds_addr(qkey), lds_qql = dense_lds_addr(qql);

    using Q0 = std::integral_constant<int, 0>; using Q1 = std::integral_constant<int, 1>;
    using Q2 = std::integral_constant<int, 2>; using Q3 = std::integral_constant<int, 3>;
    // ---- A tile that fired (rare).  For each quarter in `fired`: its products are made again (the fragments are
    //      still in registers), every lane marks which of its 16 values raw - T pass the first test, and the lanes
    //      that have any finish their (query, item) pairs one per round -- all / none clauses, timestamp window,
    //      exact ranking value against the query's bound, any-of clauses -- and queue the keys of those that hold.
    auto tile_hot = [&](const v4i& b, const TileCtx& tc, uint32_t fired) __attribute__((always_inline)) {
        while (fired) {
            const int qt = __ffs((int)fired) - 1;
            fired &= fired - 1;
            v4i H[4];
            int dq = tc.dtest[0];
            if (qt == 0) products(H, Q0{}, b);
            if constexpr (NQT > 1) { if (qt == 1) { products(H, Q1{}, b); dq = tc.dtest[1]; } }
            if constexpr (NQT > 2) { if (qt == 2) { products(H, Q2{}, b); dq = tc.dtest[2]; } }
            if constexpr (NQT > 3) { if (qt == 3) { products(H, Q3{}, b); dq = tc.dtest[3]; } }
            uint32_t lt = 0;                             // bit a: value a (group a / 4 of the quarter, query row 4 g4 + a % 4) is below the test
#pragma unroll
            for (int a = 15; a >= 0; --a)
                lt = __builtin_amdgcn_alignbit(lt, (uint32_t)(H[a >> 2][a & 3] - dq), 31);      // (lt << 1) | sign
            uint32_t bm = ~lt & 0xFFFFu;
            if (tc.item >= A.n) bm = 0u;                 // (items past the end of the index repeat the last one)
            while (wave_any(bm != 0u)) {
                const bool act = bm != 0u;
                const uint32_t a = (uint32_t)(__ffs((int)bm) - 1) & 15u;
                bm &= bm - 1u;
                const uint32_t ql = (uint32_t)(qt * 4) * 16u + (a >> 2) * 16u + 4u * (uint32_t)g4 + (a & 3u);   // wave-local query of the pair
                uint32_t fa, fn, flag, t0 = 0u, t1 = 0xFFFFFFFFu;
                int T;
                float thr;
                if constexpr (TS)
                    asm volatile("ds_read_b32 %0, %7\n\tds_read_b32 %1, %8\n\tds_read_b32 %2, %9\n\tds_read_b32 %3, %10\n\t"
                                 "ds_read_u8 %4, %11\n\tds_read_b32 %5, %12\n\tds_read_b32 %6, %13\n\ts_waitcnt lgkmcnt(0)"
                                 : "=&v"(fa), "=&v"(fn), "=&v"(T), "=&v"(thr), "=&v"(flag), "=&v"(t0), "=&v"(t1)
                                 : "v"(lds_fa + 4u * ql), "v"(lds_fn + 4u * ql), "v"(lds_T + 4u * ql), "v"(lds_thr + 4u * ql),
                                   "v"(lds_flag + ql), "v"(lds_t0 + 4u * ql), "v"(lds_t1 + 4u * ql) : "memory");
                else
                    asm volatile("ds_read_b32 %0, %5\n\tds_read_b32 %1, %6\n\tds_read_b32 %2, %7\n\tds_read_b32 %3, %8\n\t"
                                 "ds_read_u8 %4, %9\n\ts_waitcnt lgkmcnt(0)"
                                 : "=&v"(fa), "=&v"(fn), "=&v"(T), "=&v"(thr), "=&v"(flag)
                                 : "v"(lds_fa + 4u * ql), "v"(lds_fn + 4u * ql), "v"(lds_T + 4u * ql), "v"(lds_thr + 4u * ql),
                                   "v"(lds_flag + ql) : "memory");
                bool ok = act && (tc.mk & fn) == fa;
                if constexpr (TS) {
                    if (has_ts) ok = ok && tc.ts >= t0 && tc.ts <= t1;
                }
                // most pairs that beat their bound fail their filter when the pass rate is low: a round without any
                // survivor of the filter ends here, before the value is selected and scored
                if (!wave_any(ok)) continue;
                // the lane's value a: a binary tree of selects over the 16 registers
                const bool a0 = (a & 1u) != 0u, a1 = (a & 2u) != 0u, a2 = (a & 4u) != 0u, a3 = (a & 8u) != 0u;
                // (written out value by value and pinned: as an indexed array the compiler would place it in scratch memory)
                int e0 = a0 ? H[0][1] : H[0][0], e1 = a0 ? H[0][3] : H[0][2], e2 = a0 ? H[1][1] : H[1][0], e3 = a0 ? H[1][3] : H[1][2];
                int e4 = a0 ? H[2][1] : H[2][0], e5 = a0 ? H[2][3] : H[2][2], e6 = a0 ? H[3][1] : H[3][0], e7 = a0 ? H[3][3] : H[3][2];
                pin(e0); pin(e1); pin(e2); pin(e3); pin(e4); pin(e5); pin(e6); pin(e7);
                int f0 = a1 ? e1 : e0, f1 = a1 ? e3 : e2, f2 = a1 ? e5 : e4, f3 = a1 ? e7 : e6;
                pin(f0); pin(f1); pin(f2); pin(f3);
                const int hv = a3 ? (a2 ? f3 : f2) : (a2 ? f1 : f0);
                const int raw = hv + T;                  // the accumulator input was -T exactly
                uint32_t hi;
                if constexpr (SCALED) {
                    const float sv = (float)raw * tc.sc;
                    ok = ok && sv >= thr;
                    hi = ord_f32(sv);
                } else {
                    ok = ok && raw >= __float_as_int(thr);
                    hi = ord_i32(raw);
                }
                if (ok && flag) ok = filter_pass(A.filters[s_qi[ql]], tc.mk, has_ts, tc.ts);
                const u64 okm = wave_ballot(ok);
                if (okm == 0ull) continue;
                const uint32_t nok = (uint32_t)__popcll(okm);
                const u64 key = ((u64)hi << 32) | (u64)(uint32_t)~(uint32_t)tc.item;
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

    // ---- one tile (16 items, one per lane and k-slice) against the wave's queries.  Branch-free over the quarters:
    //      products, 8 v_max3 over the 16 accumulators of a quarter; then ONE compare of the maximum over all quarters
    //      with the test value of the wave's whole range of bounds.  Only if that fires are the quarters' own (tighter)
    //      test values made and compared, and the quarters that still fire handed to the slow path.
    auto score_tile = [&](const v4i& b, uint32_t mk, float sc, uint32_t ts, u64 item) __attribute__((always_inline)) {
        // right side of the first test for this lane's item (see the header comment): min(g T_min, g T_max) - 3.  One
        // of the two is the valid side (0 * inf = NaN for a zero scale is dropped by the minimum); 2 of slack for the
        // rounding of g and of the products, 1 because the conversion rounds towards zero, which for a negative
        // value is upwards by less than 1.  Raw ranking: "max >= 0".
        float g = 0.0f;
        int dqw = 0;
        if constexpr (SCALED) {
            g = __builtin_amdgcn_rcpf(sc * rho) - 1.0f;
            dqw = (int)fminf(fminf(__builtin_fmaf(g, twmin, -3.0f), __builtin_fmaf(g, twmax, -3.0f)), 268435456.0f);
        }
        int mq[4] = {INT_MIN, INT_MIN, INT_MIN, INT_MIN};
        v4i X[4];
        auto quarter = [&](auto QT) __attribute__((always_inline)) {
            constexpr int qt = decltype(QT)::value;
            if constexpr (qt < NQT) {
                products(X, QT, b);
#pragma unroll
                for (int i = 0; i < 4; ++i) mq[qt] = dense_max_acc(mq[qt], X[i]);
            }
        };
        quarter(Q0{}); quarter(Q1{}); quarter(Q2{}); quarter(Q3{});
        const int m = max(max(mq[0], mq[1]), max(mq[2], mq[3]));
        if (__builtin_expect(wave_any(m >= dqw), 0)) {
            TileCtx tc;
            tc.mk = mk; tc.sc = sc; tc.ts = ts; tc.item = item;
            uint32_t fired = 0;
#pragma unroll
            for (int r = 0; r < NQT; ++r) {
                tc.dtest[r] = 0;
                if constexpr (SCALED)
                    tc.dtest[r] = (int)fminf(fminf(__builtin_fmaf(g, tmin_f[r], -3.0f), __builtin_fmaf(g, tmax_f[r], -3.0f)), 268435456.0f);
                fired |= wave_any(mq[r] >= tc.dtest[r]) ? (1u << r) : 0u;
            }
            if (fired != 0u) tile_hot(b, tc, fired);
        }
    };

    // ---- one step: both tiles' fragments and side values are read at once, then each tile is scored
    auto consume = [&](uint32_t stage) __attribute__((always_inline)) {
        const uint32_t info = __builtin_amdgcn_readlane(stage_info, stage);
        if ((info >> 31) == 0u) return;
        const u64 item0 = (u64)(info & 0x7FFFFFFFu) << 5;
        const uint32_t addr_a = ring_lds + stage * STG + (uint32_t)lane * 16u;
        const uint32_t addr_s = ring_lds + stage * STG + 2048u + (uint32_t)col * 4u;
        v4i b0, b1;
        uint32_t mk0, mk1, ts0 = 0u, ts1 = 0u;
        float sc0, sc1;
        if constexpr (TS)
            asm volatile("ds_read_b128 %0, %8\n\tds_read_b128 %1, %8 offset:1024\n\tds_read_b32 %2, %9\n\tds_read_b32 %3, %9 offset:64\n\t"
                         "ds_read_b32 %4, %9 offset:128\n\tds_read_b32 %5, %9 offset:192\n\tds_read_b32 %6, %9 offset:256\n\t"
                         "ds_read_b32 %7, %9 offset:320\n\ts_waitcnt lgkmcnt(0)"
                         : "=&v"(b0), "=&v"(b1), "=&v"(mk0), "=&v"(mk1), "=&v"(sc0), "=&v"(sc1), "=&v"(ts0), "=&v"(ts1)
                         : "v"(addr_a), "v"(addr_s) : "memory");
        else
            asm volatile("ds_read_b128 %0, %6\n\tds_read_b128 %1, %6 offset:1024\n\tds_read_b32 %2, %7\n\tds_read_b32 %3, %7 offset:64\n\t"
                         "ds_read_b32 %4, %7 offset:128\n\tds_read_b32 %5, %7 offset:192\n\ts_waitcnt lgkmcnt(0)"
                         : "=&v"(b0), "=&v"(b1), "=&v"(mk0), "=&v"(mk1), "=&v"(sc0), "=&v"(sc1)
                         : "v"(addr_a), "v"(addr_s) : "memory");
        score_tile(b0, mk0, sc0, ts0, item0 + (uint32_t)col);
        score_tile(b1, mk1, sc1, ts1, item0 + (uint32_t)(16 + col));
        // The one place where this wave touches global memory besides its direct loads: write the queue out once it is
        // half full, shrink segments that are nearly full, re-read the bounds now and then.  (Each of these waits for
        // everything in flight: they are kept rare.)
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
        if (since_refresh >= 1024u) {
            load_bounds();
            since_refresh = 0;
            __builtin_amdgcn_s_waitcnt(DENSE_WAIT_VM(0));
        }
    };

    // The loop over the steps.  Steps 0 .. NST - 2 are fetched ahead; iteration i waits until at most the loads of the
    // NST - 2 steps after it are outstanding (every step is exactly DMA loads and nothing else is in flight: whatever
    // else touches memory ends with a wait for all of it), refills the stage consumed one iteration ago with the step
    // NST - 1 ahead, and consumes its own stage.
    if (nsteps) {
        for (uint32_t sg = 0; sg + 1 < (uint32_t)NST; ++sg) fetch(sg);
        uint32_t st = 0;
        for (uint32_t i = 0; i < nsteps; ++i) {
            __builtin_amdgcn_s_waitcnt(DENSE_WAIT_VM((NST - 2) * DMA));
            fetch(st == 0 ? (uint32_t)NST - 1 : st - 1);
            if (nqt > 0) consume(st);
            st = st + 1 == (uint32_t)NST ? 0u : st + 1;
            if (nsets > 1 && (i & 15u) == 15u) __builtin_amdgcn_s_barrier();
        }
        // nothing of this wave may still be on its way to LDS when it ends
        __builtin_amdgcn_s_waitcnt(DENSE_WAIT_VM(0));
    }
    if (nqt > 0) {
        flush_queue();
        own_stores_done();
        flush_segments(A, qs, slot, 0, NQW, lane, scratch_all[wib], s_qi);
    }
}

// ---------------------------------------------------------------------------
// order[0 .. B) = the queries of a pass in ascending order of their current bounds (queries without one first), ties
// by query index: one workgroup, bitonic sort of (bound, index) pairs in LDS.  B <= 1024.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(1024) dense_order_kernel(const u64* tau, uint32_t B, uint32_t* order)
{
    __shared__ u64 key[1024];
    const uint32_t t = threadIdx.x;
    key[t] = t < B ? (((aload64(tau + t) >> 32) << 32) | t) : ~0ull;
    __syncthreads();
    for (uint32_t size = 2; size <= 1024; size <<= 1)
        for (uint32_t str = size >> 1; str > 0; str >>= 1) {
            const uint32_t o = t ^ str;
            if (o > t) {
                const u64 x = key[t], y = key[o];
                const bool asc = (t & size) == 0;
                if (asc ? (x > y) : (x < y)) { key[t] = y; key[o] = x; }
            }
            __syncthreads();
        }
    if (t < B) order[t] = (uint32_t)key[t];
}

hipError_t linr_launch_dense_order(const unsigned long long* tau, uint32_t B, uint32_t* order, hipStream_t s)
{
    if (B == 0 || B > 1024) return hipErrorInvalidValue;
    hipLaunchKernelGGL(dense_order_kernel, dim3(1), dim3(1024), 0, s, (const u64*)tau, B, order);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// host side: which variants exist, their occupancy, their launch
// ---------------------------------------------------------------------------
template <typename K>
static hipError_t dense_act(K kern, int what, uint32_t grid, hipStream_t s, const linr_scan_args* a, int* blocks_per_cu)
{
    if (what == 0) return hipSuccess;
    if (what == 1) return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, kern, 64 * WPB, 0);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * WPB), 0, s, *a);
    return hipGetLastError();
}

#define DENSE_CASE(VK_, NG_)                                                                                    \
    if (vk == VK_ && ng == NG_)                                                                                 \
        return ts ? dense_act(scan_kernel_dense<VK_, NG_, true>, what, grid, s, a, blocks_per_cu)               \
                  : dense_act(scan_kernel_dense<VK_, NG_, false>, what, grid, s, a, blocks_per_cu);

// what: 0 = does the variant exist, 1 = workgroups per compute unit, 2 = launch
hipError_t linr_dense_dispatch(int what, int vk, uint32_t ng, bool ts, uint32_t grid, hipStream_t s, const linr_scan_args* a,
                               int* blocks_per_cu)
{
    DENSE_CASE(LINR_VK_I8_SCALED, 16) DENSE_CASE(LINR_VK_I8_SCALED, 12) DENSE_CASE(LINR_VK_I8_SCALED, 8) DENSE_CASE(LINR_VK_I8_SCALED, 4)
    DENSE_CASE(LINR_VK_I8_RAW, 16)    DENSE_CASE(LINR_VK_I8_RAW, 12)    DENSE_CASE(LINR_VK_I8_RAW, 8)    DENSE_CASE(LINR_VK_I8_RAW, 4)
    return hipErrorInvalidDeviceFunction;
}
