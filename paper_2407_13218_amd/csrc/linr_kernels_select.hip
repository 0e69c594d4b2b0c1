// HIP kernels (gfx950 / CDNA4) of the large-K selection by bit matching (linr_select_bits).
#include "linr_device.h"

// ---------------------------------------------------------------------------
// large-K selection by bit matching (LiNR Sec. 3.2: the quantised module on its own when K is large; the notification
// use case of Sec. 5.3).  The number of differing bits takes k_bits + 1 values only, so the K best feasible items --
// ties to the lower id -- follow from counting: pass 1 counts, per segment of 16384 or 65536 items and per query, how many
// feasible items differ in 0, 1, 2, ... bits; a small kernel finds the cut (every item below `t_diff` differing bits,
// and the first `need_eq` items, by id, with exactly `t_diff`) and turns the segments' counts into output offsets;
// pass 2 recomputes the counts of differing bits and writes the selected ids, in ascending id order.
// ---------------------------------------------------------------------------
#define LINR_SELECT_TILE 1024          // items per workgroup step: 256 lanes x 4 neighbours

// one query's filter in the compact form the scans use: (mask & care) == must, an unsigned window test for the
// timestamp, and a flag for "any of" groups (checked with the full rule, only where the rest passed)
struct SelectFilter {
    uint32_t care, must, t0, span; bool any;
    // has_ts: the index has a timestamp column (without one, windows are not evaluated, not even empty ones)
    __device__ __forceinline__ void set(const linr_filter& F, uint32_t dead_bit, bool has_ts)
    {
        const uint32_t none = F.none_bits | dead_bit;
        const bool impossible = (F.all_bits & none) != 0u || (has_ts && F.ts_min > F.ts_max);
        must = impossible ? 0xFFFFFFFFu : F.all_bits;
        care = impossible ? 0u : (F.all_bits | none);
        t0 = F.ts_min; span = F.ts_max - F.ts_min;
        any = F.n_any != 0u && !impossible;
    }
};

#define LINR_SELECT_QB 8               // queries one workgroup of the counting pass serves from one read of its items

template <int W, bool TS>
struct SelectTile {
    uint32_t mk[4], tv[4];             // the lane's four neighbouring items: masks, timestamps, codes
    u64 x[4][W];
    // with_mask == false (uniform): no query looks at the attributes, the mask column is not read
    __device__ __forceinline__ void load(const linr_select_args& A, u64 i0, bool with_mask = true)
    {
        if (i0 + 4 <= A.n) {
            mk[0] = mk[1] = mk[2] = mk[3] = 0u;
            if (with_mask) {
                const v4i m4 = __builtin_nontemporal_load((const v4i*)(A.mask + i0));
                mk[0] = (uint32_t)m4[0]; mk[1] = (uint32_t)m4[1]; mk[2] = (uint32_t)m4[2]; mk[3] = (uint32_t)m4[3];
            }
            if (TS) {
                const v4i t4 = __builtin_nontemporal_load((const v4i*)(A.ts + i0));
                tv[0] = (uint32_t)t4[0]; tv[1] = (uint32_t)t4[1]; tv[2] = (uint32_t)t4[2]; tv[3] = (uint32_t)t4[3];
            }
            const v4i* src = (const v4i*)(A.bits + i0 * W);
#pragma unroll
            for (int j = 0; j < 2 * W; ++j) {                 // 32 W contiguous bytes: two words per load
                // (codes of two words and more: a lane's loads touch every 64-byte sector 2 to 4 times in a row, which
                // only an allocating load lets the first-level cache serve; measured on 15.5 M x 512-bit codes)
                const v4i c = W >= 2 ? src[j] : __builtin_nontemporal_load(src + j);
                const u64 lo = (u64)(uint32_t)c[0] | ((u64)(uint32_t)c[1] << 32), hi = (u64)(uint32_t)c[2] | ((u64)(uint32_t)c[3] << 32);
                x[(2 * j) / W][(2 * j) % W] = lo;
                x[(2 * j + 1) / W][(2 * j + 1) % W] = hi;
            }
        } else {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool in = i0 + r < A.n;
                const u64 ic = in ? i0 + r : A.n - 1;
                mk[r] = in && with_mask ? A.mask[ic] : 0u;
                tv[r] = TS ? A.ts[ic] : 0u;
#pragma unroll
                for (int w = 0; w < W; ++w) x[r][w] = A.bits[ic * W + w];
            }
        }
        if (!TS) {
#pragma unroll
            for (int r = 0; r < 4; ++r) tv[r] = 0u;
        }
    }
    // differing bits of the four items for one query; 0xFFFFFFFF = infeasible / beyond the end
    __device__ __forceinline__ void eval(const linr_select_args& A, const linr_filter* F, const SelectFilter& C, const u64* q, u64 i0,
                                         uint32_t (&diff)[4]) const
    {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            uint32_t d = 0;
#pragma unroll
            for (int w = 0; w < W; ++w) d += (uint32_t)__popcll(x[r][w] ^ q[w]);
            bool ok = (i0 + r < A.n) & ((mk[r] & C.care) == C.must);
            if (TS) ok = ok & (tv[r] - C.t0 <= C.span);
            diff[r] = ok ? d : 0xFFFFFFFFu;
        }
        if (C.any) {                                          // (uniform)
            const linr_filter f = *F;
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (diff[r] != 0xFFFFFFFFu && !filter_pass(f, mk[r], TS, tv[r])) diff[r] = 0xFFFFFFFFu;
        }
    }
};

// pass 1: grid (segments, groups of up to 8 queries): every item of the segment is read once and compared with each
// query of the group.  seg_hist[b][segment][bins], hist[b][bins] (zeroed by the caller); with `dcache` the count of
// differing bits of every (query, item) is kept, one byte each (255 = infeasible, or 255 bits and more), so that pass 2 reads 1 byte per item
template <int W, bool TS>
__global__ void __launch_bounds__(256) select_hist_kernel(linr_select_args A)
{
    constexpr int HB = 64 * W + 4;
    __shared__ uint32_t h[LINR_SELECT_QB][4][HB];    // four copies per query (lane % 4): match counts cluster
    __shared__ SelectFilter Cs[LINR_SELECT_QB];
    __shared__ u64 qs[LINR_SELECT_QB][W];
    __shared__ uint32_t s_need_mask;
    const uint32_t b0 = blockIdx.y * LINR_SELECT_QB, seg = blockIdx.x, bins = A.k_bits + 1;
    const uint32_t nqb = A.B - b0 < (uint32_t)LINR_SELECT_QB ? A.B - b0 : (uint32_t)LINR_SELECT_QB;
    for (uint32_t j = threadIdx.x; j < LINR_SELECT_QB * 4 * HB; j += 256) (&h[0][0][0])[j] = 0u;
    if (threadIdx.x == 0) s_need_mask = 0u;
    __syncthreads();
    if (threadIdx.x < nqb) {
        SelectFilter c;
        c.set(A.filters[b0 + threadIdx.x], A.dead_bit, TS);
        Cs[threadIdx.x] = c;
        if (c.care != 0u || c.must != 0u || c.any) atomicOr(&s_need_mask, 1u);      // (must != 0 with care == 0: nothing passes)
        for (int w = 0; w < W; ++w) qs[threadIdx.x][w] = A.q_codes[(u64)(b0 + threadIdx.x) * W + w];
    }
    __syncthreads();
    const u64 lo = (u64)seg * A.seg_items;
    const u64 hi = lo + A.seg_items < A.n ? lo + A.seg_items : A.n;
    const u64 row = (u64)A.n_seg * A.seg_items;                      // bytes of one query's kept counts
    const bool with_mask = s_need_mask != 0u;         // a pass-all group (the notification use case) reads the codes only
    // one query's counts of a tile: infeasible items go to a spare slot behind the last bin, so that nothing branches
    uint32_t* mine = &h[0][threadIdx.x & 3][0];
    auto one_query = [&](const SelectTile<W, TS>& T, u64 i0, uint32_t qi, const SelectFilter& C, const u64* q) {
        uint32_t diff[4];
        T.eval(A, A.filters + b0 + qi, C, q, i0, diff);
        uint32_t packed = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            atomicAdd(&mine[qi * 4 * HB + (diff[r] < (uint32_t)(HB - 1) ? diff[r] : (uint32_t)(HB - 1))], 1u);
            packed |= (diff[r] < 255u ? diff[r] : 255u) << (8 * r);      // 255: infeasible, or (codes of more than 254 bits) 255 bits or more
        }
        // (the segments are whole tiles: the cache is padded to them)
        if (A.dcache) __builtin_nontemporal_store(packed, (uint32_t*)(A.dcache + (u64)(b0 + qi) * row + i0));
    };
    const SelectFilter C0 = Cs[0];
    u64 q0[W];
#pragma unroll
    for (int w = 0; w < W; ++w) q0[w] = qs[0][w];
    SelectTile<W, TS> T, N;
    if (lo < hi) N.load(A, lo + 4 * threadIdx.x, with_mask);
    for (u64 t0 = lo; t0 < hi; t0 += LINR_SELECT_TILE) {
        const u64 i0 = t0 + 4 * threadIdx.x;
        const bool more = t0 + LINR_SELECT_TILE < hi;
        // The tile is copied out of the registers its loads went to BEFORE the next tile's loads are issued: the one
        // wait for memory stands here, and the loop over the queries below has none (a wait inside it would also wait
        // for the store of the query before, a full round trip to memory per query).
        T = N;
        if (more) N.load(A, i0 + LINR_SELECT_TILE, with_mask);   // the next tile's loads are in flight meanwhile
        if (nqb == 1) one_query(T, i0, 0u, C0, q0);          // (its filter and code stay in registers)
        else
            for (uint32_t qi = 0; qi < nqb; ++qi) {
                u64 q[W];
#pragma unroll
                for (int w = 0; w < W; ++w) q[w] = qs[qi][w];
                one_query(T, i0, qi, Cs[qi], q);
            }
    }
    __syncthreads();
    for (uint32_t j = threadIdx.x; j < nqb * bins; j += 256) {
        const uint32_t qi = j / bins, d = j % bins;
        const uint32_t c = h[qi][0][d] + h[qi][1][d] + h[qi][2][d] + h[qi][3][d];
        A.seg_hist[((u64)(b0 + qi) * A.n_seg + seg) * bins + d] = c;
        if (c) atomicAdd(&A.hist[(u64)(b0 + qi) * LINR_SELECT_BINS + d], (unsigned long long)c);
    }
}

// the cut, and per segment the number of items below it and on it: grid (segments / 64, queries)
__global__ void __launch_bounds__(256) select_cut_kernel(linr_select_args A)
{
    __shared__ uint32_t s_t;
    __shared__ u64 H[LINR_SELECT_BINS];               // the query's counts, fetched by all lanes at once
    const uint32_t b = blockIdx.y, bins = A.k_bits + 1;
    for (uint32_t j = threadIdx.x; j < bins; j += 256) H[j] = A.hist[(u64)b * LINR_SELECT_BINS + j];
    __syncthreads();
    if (threadIdx.x == 0) {
        u64 cum = 0, need = 0, n_gt = 0;
        uint32_t t = 0xFFFFFFFFu, last = 0xFFFFFFFFu;
        for (uint32_t d = 0; d < bins; ++d) {
            if (H[d] == 0) continue;
            last = d;
            if (cum + H[d] >= A.K) { t = d; n_gt = cum; need = A.K - cum; break; }
            cum += H[d];
        }
        if (t == 0xFFFFFFFFu && last != 0xFFFFFFFFu) {        // fewer than K feasible items: all of them
            t = last; n_gt = cum - H[last]; need = H[last];
        }
        s_t = t;
        if (blockIdx.x == 0) {
            linr_select_cut c;
            c.t_diff = t; c.need_eq = need;
            A.cut[b] = c;
            A.out_counts[b] = t == 0xFFFFFFFFu ? 0ull : n_gt + need;
            A.out_thresholds[b] = t == 0xFFFFFFFFu ? -1 : (int32_t)(A.k_bits - t);
        }
    }
    __syncthreads();
    // a wave per segment: its lanes read the segment's counts side by side
    const uint32_t t = s_t, lane = threadIdx.x & 63;
    for (uint32_t seg = blockIdx.x * 64 + (threadIdx.x >> 6); seg < A.n_seg && seg < (blockIdx.x + 1) * 64; seg += 4) {
        uint32_t g = 0, e = 0;
        if (t != 0xFFFFFFFFu) {
            const uint32_t* row = A.seg_hist + ((u64)b * A.n_seg + seg) * bins;
            for (uint32_t d = lane; d <= t; d += 64) {
                const uint32_t c = row[d];
                if (d < t) g += c; else e = c;
            }
        }
#pragma unroll
        for (int st = 32; st >= 1; st >>= 1) { g += __shfl_xor(g, st); e += __shfl_xor(e, st); }
        if (lane == 0) { A.gt_base[(u64)b * A.n_seg + seg] = g; A.eq_base[(u64)b * A.n_seg + seg] = e; }
    }
}

// the segments' counts -> output offsets (exclusive prefix sums, in place): one workgroup of 1024 lanes per query
__global__ void __launch_bounds__(1024) select_scan_kernel(linr_select_args A)
{
    __shared__ u64 part_gt[1024], part_eq[1024];
    const uint32_t b = blockIdx.x;
    unsigned long long* G = A.gt_base + (u64)b * A.n_seg;
    unsigned long long* E = A.eq_base + (u64)b * A.n_seg;
    const uint32_t per = (A.n_seg + 1023u) / 1024u;
    const uint32_t s0 = threadIdx.x * per, s1 = s0 + per < A.n_seg ? s0 + per : A.n_seg;
    u64 g = 0, e = 0;
    for (uint32_t sgm = s0; sgm < s1; ++sgm) { g += G[sgm]; e += E[sgm]; }
    part_gt[threadIdx.x] = g; part_eq[threadIdx.x] = e;
    __syncthreads();
    for (uint32_t st = 1; st < 1024; st <<= 1) {              // inclusive scan of the 1024 partial sums
        const u64 ag = threadIdx.x >= st ? part_gt[threadIdx.x - st] : 0ull, ae = threadIdx.x >= st ? part_eq[threadIdx.x - st] : 0ull;
        __syncthreads();
        part_gt[threadIdx.x] += ag; part_eq[threadIdx.x] += ae;
        __syncthreads();
    }
    u64 bg = part_gt[threadIdx.x] - g, be = part_eq[threadIdx.x] - e;      // exclusive
    for (uint32_t sgm = s0; sgm < s1; ++sgm) {
        const u64 cg = G[sgm], ce = E[sgm];
        G[sgm] = bg; E[sgm] = be;
        bg += cg; be += ce;
    }
}

// pass 2: grid (segments, queries); ids of the selected items to out_ids[b][position], positions ascending with the id
template <int W, bool TS>
__global__ void __launch_bounds__(256) select_write_kernel(linr_select_args A)
{
    __shared__ uint32_t wave_tot[4];
    const uint32_t b = blockIdx.y, seg = blockIdx.x;
    const linr_select_cut cut = A.cut[b];
    if (cut.t_diff == 0xFFFFFFFFu) return;
    if (A.dcache && cut.t_diff <= 254u) return;       // this query's cut is decided by the kept bytes (the other pass-2 kernel)
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    SelectFilter C;
    C.set(A.filters[b], A.dead_bit, TS);
    u64 q[W];
#pragma unroll
    for (int w = 0; w < W; ++w) q[w] = A.q_codes[(u64)b * W + w];
    u64 run_gt = A.gt_base[(u64)b * A.n_seg + seg], run_eq = A.eq_base[(u64)b * A.n_seg + seg];
    const u64 need = cut.need_eq;
    uint32_t* out = A.out_ids + (u64)b * A.K;
    const u64 lo = (u64)seg * A.seg_items;
    const u64 hi = lo + A.seg_items < A.n ? lo + A.seg_items : A.n;
    for (u64 t0 = lo; t0 < hi; t0 += LINR_SELECT_TILE) {
        SelectTile<W, TS> T;
        const u64 i0 = t0 + 4 * threadIdx.x;
        T.load(A, i0);
        uint32_t diff[4];
        T.eval(A, A.filters + b, C, q, i0, diff);
        uint32_t cg = 0, ce = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) { cg += diff[r] < cut.t_diff ? 1u : 0u; ce += diff[r] == cut.t_diff ? 1u : 0u; }
        // exclusive scan over the 256 lanes of (ties << 16 | better): wave by shuffles, waves through LDS
        const uint32_t mine = (ce << 16) | cg;
        uint32_t inc = mine;
#pragma unroll
        for (int st = 1; st < 64; st <<= 1) {
            const uint32_t o = __shfl_up(inc, st);
            if (lane >= st) inc += o;
        }
        if (lane == 63) wave_tot[wib] = inc;
        __syncthreads();
        uint32_t before = inc - mine, total = 0;
#pragma unroll
        for (int v = 0; v < 4; ++v) { if (v < wib) before += wave_tot[v]; total += wave_tot[v]; }
        __syncthreads();
        u64 g_before = run_gt + (before & 0xFFFFu), e_before = run_eq + (before >> 16);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const bool better = diff[r] < cut.t_diff, tie = diff[r] == cut.t_diff;
            // (pos < K always when the codes are what the counting pass saw; an update that lands between the two passes
            // can break that, and must cost a wrong id at most, not a write past the output)
            const u64 pos = g_before + (e_before < need ? e_before : need);
            if ((better || (tie && e_before < need)) && pos < A.K) out[pos] = (uint32_t)(i0 + r) + A.id_base;
            g_before += better ? 1u : 0u; e_before += tie ? 1u : 0u;
        }
        run_gt += total & 0xFFFFu; run_eq += total >> 16;
    }
}


// pass 2 over the kept byte per item: 16 items per lane and step
__global__ void __launch_bounds__(256) select_write_cached_kernel(linr_select_args A)
{
    __shared__ uint32_t wave_tot[4];
    const uint32_t b = blockIdx.y, seg = blockIdx.x;
    const linr_select_cut cut = A.cut[b];
    if (cut.t_diff == 0xFFFFFFFFu) return;
    if (cut.t_diff > 254u) return;                    // (long codes) the kept bytes saturate at 255: the recomputing kernel serves this query
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    u64 run_gt = A.gt_base[(u64)b * A.n_seg + seg], run_eq = A.eq_base[(u64)b * A.n_seg + seg];
    const u64 need = cut.need_eq;
    uint32_t* out = A.out_ids + (u64)b * A.K;
    const uint8_t* dc = A.dcache + (u64)b * A.n_seg * A.seg_items;
    const u64 lo = (u64)seg * A.seg_items;
    const u64 hi = lo + A.seg_items < A.n ? lo + A.seg_items : A.n;
    for (u64 t0 = lo; t0 < hi; t0 += 16 * 256) {
        const u64 i0 = t0 + 16 * threadIdx.x;
        v4i raw = {-1, -1, -1, -1};
        if (i0 < hi) raw = __builtin_nontemporal_load((const v4i*)(dc + i0));
        if (i0 < hi && i0 + 16 > hi) {                // the index's last bytes: what lies beyond counts as infeasible
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (i0 + r >= hi) raw[r >> 2] |= (int)(0xFFu << (8 * (r & 3)));
        }
        // four bytes at a time: bit 7 of a byte of `lt` / `eq` says "fewer differing bits than the cut" / "as many"
        // (0xFF, infeasible, is neither: the cut is at most 254); then one bit per item of the lane
        uint32_t better = 0, tie = 0;
        const uint32_t t4 = cut.t_diff * 0x01010101u;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t w = (uint32_t)raw[j], x = w ^ t4;
            const uint32_t eq = ((((x & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | x) & 0x80808080u) ^ 0x80808080u;
            const uint32_t s7 = (w | 0x80808080u) - (t4 & 0x7F7F7F7Fu);
            const uint32_t lt = ((~w & t4) | (~x & ~s7)) & 0x80808080u;
            better |= ((((lt >> 7) & 0x01010101u) * 0x10204080u) >> 28) << (4 * j);
            tie |= ((((eq >> 7) & 0x01010101u) * 0x10204080u) >> 28) << (4 * j);
        }
        const uint32_t mine = ((uint32_t)__popc(tie) << 16) | (uint32_t)__popc(better);
        uint32_t inc = mine;
#pragma unroll
        for (int st = 1; st < 64; st <<= 1) {
            const uint32_t o = __shfl_up(inc, st);
            if (lane >= st) inc += o;
        }
        if (lane == 63) wave_tot[wib] = inc;
        __syncthreads();
        uint32_t before = inc - mine, total = 0;
#pragma unroll
        for (int v = 0; v < 4; ++v) { if (v < wib) before += wave_tot[v]; total += wave_tot[v]; }
        __syncthreads();
        u64 g_before = run_gt + (before & 0xFFFFu), e_before = run_eq + (before >> 16);
        uint32_t todo = better | tie;
        while (todo) {
            const int r = __builtin_ctz(todo);
            todo &= todo - 1u;
            const uint32_t below = (1u << r) - 1u;
            const u64 g = g_before + (uint32_t)__popc(better & below), e = e_before + (uint32_t)__popc(tie & below);
            const u64 pos = g + (e < need ? e : need);
            if ((((better >> r) & 1u) || e < need) && pos < A.K) out[pos] = (uint32_t)(i0 + r) + A.id_base;   // (pos < K: see the other write pass)
        }
        run_gt += total & 0xFFFFu; run_eq += total >> 16;
    }
}

template <int W>
static void select_launch(const linr_select_args& a, int pass, hipStream_t s)
{
    const dim3 grid(a.n_seg, a.B), block(256);
    if (pass == 0) {
        const dim3 grid1(a.n_seg, (a.B + LINR_SELECT_QB - 1) / LINR_SELECT_QB);
        if (a.ts) hipLaunchKernelGGL((select_hist_kernel<W, true>), grid1, block, 0, s, a);
        else hipLaunchKernelGGL((select_hist_kernel<W, false>), grid1, block, 0, s, a);
    } else {
        // with the kept byte per (query, item): one pass over those bytes.  Codes of more than 254 bits: a query whose cut
        // lies at 255 differing bits or beyond (rare: it keeps most of the items) is served by the recomputing kernel,
        // whose workgroups leave at once for every other query.
        if (a.dcache) hipLaunchKernelGGL(select_write_cached_kernel, grid, block, 0, s, a);
        if (!a.dcache || a.k_bits > 254) {
            if (a.ts) hipLaunchKernelGGL((select_write_kernel<W, true>), grid, block, 0, s, a);
            else hipLaunchKernelGGL((select_write_kernel<W, false>), grid, block, 0, s, a);
        }
    }
}

// large-K selection: counts, cut, ids.  `hist` must be zero.
hipError_t linr_launch_select(const linr_select_args& a, hipStream_t s)
{
    if (a.B == 0 || a.B > 65535u || a.n == 0 || a.K == 0 || a.k_bits == 0 || a.k_bits + 1 > LINR_SELECT_BINS ||
        a.seg_items == 0 || a.seg_items % 4096 != 0 || a.seg_items > 65536 ||
        a.n_seg != (uint32_t)((a.n + a.seg_items - 1) / a.seg_items) ||
        (a.words != 1 && a.words != 2 && a.words != 3 && a.words != 4 && a.words != 6 && a.words != 8) || a.k_bits > 64 * a.words ||
        (((uintptr_t)a.dcache) & 15u))
        return hipErrorInvalidValue;
    if ((((uintptr_t)a.bits) | ((uintptr_t)a.mask) | ((uintptr_t)a.ts)) & 15u) return hipErrorInvalidValue;
    for (int pass = 0; pass < 2; ++pass) {
        if (a.words == 1) select_launch<1>(a, pass, s);
        else if (a.words == 2) select_launch<2>(a, pass, s);
        else if (a.words == 3) select_launch<3>(a, pass, s);
        else if (a.words == 4) select_launch<4>(a, pass, s);
        else if (a.words == 6) select_launch<6>(a, pass, s);
        else select_launch<8>(a, pass, s);
        if (pass == 0) {
            hipLaunchKernelGGL(select_cut_kernel, dim3((a.n_seg + 63) / 64, a.B), dim3(256), 0, s, a);
            hipLaunchKernelGGL(select_scan_kernel, dim3(a.B), dim3(1024), 0, s, a);
        }
    }
    return hipGetLastError();
}

