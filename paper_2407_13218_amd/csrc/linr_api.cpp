// Host side of the C ABI declared in include/linr.h: index object, argument
// validation, launch planning and the enqueue sequence of one search.
// (LiNR, arXiv 2407.13218: Sec. 4.2 -- the served model is the item embeddings plus
// their filter attributes resident in GPU memory; Sec. 3.1 -- the search itself.)
#include "linr_internal.h"
#include <algorithm>
#include <cstdlib>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

static thread_local int g_last_hip = 0;
static linr_tuning g_tuning = {};                       // all zero: library defaults

#define HIP_TRY(expr)                                   \
    do {                                                \
        hipError_t e__ = (expr);                        \
        if (e__ != hipSuccess) { g_last_hip = (int)e__; return LINR_E_HIP; } \
    } while (0)

extern "C" const char* linr_strerror(int code)
{
    switch (code) {
    case LINR_OK: return "ok";
    case LINR_E_NULL: return "required pointer is NULL";
    case LINR_E_SHAPE: return "unsupported shape (d, m, B or alignment)";
    case LINR_E_DTYPE: return "element type mismatch";
    case LINR_E_K: return "k out of range";
    case LINR_E_CAPACITY: return "item count exceeds capacity";
    case LINR_E_NOT_LOADED: return "index holds no items";
    case LINR_E_WORKSPACE: return "workspace missing, misaligned or too small";
    case LINR_E_HIP: return "HIP runtime error";
    case LINR_E_FILTER: return "malformed filter";
    case LINR_E_STATE: return "index is not in the state the call needs";
    case LINR_E_TOO_LARGE: return "search needs more scratch memory than the allocation-free entry point holds";
    default: return "unknown error";
    }
}
extern "C" int linr_last_hip_error(void) { return g_last_hip; }

extern "C" int linr_set_tuning(const linr_tuning* t)
{
    if (!t) { memset(&g_tuning, 0, sizeof(g_tuning)); return LINR_OK; }
    if (t->sample_ratio && (t->sample_ratio < 2 || (t->sample_ratio & (t->sample_ratio - 1)))) return LINR_E_SHAPE;
    g_tuning = *t;
    return LINR_OK;
}

static uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }
static uint32_t elt_bytes(int dtype) { return dtype == LINR_F32 ? 4u : dtype == LINR_BF16 ? 2u : 1u; }

// code lengths the bit-matching kernels exist for: 1, 2, 3, 4, 6 or 8 words of 64 bits (up to 512 bits)
static bool bits_words_supported(uint32_t k_bits)
{
    const uint32_t w = (k_bits + 63) / 64;
    return k_bits != 0 && (w <= 4 || w == 6 || w == 8);
}

extern "C" int linr_index_create(linr_index** out, uint64_t capacity, uint32_t d, int dtype, int device)
{
    if (!out) return LINR_E_NULL;
    *out = nullptr;
    if (dtype != LINR_F32 && dtype != LINR_BF16 && dtype != LINR_I8 && dtype != LINR_BITS) return LINR_E_DTYPE;
    if (d == 0) return LINR_E_SHAPE;
    uint64_t rb = (uint64_t)d * elt_bytes(dtype);
    if (dtype == LINR_BITS) {                           // d = bits per code; a code is ceil(d / 64) words
        if (!bits_words_supported(d)) return LINR_E_SHAPE;
        rb = (uint64_t)((d + 63) / 64) * 8;
    } else if (rb % 16 != 0 || rb > 512) return LINR_E_SHAPE;
    if (capacity == 0 || capacity > 0xFFFFFFFEull) return LINR_E_CAPACITY;
    int ndev = 0;
    HIP_TRY(hipGetDeviceCount(&ndev));
    if (device < 0 || device >= ndev) return LINR_E_SHAPE;
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDeviceProperties(&prop, device));
    linr_index* ix = new (std::nothrow) linr_index();
    if (!ix) return LINR_E_HIP;
    memset(ix, 0, sizeof(*ix));
    ix->device = device; ix->dtype = dtype; ix->d = d; ix->row_bytes = (uint32_t)rb;
    ix->capacity = capacity; ix->num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 1;
    if (dtype == LINR_BITS) { ix->k_bits = d; ix->bits_words = (d + 63) / 64; }
    *out = ix;
    return LINR_OK;
}

// Host-side bookkeeping of live updates (Sec. 4 "Model Live Update").  `n` of the index is the published
// high-water mark: searches on other streams use it, so it only rises once the update that wrote the new slots
// has finished on the device; `n_pending` is the mark after the last enqueued update.
struct linr_update_state {
    std::mutex writer;          // one updater at a time (held for a whole upsert / delete call)
    std::mutex mu;              // the fields below and linr_index::n (held for a few loads and stores)
    uint64_t n_pending;
    hipEvent_t done;            // recorded behind the last enqueued update
    hipStream_t stream;         // ... on this stream
    bool pending;
    void* staging;              // device copy of an update batch (slots, and host-side rows / columns)
    void* host_staging;         // its pinned host image (filled by the caller's thread, copied asynchronously)
    uint64_t staging_bytes;
};

static void release_update_state(linr_index* ix)
{
    if (!ix->upd) return;
    if (ix->upd->pending) (void)hipEventSynchronize(ix->upd->done);
    (void)hipEventDestroy(ix->upd->done);
    if (ix->upd->staging) (void)hipFree(ix->upd->staging);
    if (ix->upd->host_staging) (void)hipHostFree(ix->upd->host_staging);
    delete ix->upd;
    ix->upd = nullptr;
    ix->dead_bit = 0;
}

static void release_columns(linr_index* ix)
{
    release_update_state(ix);
    if (ix->owned) {
        if (ix->emb) (void)hipFree((void*)ix->emb);
        if (ix->row_scale) (void)hipFree((void*)ix->row_scale);
        if (ix->mask) (void)hipFree((void*)ix->mask);
        if (ix->ts) (void)hipFree((void*)ix->ts);
    }
    if (ix->bits && ix->dtype != LINR_BITS) (void)hipFree(ix->bits);     // (a codes-only index keeps its codes in `emb`)
    if (ix->perm) (void)hipFree(ix->perm);
    if (ix->signs) (void)hipFree(ix->signs);
    ix->bits = nullptr; ix->perm = nullptr; ix->signs = nullptr;
    if (ix->dtype != LINR_BITS) { ix->k_bits = 0; ix->bits_words = 0; }
    if (ix->clause_values) (void)hipFree(ix->clause_values);
    if (ix->clause_counts) (void)hipFree(ix->clause_counts);
    ix->clause_values = nullptr; ix->clause_counts = nullptr; ix->n_clauses = 0; ix->clause_n = 0;
    if (ix->scale_stats) (void)hipFree(ix->scale_stats);
    if (ix->scale_code) (void)hipFree(ix->scale_code);
    ix->scale_stats = nullptr; ix->scale_code = nullptr;
    ix->emb = nullptr; ix->row_scale = nullptr; ix->mask = nullptr; ix->ts = nullptr;
    ix->owned = 0; ix->n = 0;
}

extern "C" int linr_index_destroy(linr_index* ix)
{
    if (!ix) return LINR_E_NULL;
    int dev = 0;
    bool have = hipGetDevice(&dev) == hipSuccess;
    if (have) (void)hipSetDevice(ix->device);
    release_columns(ix);
    if (have) (void)hipSetDevice(dev);
    delete ix;
    return LINR_OK;
}

// The index as a search enqueued on stream `st` may see it.  Without live updates: the index itself.  With them:
// a copy taken under the lock whose item count is the published high-water mark -- raised here if the last update
// has finished, or taken from that update directly when the search runs on the update's own stream (stream order
// then guarantees that the new slots are written before they are read; `same_stream_ok`).
static const linr_index* view_for(const linr_index* ix, hipStream_t st, bool same_stream_ok, linr_index* snap)
{
    if (!ix || !ix->upd) return ix;
    linr_index* mix = const_cast<linr_index*>(ix);      // index objects are heap objects of this library, never const
    linr_update_state* u = ix->upd;
    std::lock_guard<std::mutex> g(u->mu);
    if (u->pending && hipEventQuery(u->done) == hipSuccess) {
        mix->n = u->n_pending;
        u->pending = false;
    }
    *snap = *mix;
    if (u->pending && same_stream_ok && st == u->stream) snap->n = u->n_pending;
    return snap;
}

extern "C" int linr_index_info(const linr_index* ix, uint64_t* n, uint32_t* d, int* dtype, int* has_ts, int* has_row_scale)
{
    if (!ix) return LINR_E_NULL;
    linr_index snap;
    ix = view_for(ix, nullptr, false, &snap);
    if (n) *n = ix->n;
    if (d) *d = ix->d;
    if (dtype) *dtype = ix->dtype;
    if (has_ts) *has_ts = ix->ts != nullptr;
    if (has_row_scale) *has_row_scale = ix->row_scale != nullptr;
    return LINR_OK;
}

// library-owned columns are allocated for the whole capacity, so that live updates can add items in place
// (Sec. 4: columns pre-allocated larger than the initial index)
static int copy_column(const void** dst, const void* src, uint64_t bytes, uint64_t alloc_bytes, int from_host)
{
    void* p = nullptr;
    if (alloc_bytes < bytes) alloc_bytes = bytes;
    HIP_TRY(hipMalloc(&p, alloc_bytes ? alloc_bytes : 16));
    hipError_t e = hipMemcpy(p, src, bytes, from_host ? hipMemcpyHostToDevice : hipMemcpyDeviceToDevice);
    if (e != hipSuccess) { (void)hipFree(p); g_last_hip = (int)e; return LINR_E_HIP; }
    *dst = p;
    return LINR_OK;
}

static int load_common(linr_index* ix, int dtype, const void* emb, const float* row_scale, const uint32_t* mask,
                       const uint32_t* ts, uint64_t n, int src)
{
    if (!ix) return LINR_E_NULL;
    if (ix->dtype != dtype) return LINR_E_DTYPE;
    if (!emb || !mask) return LINR_E_NULL;
    if (n == 0 || n > ix->capacity) return LINR_E_CAPACITY;
    if (src != LINR_SRC_HOST && src != LINR_SRC_DEVICE_COPY && src != LINR_SRC_DEVICE_BORROW) return LINR_E_SHAPE;
    if (src == LINR_SRC_DEVICE_BORROW) {
        if (((uintptr_t)emb | (uintptr_t)mask | (uintptr_t)ts | (uintptr_t)row_scale) & 15u) return LINR_E_SHAPE;
    }
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipSetDevice(ix->device));
    release_columns(ix);
    int rc = LINR_OK;
    if (src == LINR_SRC_DEVICE_BORROW) {
        ix->emb = emb; ix->row_scale = row_scale; ix->mask = mask; ix->ts = ts; ix->owned = 0;
    } else {
        int fh = src == LINR_SRC_HOST;
        ix->owned = 1;
        const uint64_t cap = ix->capacity;
        rc = copy_column(&ix->emb, emb, n * ix->row_bytes, cap * ix->row_bytes, fh);
        if (rc == LINR_OK) rc = copy_column((const void**)&ix->mask, mask, n * 4, cap * 4, fh);
        if (rc == LINR_OK && ts) rc = copy_column((const void**)&ix->ts, ts, n * 4, cap * 4, fh);
        if (rc == LINR_OK && row_scale) rc = copy_column((const void**)&ix->row_scale, row_scale, n * 4, cap * 4, fh);
        if (rc != LINR_OK) release_columns(ix);
    }
    if (rc == LINR_OK && dtype == LINR_I8 && ix->row_scale) {
        // statistics of the row scales for the large-batch kernel's first test (Sec. 5.1: a quantised index
        // carries its scales); 4 floats of results followed by the reduction's scratch
        const uint64_t n_pad = align_up(n, 256);
        hipError_t e = hipMalloc((void**)&ix->scale_stats, (4 + 4 * LINR_SCALE_STAT_BLOCKS) * sizeof(float));
        if (e == hipSuccess) e = hipMalloc((void**)&ix->scale_code, n_pad);
        if (e == hipSuccess)
            e = linr_launch_scale_stats(ix->row_scale, n, n_pad, ix->scale_stats + 4, ix->scale_stats, ix->scale_code, nullptr);
        if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
        if (e != hipSuccess) { g_last_hip = (int)e; rc = LINR_E_HIP; release_columns(ix); }
    }
    ix->have_bit_freq = 0;
    if (rc == LINR_OK) {
        // how often each mask bit is set, from an evenly spaced sample of at most 2^24 items: what the planner of
        // linr_search_filtered estimates a filter's pass rate from (Sec. 3.1.2: masking or explicit pre-filtering)
        unsigned long long* dc = nullptr;
        unsigned long long hc[33];
        hipError_t e = hipMalloc((void**)&dc, sizeof(hc));
        if (e == hipSuccess) e = hipMemsetAsync(dc, 0, sizeof(hc), nullptr);
        if (e == hipSuccess) e = linr_launch_mask_bit_counts(ix->mask, n, (n + (1ull << 24) - 1) >> 24, dc, nullptr);
        if (e == hipSuccess) e = hipMemcpy(hc, dc, sizeof(hc), hipMemcpyDeviceToHost);
        if (dc) (void)hipFree(dc);
        if (e != hipSuccess) { g_last_hip = (int)e; rc = LINR_E_HIP; release_columns(ix); }
        else if (hc[32]) {
            for (int b = 0; b < 32; ++b) ix->bit_freq[b] = (float)((double)hc[b] / (double)hc[32]);
            ix->have_bit_freq = 1;
        }
    }
    if (rc == LINR_OK) ix->n = n;
    (void)hipSetDevice(dev);
    return rc;
}

extern "C" int linr_index_load_fp32(linr_index* ix, const float* emb, const uint32_t* mask, const uint32_t* ts, uint64_t n, int src)
{
    return load_common(ix, LINR_F32, emb, nullptr, mask, ts, n, src);
}
extern "C" int linr_index_load_bf16(linr_index* ix, const uint16_t* emb, const uint32_t* mask, const uint32_t* ts, uint64_t n, int src)
{
    return load_common(ix, LINR_BF16, emb, nullptr, mask, ts, n, src);
}
extern "C" int linr_index_load_int8(linr_index* ix, const int8_t* emb, const float* row_scale, const uint32_t* mask,
                                    const uint32_t* ts, uint64_t n, int src)
{
    return load_common(ix, LINR_I8, emb, row_scale, mask, ts, n, src);
}

// ---------------------------------------------------------------------------
// planning
// ---------------------------------------------------------------------------

// occupancy of each kernel variant, asked from the runtime once per process
static int cached_blocks_per_cu(const linr_index* ix, const linr_plan& p, uint32_t Bp, uint32_t m)
{
    static int cache[3][3][2][3][9][17][9][2];       // dtype, vk, generic, coop / wide, ks, qg, m, ts  (0 = unknown)
    static int cache_dyn = 0;                          // the LDS-streamed kernel depends on (B, m): not cached
    (void)cache_dyn;
    const int ts = ix->ts != nullptr;
    if (p.generic) return linr_scan_blocks_per_cu(p, ix->dtype, Bp, m, ts);
    if (p.dense) {
        static int dense_cache[3][17][2];
        int& dslot = dense_cache[p.vk][p.qg <= 16 ? p.qg : 0][ts];
        if (dslot == 0) { int v = linr_scan_blocks_per_cu(p, ix->dtype, Bp, m, ts); dslot = v > 0 ? v : -1; }
        return dslot > 0 ? dslot : 0;
    }
    if (p.bits) {
        static int bits_cache[3][5][9][2];
        int& bslot = bits_cache[p.bits <= 2 ? p.bits : 0][p.ks <= 4 ? p.ks : 0][p.qg <= 8 ? p.qg : 0][ts];
        if (bslot == 0) { int v = linr_scan_blocks_per_cu(p, ix->dtype, Bp, m, ts); bslot = v > 0 ? v : -1; }
        return bslot > 0 ? bslot : 0;
    }
    int& slot = cache[ix->dtype][p.vk][0][p.wide ? 2 : p.coop ? 1 : 0][p.ks][p.qg][m][ts];
    if (slot == 0) {
        int v = linr_scan_blocks_per_cu(p, ix->dtype, Bp, m, ts);
        slot = v > 0 ? v : -1;
    }
    return slot > 0 ? slot : 0;
}

// Choose kernel shape, grid and the sequence of threshold-seeding sweeps for a pass of
// at most B queries.  Returns LINR_OK or LINR_E_SHAPE.
static int make_plan(const linr_index* ix, uint32_t B, uint32_t m, uint32_t k, linr_plan* p)
{
    memset(p, 0, sizeof(*p));
    if (m == 0 || m > LINR_MAX_M) return LINR_E_SHAPE;
    const bool bits_mode = ix->dtype == LINR_BITS;
    p->vk = (ix->dtype == LINR_I8 || bits_mode) ? (ix->row_scale ? LINR_VK_I8_SCALED : LINR_VK_I8_RAW) : LINR_VK_FLOAT;
    uint32_t ks = (ix->row_bytes + 63) / 64;
    p->ks = ks <= 1 ? 1 : ks <= 2 ? 2 : ks <= 4 ? 4 : 8;
    p->tpc = 8 / p->ks;
    p->chunk_items = 16 * p->tpc;
    const uint32_t nsg = (B + 15) / 16;
    // smallest group count covering the batch for which a register-resident kernel exists,
    // else the largest existing one (the batch is then split over several waves per chunk)
    uint32_t qg = 0;
    if (!g_tuning.force_generic)
        for (uint32_t c = 1; c <= (g_tuning.max_qg ? g_tuning.max_qg : 16u); c <<= 1) {
            if (!linr_fast_variant_exists(ix->dtype, p->vk, p->ks, m, c)) continue;
            qg = c;
            if (c >= nsg) break;
        }
    // batches of more than two groups: workgroup-cooperative kernel, 4 waves x cq groups each
    uint32_t cq = 0;
    if (!g_tuning.force_generic && !g_tuning.no_coop && nsg > (g_tuning.coop_min_groups ? g_tuning.coop_min_groups : 8u))
        for (uint32_t c = 1; c <= 4; c <<= 1) {
            if (!linr_coop_variant_exists(ix->dtype, p->vk, p->ks, m, c)) continue;
            cq = c;
            if (c * LINR_WAVES_PER_BLOCK >= nsg) break;
        }
    // opt-in (tuning.wide_min_batch): cooperative kernel with 32x32 tiles for int8 rows of exactly 64, 128 or 256
    // bytes, 4 waves x qw groups of 32 queries.  Not the default: on the measured configurations it only matches
    // the 16x16-tile kernels (its loop is bound by instruction issue, not by the matrix pipe).
    uint32_t qw = 0;
    if (!g_tuning.force_generic && !g_tuning.no_coop && g_tuning.wide_min_batch && B >= g_tuning.wide_min_batch &&
        ix->row_bytes == p->ks * 64u && !ix->dead_bit)  // (its per-item scale codes are not kept up to date by updates)
        for (uint32_t c = 1; c <= 4; c <<= 1) {
            if (!linr_wide_variant_exists(ix->dtype, p->vk, p->ks, m, c)) continue;
            qw = c;
            if (c * LINR_WAVES_PER_BLOCK * 32 >= B) break;
        }
    // Large int8 batches on rows of exactly 64 bytes: queries as the row operand, bounds through the accumulator
    // input, up to 1024 queries per stream of the index (linr_kernels_dense.hip).  (Its reference row scale, the mean
    // at load time, only has to be positive to be valid, so live updates do not disturb it.)
    // (a tuning that asks for one of the other kernel families is honoured)
    const bool other_family = g_tuning.force_generic || g_tuning.no_coop || g_tuning.max_qg || g_tuning.coop_min_groups ||
                              g_tuning.wide_min_batch;
    const bool dense_common = !other_family && !g_tuning.no_dense && !bits_mode && m == 1 &&
                              B >= (g_tuning.dense_min_batch ? g_tuning.dense_min_batch : 65u);
    const bool dense_ok = dense_common && ix->dtype == LINR_I8 && ix->row_bytes == 64 && !(ix->row_scale && !ix->scale_stats);
    // the same design for bf16 rows of 256 bytes (linr_kernels_dense_bf16.hip): up to 8 groups per wave, 512 queries per stream
    const bool dense_bf16_ok = dense_common && ix->dtype == LINR_BF16 && ix->row_bytes == 256;
    // ... and for bf16 rows of 128 bytes with eight embeddings per query: 32 queries per wave, 128 per stream
    const bool dense_bf16_m8_ok = !other_family && !g_tuning.no_dense && m == 8 && ix->dtype == LINR_BF16 && ix->row_bytes == 128 &&
                                  B >= (g_tuning.dense_min_batch ? g_tuning.dense_min_batch : 24u);
    uint32_t dg = 0, dsets = 1, dmax = 1024;
    if (dense_ok) {
        // up to four query sets per workgroup, each an equal run (a multiple of 64) of the batch's order; a wave keeps
        // its set's queries in registers, 4 to 16 groups of 16
        if (g_tuning.dense_groups) {
            dg = g_tuning.dense_groups;
            dmax = LINR_WAVES_PER_BLOCK * dg * 16;
            const uint32_t b1 = B < dmax ? B : dmax, sets = (b1 + dg * 16 - 1) / (dg * 16);
            dsets = sets <= 1 ? 1u : sets <= 2 ? 2u : 4u;
        } else {
            const uint32_t b1 = B < dmax ? B : dmax;
            dsets = b1 <= 256 ? 1u : b1 <= 512 ? 2u : 4u;
            dg = ((((b1 + dsets - 1) / dsets) + 63u) & ~63u) / 16;
        }
        if (linr_dense_dispatch(0, p->vk, dg, ix->ts != nullptr, 0, nullptr, nullptr, nullptr) != hipSuccess) dg = 0;
    } else if (dense_bf16_ok) {
        dmax = 512;
        const uint32_t b1 = B < dmax ? B : dmax;
        dsets = b1 <= 128 ? 1u : b1 <= 256 ? 2u : 4u;
        dg = ((((b1 + dsets - 1) / dsets) + 63u) & ~63u) / 16;
        if (g_tuning.dense_groups == 4 || g_tuning.dense_groups == 8) {
            dg = g_tuning.dense_groups;
            dmax = LINR_WAVES_PER_BLOCK * dg * 16;
            const uint32_t b2 = B < dmax ? B : dmax, sets = (b2 + dg * 16 - 1) / (dg * 16);
            dsets = sets <= 1 ? 1u : sets <= 2 ? 2u : 4u;
        }
        if (linr_dense_bf16_dispatch(0, p->ks, dg, 1, ix->ts != nullptr, 0, nullptr, nullptr, nullptr) != hipSuccess) dg = 0;
    } else if (dense_bf16_m8_ok) {
        dmax = 128;
        const uint32_t b1 = B < dmax ? B : dmax;
        dsets = b1 <= 32 ? 1u : b1 <= 64 ? 2u : 4u;
        dg = 16;
        if (linr_dense_bf16_dispatch(0, p->ks, dg, 8, ix->ts != nullptr, 0, nullptr, nullptr, nullptr) != hipSuccess) dg = 0;
    }
    uint32_t Bp;
    if (dg) {
        p->qg = dg;
        p->dense = 1;
        p->coop = 1;                                    // (sweep schedule and slot count as for the cooperative kernels)
        p->generic = 0;
        p->chunk_items = 128;
        p->max_batch = dmax;
        Bp = B < p->max_batch ? B : p->max_batch;
        p->nsplit = dsets;
    } else if (bits_mode) {
        if (m != 1) return LINR_E_SHAPE;
        p->ks = ix->bits_words;
        p->generic = 0;
        p->nsplit = 1;
        // two dozen queries or more: bit matching on the matrix cores (16 x 16 match counts per instruction; codes of
        // up to 128 bits), 16 * qg queries per wave and pass (measured at 1e9 x 64 bits: 6.5 vs 7.1 ms at B = 32,
        // 16.9 vs 25.2 ms at B = 128; at B = 16 the popcount kernel still wins, 4.3 vs 5.0 ms).  Fewer: the popcount
        // kernel, which is bound by HBM for a few queries.
        // (tests: no_coop = 1 forces the popcount kernel, force_generic = 1 the matrix-core kernel)
        uint32_t mq = 0;
        if ((B >= 24 || g_tuning.force_generic) && !g_tuning.no_coop)
            for (uint32_t c = 1; c <= 8; c <<= 1) {
                if (!linr_bits_mfma_variant_exists(p->ks, c)) continue;
                mq = c;
                if (c >= nsg) break;
            }
        if (mq) {
            p->bits = 2;
            p->qg = mq;
            p->chunk_items = 128;
            p->max_batch = mq * 16;
        } else {                                        // every wave a chunk-slot, 64 queries per pass
            p->bits = 1;
            p->qg = 4;
            p->chunk_items = 256;
            p->max_batch = 64;
        }
        Bp = B < p->max_batch ? B : p->max_batch;
    } else if (qw) {
        p->qg = qw;
        p->coop = 1;
        p->wide = 1;
        p->chunk_items = 256 / p->ks;                   // this kernel stages 16 KB of rows per step
        p->generic = 0;
        p->max_batch = LINR_WAVES_PER_BLOCK * qw * 32;
        Bp = B < p->max_batch ? B : p->max_batch;
        p->nsplit = LINR_WAVES_PER_BLOCK;
    } else if (cq) {
        p->qg = cq;
        p->coop = 1;
        p->generic = 0;
        p->max_batch = LINR_WAVES_PER_BLOCK * cq * 16;
        Bp = B < p->max_batch ? B : p->max_batch;
        p->nsplit = LINR_WAVES_PER_BLOCK;              // one chunk-slot per workgroup
    } else if (qg) {
        p->qg = qg;
        p->generic = 0;
        p->max_batch = LINR_MAX_NSPLIT * qg * 16;
        Bp = B < p->max_batch ? B : p->max_batch;
        p->nsplit = ((Bp + 15) / 16 + qg - 1) / qg;
    } else {                                            // queries streamed from LDS
        // LDS of that kernel: 38 KB of chunk staging + per 16-query group m*ks KB of fragments
        // and 704 bytes of bounds, compact filters and counters; 160 KB per workgroup
        uint32_t groups = LINR_LDS_SCAN_BUDGET / (m * p->ks * 1024u + 704u);
        if (groups < 1) return LINR_E_SHAPE;
        p->generic = 1;
        p->max_batch = groups * 16;
        Bp = B < p->max_batch ? B : p->max_batch;
        p->qg = (Bp + 15) / 16;
        p->nsplit = 1;
    }
    if (p->nsplit < 1) p->nsplit = 1;
    // persistent grid: exactly the workgroups that are resident at once (a larger grid would leave
    // a tail of workgroups running on a mostly idle chip, since chunks are assigned statically)
    uint32_t bpc = g_tuning.blocks_per_cu;
    if (!bpc) {
        int occ = cached_blocks_per_cu(ix, *p, Bp, m);
        bpc = occ > 0 ? (uint32_t)occ : 2u;
        if (bpc > 8) bpc = 8;
        if (p->bits == 1 && bpc > 4) bpc = 4;           // every wave is a chunk-slot: 256 CUs x 4 x 4 waves = LINR_MAX_SLOTS
    }
    p->n_chunks = (ix->n + p->chunk_items - 1) / p->chunk_items;
    uint64_t waves_wanted = p->n_chunks * p->nsplit;
    uint64_t grid = (uint64_t)ix->num_cu * bpc;
    uint64_t grid_needed = (waves_wanted + LINR_WAVES_PER_BLOCK - 1) / LINR_WAVES_PER_BLOCK;
    if (grid > grid_needed) grid = grid_needed;
    if (grid < 1) grid = 1;
    uint64_t nslots = grid * LINR_WAVES_PER_BLOCK / p->nsplit;
    if (nslots < 1) {                                   // fewer waves than splits: one slot
        grid = (p->nsplit + LINR_WAVES_PER_BLOCK - 1) / LINR_WAVES_PER_BLOCK;
        nslots = 1;
    }
    if (p->dense && nslots > LINR_MAX_SLOTS) {          // every wave of this kernel owns its slot: shrink the grid instead
        grid = (uint64_t)LINR_MAX_SLOTS * p->nsplit / LINR_WAVES_PER_BLOCK;
        nslots = grid * LINR_WAVES_PER_BLOCK / p->nsplit;
    }
    if (nslots > LINR_MAX_SLOTS) nslots = LINR_MAX_SLOTS;
    p->grid = (uint32_t)grid;
    p->nslots = (uint32_t)nslots;
    // a segment must take what one append round can add on top of the k keys a compaction leaves
    p->cap = (uint32_t)align_up((uint64_t)k + (p->dense ? (uint32_t)LINR_DENSE_SLACK : p->wide ? (uint32_t)LINR_WIDE_QCAP : p->chunk_items), 64);

    // Sweeps, coarse to fine.  Sweep l visits the chunks whose index is a multiple of stride[l] but not of
    // stride[l-1] (those were visited before), so every chunk is scored exactly once per search; the k best keys
    // found so far are carried from merge to merge and the k-th of them bounds the next sweep.  A sweep that
    // multiplies the number of visited items by r lets about k * (r - 1) / pass_rate items per query through
    // its score test, so the last, largest sweeps use small factors (2, 4, 4 by default) and the early, tiny ones a
    // big one.
    uint32_t ratio = g_tuning.sample_ratio ? g_tuning.sample_ratio : 8;
    uint64_t min_sample = g_tuning.min_sample ? g_tuning.min_sample : (uint64_t)4 * k;
    uint32_t max_levels = g_tuning.max_levels ? g_tuning.max_levels : LINR_MAX_LEVELS;
    if (max_levels > LINR_MAX_LEVELS) max_levels = LINR_MAX_LEVELS;
    // (kernels that already fold the predicate into their first test gain nothing from the finer split)
    // (... nor does the bit-matching scan for a few queries: it is bound by HBM there, and a sweep over 7/8 of the
    // chunks reads them in longer contiguous runs than the finer sweeps do)
    const bool top_split = !g_tuning.no_top_split && p->n_chunks >= 65536 && (p->coop || p->generic || p->qg > 2) &&
                           !(p->bits && B <= 8);
    // (the large-batch kernels pay for every pair that beats its query's bound, and a sweep that multiplies the visited
    // items by r lets k * (r - 1) / pass_rate of them through per query: they halve all the way down to sweeps of a few
    // million items -- measured at 1e9 x 64 B, B = 256: 23.0 / 29.0 ms at 50 / 5 % pass against 23.9 / 31.5 with {2, 4, 4})
    const uint32_t top_code = g_tuning.top_ratios ? g_tuning.top_ratios
                              : p->dense ? (ix->n >= (1ull << 28) ? 0x2222222u : 0x44222u) : 0x442u;
    uint32_t strides[LINR_MAX_LEVELS];
    uint32_t nl = 0;
    uint64_t s = 1;
    strides[nl++] = 1;
    while (nl < max_levels) {
        uint32_t r = ratio;
        if (top_split && nl - 1 < 8) {
            const uint32_t digit = (top_code >> (4 * (nl - 1))) & 15u;
            if (digit == 2 || digit == 4 || digit == 8) r = digit;
        }
        uint64_t s2 = s * r;
        uint64_t items = (p->n_chunks / s2) * p->chunk_items;
        if (s2 > 0x40000000ull || items < min_sample) break;
        strides[nl++] = (uint32_t)s2;
        s = s2;
    }
    p->nlevels = nl;
    for (uint32_t l = 0; l < nl; ++l) p->stride[l] = strides[nl - 1 - l];
    for (uint32_t l = 0; l < nl; ++l) p->skip_mod[l] = l == 0 ? 0u : p->stride[l - 1] / p->stride[l];

    // flat candidate array per query: the carried k keys plus what one sweep appends (about k * (factor - 1)
    // per query when the bound is good), with room to spare; anything beyond it stays in the per-slot segments
    uint64_t fc = (uint64_t)4 * ratio * k;
    if (fc < 4096) fc = 4096;
    p->flat_cap = (uint32_t)align_up(fc, LINR_FLAT_REGIONS);
    uint64_t off = 0;
    p->off_tau = off;      off = align_up(off + (uint64_t)Bp * 8, 256);
    p->off_ccnt = off;     off = align_up(off + (uint64_t)Bp * 4, 256);
    p->off_carry = off;    off = align_up(off + (uint64_t)Bp * k * 8, 256);
    p->off_gcnt = off;     off = align_up(off + (uint64_t)Bp * LINR_FLAT_REGIONS * LINR_COUNTER_STRIDE * 4, 256);
    p->off_fvalid = off;   off = align_up(off + (uint64_t)Bp * LINR_FLAT_REGIONS * LINR_COUNTER_STRIDE * 4, 256);
    p->off_cnt = off;      off = align_up(off + (uint64_t)Bp * p->nslots * 4, 256);
    p->off_filters = off;  off = align_up(off + (uint64_t)Bp * sizeof(linr_filter), 256);
    p->off_order = off;    off = align_up(off + (uint64_t)Bp * 4, 256);
    p->off_flat = off;     off = align_up(off + (uint64_t)Bp * p->flat_cap * 8, 256);
    p->off_seg = off;      off = align_up(off + (uint64_t)p->nslots * Bp * p->cap * 8, 256);
    p->total_bytes = off;
    return LINR_OK;
}

// The plans of one call: every pass but possibly the last serves max_batch queries with `first`; a ragged last
// pass (B % max_batch queries) is planned for its own size, and that plan can need more workspace than the
// first (fewer queries per wave means more chunk-slots, each with a segment per query).  Both are made -- and
// checked against the caller's workspace -- before anything is enqueued.
struct linr_call_plans {
    linr_plan first, last;
    bool ragged;
    uint64_t bytes;             // workspace the call needs: the larger of the two plans
};

static int make_call_plans(const linr_index* ix, uint32_t B, uint32_t m, uint32_t k, linr_call_plans* cp)
{
    int rc = make_plan(ix, B, m, k, &cp->first);
    if (rc != LINR_OK) return rc;
    cp->ragged = false;
    cp->bytes = cp->first.total_bytes;
    const uint32_t rest = B > cp->first.max_batch ? B % cp->first.max_batch : 0u;
    if (rest) {
        rc = make_plan(ix, rest, m, k, &cp->last);
        if (rc != LINR_OK) return rc;
        cp->ragged = true;
        if (cp->last.total_bytes > cp->bytes) cp->bytes = cp->last.total_bytes;
    }
    return LINR_OK;
}

extern "C" int linr_search_workspace_bytes(const linr_index* ix, uint32_t B, uint32_t m, uint32_t k, uint64_t* bytes)
{
    if (!ix || !bytes) return LINR_E_NULL;
    if (k == 0 || k > LINR_MAX_K) return LINR_E_K;
    if (ix->n == 0) return LINR_E_NOT_LOADED;
    if (B == 0) { *bytes = 256; return LINR_OK; }
    linr_index full;
    if (ix->dead_bit) {                                 // live updates: sized for a full index (the size grows with n)
        full = *ix;
        full.n = ix->capacity;
        full.upd = nullptr;
        ix = &full;
    }
    linr_call_plans cp;
    int rc = make_call_plans(ix, B, m, k, &cp);
    if (rc != LINR_OK) return rc;
    *bytes = cp.bytes;
    return LINR_OK;
}

// Workspace of a search that is issued in groups of at most G queries (clause lists, explicit pre-filtering): the
// larger of what a full group and a ragged last group need.
static int group_workspace_bytes(const linr_index* ix, uint32_t B, uint32_t G, uint32_t m, uint32_t k, uint64_t* bytes)
{
    int rc = linr_search_workspace_bytes(ix, B < G ? B : G, m, k, bytes);
    if (rc != LINR_OK) return rc;
    if (B > G && B % G) {
        uint64_t rest = 0;
        rc = linr_search_workspace_bytes(ix, B % G, m, k, &rest);
        if (rc != LINR_OK) return rc;
        if (rest > *bytes) *bytes = rest;
    }
    return LINR_OK;
}

// ---------------------------------------------------------------------------
// search
// ---------------------------------------------------------------------------
static int search_impl(const linr_index* ix, const void* Q, const float* q_scale, uint32_t B, uint32_t m,
                       const linr_filter* filters, uint32_t k, uint32_t* out_ids, float* out_scores, int32_t* out_raw,
                       uint32_t* out_counts, void* workspace, uint64_t workspace_bytes, void* hip_stream, uint32_t flags,
                       void** events, uint32_t* n_stages, uint32_t* kinds, uint64_t* stage_items,
                       uint32_t max_stages = LINR_MAX_STAGES)
{
    if (n_stages) *n_stages = 0;
    if (!ix) return LINR_E_NULL;
    linr_index snap;
    ix = view_for(ix, (hipStream_t)hip_stream, true, &snap);
    if (k == 0 || k > LINR_MAX_K) return LINR_E_K;
    if (m == 0 || m > LINR_MAX_M) return LINR_E_SHAPE;
    if (ix->n == 0 || !ix->emb) return LINR_E_NOT_LOADED;
    if (B == 0) return LINR_OK;
    if (!Q || !filters || !out_ids || !out_scores || !out_counts) return LINR_E_NULL;
    if (((uintptr_t)Q) & 15u) return LINR_E_SHAPE;
    linr_call_plans cp;
    int rc = make_call_plans(ix, B, m, k, &cp);
    if (rc != LINR_OK) return rc;
    const linr_plan& p = cp.first;
    if (!workspace || (((uintptr_t)workspace) & 255u) || workspace_bytes < cp.bytes) return LINR_E_WORKSPACE;
    if (flags & LINR_FILTERS_ON_HOST) {
        for (uint32_t b = 0; b < B; ++b) {
            if (filters[b].n_any > LINR_MAX_ANY) return LINR_E_FILTER;
            if (filters[b].ts_min > filters[b].ts_max) return LINR_E_FILTER;
        }
    }
    hipStream_t st = (hipStream_t)hip_stream;
    char* ws = (char*)workspace;
    uint32_t stage = 0;
    auto ev = [&](int which, int kind, uint64_t items) -> hipError_t {
        if (!events || stage >= max_stages) return hipSuccess;
        hipError_t e = hipEventRecord((hipEvent_t)events[2 * stage + which], st);
        if (which == 1) {
            if (kinds) kinds[stage] = (uint32_t)kind;
            if (stage_items) stage_items[stage] = items;
            ++stage;
        }
        return e;
    };

    for (uint32_t b0 = 0; b0 < B; b0 += p.max_batch) {
        const uint32_t Bp = (B - b0) < p.max_batch ? (B - b0) : p.max_batch;
        const linr_plan& pp = (cp.ragged && Bp != p.max_batch) ? cp.last : p;       // ragged last pass: its own plan
        unsigned long long* tau = (unsigned long long*)(ws + pp.off_tau);
        uint32_t* cnt = (uint32_t*)(ws + pp.off_cnt);
        uint32_t* gcnt = (uint32_t*)(ws + pp.off_gcnt);
        uint32_t* fvalid = (uint32_t*)(ws + pp.off_fvalid);
        unsigned long long* flat = (unsigned long long*)(ws + pp.off_flat);
        unsigned long long* carry = (unsigned long long*)(ws + pp.off_carry);
        uint32_t* ccnt = (uint32_t*)(ws + pp.off_ccnt);
        linr_filter* dfilt = (linr_filter*)(ws + pp.off_filters);
        unsigned long long* seg = (unsigned long long*)(ws + pp.off_seg);
        const linr_filter* use_filt = filters + b0;
        if (flags & LINR_FILTERS_ON_HOST) {
            HIP_TRY(hipMemcpyAsync(dfilt, filters + b0, (size_t)Bp * sizeof(linr_filter), hipMemcpyHostToDevice, st));
            use_filt = dfilt;
        }
        HIP_TRY(ev(0, LINR_STAGE_INIT, 0));
        HIP_TRY(linr_launch_init(tau, ccnt, gcnt, fvalid, cnt, (uint64_t)Bp * pp.nslots, Bp, st));
        HIP_TRY(ev(1, LINR_STAGE_INIT, 0));

        linr_scan_args sa;
        memset(&sa, 0, sizeof(sa));
        sa.emb = ix->emb; sa.row_scale = ix->row_scale; sa.mask = ix->mask; sa.ts = ix->ts; sa.scale_stats = ix->scale_stats; sa.scale_code = ix->scale_code; sa.k_bits = ix->k_bits; sa.dead_bit = ix->dead_bit;
        sa.n = ix->n; sa.row_bytes = ix->row_bytes;
        sa.Q = (const char*)Q + (uint64_t)b0 * m * ix->row_bytes; sa.B = Bp; sa.m = m;
        sa.filters = use_filt; sa.tau = tau; sa.cnt = cnt; sa.seg = seg;
        sa.nslots = pp.nslots; sa.cap = pp.cap; sa.nsplit = pp.nsplit; sa.k = k;
        sa.gcnt = gcnt; sa.fvalid = fvalid; sa.flat = flat; sa.flat_cap = pp.flat_cap;

        linr_merge_args ma;
        memset(&ma, 0, sizeof(ma));
        ma.tau = tau; ma.cnt = cnt; ma.seg = seg; ma.nslots = pp.nslots; ma.cap = pp.cap; ma.B = Bp; ma.k = k;
        ma.gcnt = gcnt; ma.fvalid = fvalid; ma.flat = flat; ma.flat_cap = pp.flat_cap; ma.carry = carry; ma.ccnt = ccnt;
        ma.dtype = ix->dtype; ma.vk = pp.vk; ma.emb = ix->emb; ma.row_scale = ix->row_scale;
        ma.row_bytes = ix->row_bytes; ma.d = ix->d; ma.Q = sa.Q; ma.q_scale = q_scale ? q_scale + b0 : nullptr; ma.m = m;
        ma.out_ids = out_ids + (uint64_t)b0 * k; ma.out_scores = out_scores + (uint64_t)b0 * k;
        ma.out_raw = out_raw ? out_raw + (uint64_t)b0 * k : nullptr; ma.out_counts = out_counts + b0;

        for (uint32_t l = 0; l < pp.nlevels; ++l) {
            sa.stride = pp.stride[l];
            sa.skip_mod = pp.skip_mod[l];
            const uint64_t n_lc = (pp.n_chunks + sa.stride - 1) / sa.stride;
            sa.n_dense = sa.skip_mod ? n_lc - (n_lc + sa.skip_mod - 1) / sa.skip_mod : n_lc;
            uint64_t items = sa.n_dense * pp.chunk_items;
            if (items > ix->n) items = ix->n;
            HIP_TRY(ev(0, LINR_STAGE_SCAN, items));
            // (int8: the first test works from the smallest and largest bound of a group of queries, and is tightest when
            // neighbouring queries have similar bounds; the bf16 kernel carries every query's own bound in its accumulator)
            if (pp.dense && ix->dtype == LINR_I8) {
                uint32_t* order = (uint32_t*)(ws + pp.off_order);
                HIP_TRY(linr_launch_dense_order(tau, Bp, order, st));
                sa.qorder = order;
            }
            HIP_TRY(linr_launch_scan(pp, ix->dtype, sa, st));
            HIP_TRY(ev(1, LINR_STAGE_SCAN, items));
            ma.final_level = (l + 1 == pp.nlevels);
            HIP_TRY(ev(0, LINR_STAGE_MERGE, 0));
            HIP_TRY(linr_launch_merge(ma, st));
            HIP_TRY(ev(1, LINR_STAGE_MERGE, 0));
        }
    }
    if (n_stages) *n_stages = stage;
    return LINR_OK;
}

// ---------------------------------------------------------------------------
// masking or explicit pre-filtering (Sec. 3.1.2; the trade-off of Sec. 5.3.1 / 5.3.2, Tables 3 - 4)
// ---------------------------------------------------------------------------
static int prefilter_impl(const linr_index* ix, const void* Q, const float* q_scale, uint32_t B, uint32_t m,
                          const linr_filter* filters, uint32_t k, uint32_t* out_ids, float* out_scores,
                          int32_t* out_raw, uint32_t* out_counts, void* workspace, uint64_t workspace_bytes,
                          void* hip_stream, uint32_t flags);

// Share of the items a filter lets through if the attribute bits were independent (each with the frequency sampled
// when the index was loaded).  The timestamp window is not estimated (taken as "all").
static double filter_pass_estimate(const float* freq, const linr_filter& f)
{
    if (f.all_bits & f.none_bits) return 0.0;
    double p = 1.0;
    for (int b = 0; b < 32; ++b) {
        if ((f.all_bits >> b) & 1u) p *= freq[b];
        if ((f.none_bits >> b) & 1u) p *= 1.0 - freq[b];
    }
    for (uint32_t g = 0; g < f.n_any && g < LINR_MAX_ANY; ++g) {
        double none_set = 1.0;
        for (int b = 0; b < 32; ++b)
            if ((f.any_bits[g] >> b) & 1u) none_set *= 1.0 - freq[b];
        p *= 1.0 - none_set;
    }
    return p;
}

// Modelled cost of the two strategies, in milliseconds per 1e9 items (both grow in proportion to the index; only
// their ratio matters).  The constants are fits to searches timed on an MI355X over a 1e9 x 64-byte int8 index with
// per-row scales, k = 1000, B = 1 ... 1024, pass rates 0.1 % ... 50 %:
//   pre-filtering, per group of Bg <= 32 queries: one pass over the mask column, 0.72 + 0.10 Bg with the clauses tested
//     query by query, 1.2 + 0.01 Bg with the byte table (the default from 6 queries on), plus per feasible
//     (item, query) pair 15 + 27 / Bg picoseconds per 64 bytes of row (gathered rows are shared by the group's queries);
//   masking, up to 64 queries: bound by HBM, (row bytes + 8) / 6.3 TB/s whatever the pass rate;
//   masking, larger batches (bound by instruction issue): per 256 queries 23 + 7.6 (log10(0.5 / pass rate))^2 on
//     64-byte int8 rows -- the lower the pass rate, the later the bounds of the score test tighten; other row shapes
//     in proportion to their bytes.
// Returns 1 if explicit pre-filtering is modelled to be faster by a margin (masking cannot overflow: it is the default).
static int plan_prefers_prefilter(const linr_index* ix, uint32_t B, uint32_t m, const double* pass, double* est_pairs)
{
    const double row64 = (double)((ix->row_bytes + 63) / 64) * m;
    double t_pre = 0.0, sum_p = 0.0;
    for (uint32_t b0 = 0; b0 < B; b0 += 32) {
        const uint32_t Bg = (B - b0) < 32 ? (B - b0) : 32;
        double pg = 0.0;
        for (uint32_t b = 0; b < Bg; ++b) pg += pass[b0 + b];
        const uint32_t table_min = g_tuning.prefilter_table_min ? g_tuning.prefilter_table_min : LINR_PREFILTER_TABLE_MIN;
        t_pre += (Bg >= table_min ? 1.2 + 0.01 * Bg : 0.72 + 0.10 * Bg) + pg * 1.0e9 * (15.0 + 27.0 / Bg) * 1.0e-9 * row64;
        sum_p += pg;
    }
    if (est_pairs) *est_pairs = sum_p * (double)ix->n;
    double t_mask = ((double)ix->row_bytes + 8.0) * 1.0e9 / 6.3e12 * 1.0e3;
    if (B > 64) {
        double pm = sum_p / B;
        pm = pm < 1.0e-4 ? 1.0e-4 : pm > 0.5 ? 0.5 : pm;
        const double x = log10(0.5 / pm);
        const double issue = (double)B / 256.0 * (23.0 + 7.6 * x * x) * row64;
        if (issue > t_mask) t_mask = issue;
    }
    return t_pre < 0.85 * t_mask;
}

extern "C" int linr_plan_filtered(const linr_index* ix, const linr_filter* host_filters, uint32_t B, uint32_t m, uint32_t k,
                                  int* strategy, double* est_pairs)
{
    (void)k;
    if (!ix || !host_filters || !strategy) return LINR_E_NULL;
    if (m == 0 || m > LINR_MAX_M) return LINR_E_SHAPE;
    *strategy = LINR_STRATEGY_MASKING;
    if (est_pairs) *est_pairs = 0.0;
    if (B == 0 || ix->n == 0) return LINR_OK;
    float ones[32];
    for (int b = 0; b < 32; ++b) ones[b] = 0.5f;
    const float* freq = ix->have_bit_freq ? ix->bit_freq : ones;
    std::vector<double> pass(B);
    for (uint32_t b = 0; b < B; ++b) {
        pass[b] = filter_pass_estimate(freq, host_filters[b]);
    }
    const int pre = ix->have_bit_freq && ix->dtype != LINR_BITS && plan_prefers_prefilter(ix, B, m, pass.data(), est_pairs);
    *strategy = pre ? LINR_STRATEGY_PREFILTER : LINR_STRATEGY_MASKING;
    return LINR_OK;
}

extern "C" int linr_search_filtered(const linr_index* ix, const void* Q, const float* q_scale, uint32_t B, uint32_t m,
                                    const linr_filter* filters, uint32_t k, uint32_t* out_ids, float* out_scores,
                                    int32_t* out_raw, uint32_t* out_counts, void* workspace, uint64_t workspace_bytes,
                                    void* hip_stream, uint32_t flags)
{
    if ((flags & LINR_PLAN_MASKING) && (flags & LINR_PLAN_PREFILTER)) return LINR_E_SHAPE;
    int strategy = LINR_STRATEGY_MASKING;
    if (flags & LINR_PLAN_PREFILTER) strategy = LINR_STRATEGY_PREFILTER;
    else if (!(flags & LINR_PLAN_MASKING) && (flags & LINR_FILTERS_ON_HOST) && ix && filters && B && k && k <= LINR_MAX_K) {
        // the planner reads the filters, so it only runs where they are in host memory; and it only chooses the
        // strategy that needs the larger workspace if the caller brought that much
        uint64_t need = 0;
        if (linr_plan_filtered(ix, filters, B, m, k, &strategy, nullptr) != LINR_OK ||
            linr_search_prefilter_workspace_bytes(ix, B, m, k, &need) != LINR_OK || workspace_bytes < need)
            strategy = LINR_STRATEGY_MASKING;
    }
    const uint32_t inner_flags = flags & ~(uint32_t)(LINR_PLAN_MASKING | LINR_PLAN_PREFILTER);
    if (strategy == LINR_STRATEGY_PREFILTER)
        return prefilter_impl(ix, Q, q_scale, B, m, filters, k, out_ids, out_scores, out_raw, out_counts, workspace,
                              workspace_bytes, hip_stream, inner_flags);
    return search_impl(ix, Q, q_scale, B, m, filters, k, out_ids, out_scores, out_raw, out_counts, workspace,
                       workspace_bytes, hip_stream, inner_flags, nullptr, nullptr, nullptr, nullptr);
}

// For callers that cannot allocate: the workspace is the library's fixed per-GPU array.  Nothing here allocates or
// frees; sizes that do not fit are refused before any device work.
extern "C" int linr_search_filtered_noalloc(const linr_index* ix, const void* Q, const float* q_scale, uint32_t B, uint32_t m,
                                            const linr_filter* filters, uint32_t k, uint32_t* out_ids, float* out_scores,
                                            int32_t* out_raw, uint32_t* out_counts, void* hip_stream, uint32_t flags)
{
    if (!ix) return LINR_E_NULL;
    if (B == 0) return search_impl(ix, Q, q_scale, B, m, filters, k, out_ids, out_scores, out_raw, out_counts, nullptr, 0,
                                   hip_stream, flags, nullptr, nullptr, nullptr, nullptr);
    uint64_t need = 0;
    int rc = linr_search_workspace_bytes(ix, B, m, k, &need);
    if (rc != LINR_OK) return rc;
    if (need > LINR_NOALLOC_SCRATCH_BYTES) return LINR_E_TOO_LARGE;
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev != ix->device) HIP_TRY(hipSetDevice(ix->device));
    void* ws = nullptr;
    hipError_t e = linr_static_scratch(ix->device, &ws);
    if (e != hipSuccess) { g_last_hip = (int)e; rc = LINR_E_HIP; }
    else rc = search_impl(ix, Q, q_scale, B, m, filters, k, out_ids, out_scores, out_raw, out_counts, ws,
                          LINR_NOALLOC_SCRATCH_BYTES, hip_stream, flags, nullptr, nullptr, nullptr, nullptr);
    if (dev != ix->device) (void)hipSetDevice(dev);
    return rc;
}

extern "C" int linr_search_filtered_timed(const linr_index* ix, const void* Q, const float* q_scale, uint32_t B, uint32_t m,
                                          const linr_filter* filters, uint32_t k, uint32_t* out_ids, float* out_scores,
                                          int32_t* out_raw, uint32_t* out_counts, void* workspace, uint64_t workspace_bytes,
                                          void* hip_stream, uint32_t flags, void** events, uint32_t* n_stages,
                                          uint32_t* kinds, uint64_t* stage_items)
{
    return search_impl(ix, Q, q_scale, B, m, filters, k, out_ids, out_scores, out_raw, out_counts, workspace,
                       workspace_bytes, hip_stream, flags, events, n_stages, kinds, stage_items);
}

extern "C" int linr_events_create(void** events, uint32_t n)
{
    if (!events) return LINR_E_NULL;
    for (uint32_t i = 0; i < n; ++i) events[i] = nullptr;
    for (uint32_t i = 0; i < n; ++i) {
        hipEvent_t e;
        hipError_t rc = hipEventCreate(&e);
        if (rc != hipSuccess) { g_last_hip = (int)rc; return LINR_E_HIP; }
        events[i] = (void*)e;
    }
    return LINR_OK;
}

extern "C" int linr_events_destroy(void** events, uint32_t n)
{
    if (!events) return LINR_E_NULL;
    for (uint32_t i = 0; i < n; ++i)
        if (events[i]) { (void)hipEventDestroy((hipEvent_t)events[i]); events[i] = nullptr; }
    return LINR_OK;
}

extern "C" int linr_events_elapsed_ms(void** events, uint32_t n_pairs, float* ms)
{
    if (!events || !ms) return LINR_E_NULL;
    for (uint32_t i = 0; i < n_pairs; ++i)
        HIP_TRY(hipEventElapsedTime(&ms[i], (hipEvent_t)events[2 * i], (hipEvent_t)events[2 * i + 1]));
    return LINR_OK;
}

// ---------------------------------------------------------------------------
// quantised search (Sec. 3.2)
// ---------------------------------------------------------------------------
static int copy_small(void** dst, const void* src, uint64_t bytes, int from_host)
{
    void* p = nullptr;
    HIP_TRY(hipMalloc(&p, bytes ? bytes : 16));
    hipError_t e = hipMemcpy(p, src, bytes, from_host ? hipMemcpyHostToDevice : hipMemcpyDeviceToDevice);
    if (e != hipSuccess) { (void)hipFree(p); g_last_hip = (int)e; return LINR_E_HIP; }
    *dst = p;
    return LINR_OK;
}

extern "C" int linr_index_build_bits(linr_index* ix, const uint32_t* perm, const int8_t* signs, uint32_t k_bits, int src)
{
    return linr_index_build_bits_rep(ix, perm, signs, k_bits, 1, src);
}

extern "C" int linr_index_build_bits_rep(linr_index* ix, const uint32_t* perm, const int8_t* signs, uint32_t k_bits, uint32_t reps,
                                         int src)
{
    if (!ix || !perm || !signs) return LINR_E_NULL;
    if (ix->dtype != LINR_F32 && ix->dtype != LINR_BF16) return LINR_E_DTYPE;
    if (ix->n == 0 || !ix->emb) return LINR_E_NOT_LOADED;
    if (reps == 0 || reps > 64 || k_bits == 0 || k_bits % reps != 0 || ix->d % (k_bits / reps) != 0 || !bits_words_supported(k_bits))
        return LINR_E_SHAPE;
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipSetDevice(ix->device));
    if (ix->bits) (void)hipFree(ix->bits);
    if (ix->perm) (void)hipFree(ix->perm);
    if (ix->signs) (void)hipFree(ix->signs);
    ix->bits = nullptr; ix->perm = nullptr; ix->signs = nullptr;
    ix->k_bits = k_bits; ix->bits_words = (k_bits + 63) / 64; ix->bits_reps = reps;
    const int fh = src == LINR_SRC_HOST;
    int rc = copy_small((void**)&ix->perm, perm, (uint64_t)reps * ix->d * 4, fh);
    if (rc == LINR_OK) rc = copy_small((void**)&ix->signs, signs, (uint64_t)reps * ix->d, fh);
    if (rc == LINR_OK) {
        hipError_t e = hipMalloc((void**)&ix->bits, ix->capacity * ix->bits_words * 8);
        if (e == hipSuccess) e = linr_launch_sign_oporp(ix->dtype, ix->emb, ix->n, ix->d, ix->perm, ix->signs, k_bits, reps, ix->bits, nullptr);
        if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
        if (e != hipSuccess) { g_last_hip = (int)e; rc = LINR_E_HIP; }
    }
    (void)hipSetDevice(dev);
    return rc;
}

extern "C" int linr_index_load_bits(linr_index* ix, const uint64_t* bits, const uint32_t* mask, const uint32_t* ts, uint64_t n,
                                    int src)
{
    if (!ix) return LINR_E_NULL;
    if (ix->dtype != LINR_BITS) return LINR_E_DTYPE;
    int rc = load_common(ix, LINR_BITS, bits, nullptr, mask, ts, n, src);       // `emb` holds the codes
    if (rc == LINR_OK) ix->bits = (uint64_t*)ix->emb;
    return rc;
}

extern "C" int linr_quantize_queries(const linr_index* ix, const void* Q, uint32_t B, uint64_t* qbits, void* hip_stream)
{
    if (!ix || !Q || !qbits) return LINR_E_NULL;
    if (ix->dtype != LINR_F32 && ix->dtype != LINR_BF16) return LINR_E_DTYPE;
    if (!ix->bits || !ix->perm) return LINR_E_NOT_LOADED;
    HIP_TRY(linr_launch_sign_oporp(ix->dtype, Q, B, ix->d, ix->perm, ix->signs, ix->k_bits, ix->bits_reps, qbits, (hipStream_t)hip_stream));
    return LINR_OK;
}

// a view of the index whose "embeddings" are the codes: the search machinery then ranks by matching bits
static int bits_view(const linr_index* ix, hipStream_t st, linr_index* v)
{
    if (!ix) return LINR_E_NULL;
    linr_index snap;
    ix = view_for(ix, st, true, &snap);
    if (ix->n == 0 || !ix->bits) return LINR_E_NOT_LOADED;
    *v = *ix;
    v->upd = nullptr;                                   // the view is already the snapshot of this search
    v->dtype = LINR_BITS; v->emb = ix->bits; v->row_scale = nullptr; v->d = ix->k_bits; v->row_bytes = ix->bits_words * 8;
    v->scale_stats = nullptr; v->scale_code = nullptr;
    return LINR_OK;
}

extern "C" int linr_search_bits_workspace_bytes(const linr_index* ix, uint32_t B, uint32_t T, uint64_t* bytes)
{
    if (!bytes) return LINR_E_NULL;
    linr_index v;
    int rc = bits_view(ix, nullptr, &v);
    if (rc != LINR_OK) return rc;
    uint64_t inner = 0;
    rc = linr_search_workspace_bytes(&v, B, 1, T, &inner);
    if (rc != LINR_OK) return rc;
    *bytes = align_up(inner, 256) + align_up((uint64_t)B * T * 4, 256);       // + the float copy of the match counts
    return LINR_OK;
}

static int search_bits_impl(const linr_index* ix, const uint64_t* qbits, uint32_t B, const linr_filter* filters, uint32_t T,
                            uint32_t* out_ids, int32_t* out_matches, uint32_t* out_counts, void* workspace,
                            uint64_t workspace_bytes, void* hip_stream, uint32_t flags, void** events, uint32_t* n_stages,
                            uint32_t* kinds, uint64_t* stage_items)
{
    if (n_stages) *n_stages = 0;
    linr_index v;
    int rc = bits_view(ix, (hipStream_t)hip_stream, &v);
    if (rc != LINR_OK) return rc;
    if (B == 0) return LINR_OK;
    if (!out_matches) return LINR_E_NULL;
    uint64_t inner = 0, total = 0;
    rc = linr_search_workspace_bytes(&v, B, 1, T, &inner);
    if (rc != LINR_OK) return rc;
    rc = linr_search_bits_workspace_bytes(ix, B, T, &total);
    if (rc != LINR_OK) return rc;
    if (!workspace || (((uintptr_t)workspace) & 255u) || workspace_bytes < total) return LINR_E_WORKSPACE;
    float* fscores = (float*)((char*)workspace + align_up(inner, 256));
    return search_impl(&v, qbits, nullptr, B, 1, filters, T, out_ids, fscores, out_matches, out_counts, workspace, inner,
                       hip_stream, flags, events, n_stages, kinds, stage_items);
}

extern "C" int linr_search_bits(const linr_index* ix, const uint64_t* qbits, uint32_t B, const linr_filter* filters, uint32_t T,
                                uint32_t* out_ids, int32_t* out_matches, uint32_t* out_counts, void* workspace,
                                uint64_t workspace_bytes, void* hip_stream, uint32_t flags)
{
    return search_bits_impl(ix, qbits, B, filters, T, out_ids, out_matches, out_counts, workspace, workspace_bytes, hip_stream,
                            flags, nullptr, nullptr, nullptr, nullptr);
}

extern "C" int linr_search_bits_timed(const linr_index* ix, const uint64_t* qbits, uint32_t B, const linr_filter* filters,
                                      uint32_t T, uint32_t* out_ids, int32_t* out_matches, uint32_t* out_counts,
                                      void* workspace, uint64_t workspace_bytes, void* hip_stream, uint32_t flags,
                                      void** events, uint32_t* n_stages, uint32_t* kinds, uint64_t* stage_items)
{
    return search_bits_impl(ix, qbits, B, filters, T, out_ids, out_matches, out_counts, workspace, workspace_bytes, hip_stream,
                            flags, events, n_stages, kinds, stage_items);
}

// large-K selection by bit matching: workspace = counts [B][264] u64 | segment counts [B][n_seg][k_bits + 1] u32 |
// two offset arrays [B][n_seg] u64 | cuts [B] | a copy of host-side filters | differing bits [B][n_seg * 65536] u8
struct select_layout { uint64_t off_hist, off_seg, off_gt, off_eq, off_cut, off_filters, off_dcache, total; uint32_t n_seg, seg_items; };
static void select_plan(const linr_index& v, uint32_t B, select_layout* L)
{
    // large segments when there are enough of them to fill the chip several times over, else smaller ones
    // (decided by the capacity, so that the workspace size does not depend on the number of items resident right now)
    const uint64_t groups = (B + 7) / 8;                      // (the counting pass serves eight queries per workgroup)
    // (a workgroup's fixed work -- clearing and adding up its counts -- grows with the code length, so long codes take
    // the large segments already when they fill the chip once; measured on 15.5 M codes of 128 and 512 bits, B = 16)
    const uint32_t words = (v.k_bits + 63) / 64;
    L->seg_items = (v.capacity / 65536) * groups >= (words >= 4 ? 256u : 8192u) ? 65536u
                   : (v.capacity / 16384) * groups >= 1024 ? 16384u : 4096u;
    if (g_tuning.select_seg_items == 4096 || g_tuning.select_seg_items == 16384 || g_tuning.select_seg_items == 65536)
        L->seg_items = g_tuning.select_seg_items;
    L->n_seg = (uint32_t)((v.n + L->seg_items - 1) / L->seg_items);
    uint64_t o = 0;
    L->off_hist = o; o += align_up((uint64_t)B * LINR_SELECT_BINS * 8, 256);
    L->off_seg = o; o += align_up((uint64_t)B * L->n_seg * (v.k_bits + 1) * 4, 256);
    L->off_gt = o; o += align_up((uint64_t)B * L->n_seg * 8, 256);
    L->off_eq = o; o += align_up((uint64_t)B * L->n_seg * 8, 256);
    L->off_cut = o; o += align_up((uint64_t)B * sizeof(linr_select_cut), 256);
    L->off_filters = o; o += align_up((uint64_t)B * sizeof(linr_filter), 256);
    // one byte per item and query: the differing bits, kept between the passes (saturating at 255 for longer codes)
    L->off_dcache = o; o += align_up((uint64_t)B * L->n_seg * L->seg_items, 256);
    L->total = o;
}

extern "C" int linr_select_bits_workspace_bytes(const linr_index* ix, uint32_t B, uint64_t* bytes)
{
    if (!bytes) return LINR_E_NULL;
    linr_index v;
    int rc = bits_view(ix, nullptr, &v);
    if (rc != LINR_OK) return rc;
    if (B > 65535u) return LINR_E_SHAPE;
    if (ix->dead_bit) v.n = ix->capacity;                    // live updates may add items up to the capacity
    select_layout L;
    select_plan(v, B ? B : 1, &L);
    *bytes = L.total;
    return LINR_OK;
}

extern "C" int linr_select_bits(const linr_index* ix, const uint64_t* qbits, uint32_t B, const linr_filter* filters, uint64_t K,
                                uint32_t* out_ids, uint64_t* out_counts, int32_t* out_thresholds, void* workspace,
                                uint64_t workspace_bytes, void* hip_stream, uint32_t flags)
{
    hipStream_t st = (hipStream_t)hip_stream;
    linr_index v;
    int rc = bits_view(ix, st, &v);
    if (rc != LINR_OK) return rc;
    if (K == 0) return LINR_E_K;
    if (B > 65535u) return LINR_E_SHAPE;
    if (B == 0) return LINR_OK;
    if (!qbits || !filters || !out_ids || !out_counts || !out_thresholds) return LINR_E_NULL;
    if (((uintptr_t)qbits) & 15u) return LINR_E_SHAPE;
    if (flags & LINR_FILTERS_ON_HOST)
        for (uint32_t b = 0; b < B; ++b) {
            if (filters[b].n_any > LINR_MAX_ANY) return LINR_E_FILTER;
            if (filters[b].ts_min > filters[b].ts_max) return LINR_E_FILTER;
        }
    select_layout L;
    select_plan(v, B, &L);
    if (!workspace || (((uintptr_t)workspace) & 255u) || workspace_bytes < L.total) return LINR_E_WORKSPACE;
    char* ws = (char*)workspace;
    const linr_filter* use = filters;
    if (flags & LINR_FILTERS_ON_HOST) {
        HIP_TRY(hipMemcpyAsync(ws + L.off_filters, filters, (size_t)B * sizeof(linr_filter), hipMemcpyHostToDevice, st));
        use = (const linr_filter*)(ws + L.off_filters);
    }
    HIP_TRY(linr_launch_fill_u32((uint32_t*)(ws + L.off_hist), (uint64_t)B * LINR_SELECT_BINS * 2, 0u, st));
    linr_select_args a;
    memset(&a, 0, sizeof(a));
    a.bits = (const unsigned long long*)v.bits; a.words = v.bits_words; a.k_bits = v.k_bits; a.mask = v.mask; a.ts = v.ts;
    a.dead_bit = v.dead_bit; a.n = v.n; a.id_base = 0; a.n_seg = L.n_seg; a.seg_items = L.seg_items; a.B = B;
    a.q_codes = (const unsigned long long*)qbits; a.filters = use; a.K = K;
    a.hist = (unsigned long long*)(ws + L.off_hist); a.seg_hist = (uint32_t*)(ws + L.off_seg);
    a.gt_base = (unsigned long long*)(ws + L.off_gt); a.eq_base = (unsigned long long*)(ws + L.off_eq);
    a.cut = (linr_select_cut*)(ws + L.off_cut);
    a.dcache = (uint8_t*)(ws + L.off_dcache);
    a.out_ids = out_ids; a.out_counts = (unsigned long long*)out_counts; a.out_thresholds = out_thresholds;
    HIP_TRY(linr_launch_select(a, st));
    return LINR_OK;
}

static int prefilter_group(const linr_index& v, const uint32_t* words, const linr_filter* filters, const uint32_t* item_mask,
                           const uint32_t* item_ts, uint32_t dead_bit, const void* Qg, const float* q_scale_g, uint32_t Bg,
                           uint32_t m, uint32_t k, uint32_t* out_ids, float* out_scores, int32_t* out_raw, uint32_t* out_counts,
                           void* workspace, uint64_t inner, uint32_t* vcnt, hipStream_t st, const uint32_t* cand,
                           const unsigned long long* cand_counts, uint64_t cand_T);

// Two-stage search with more candidates than a ranking holds (T > LINR_MAX_K; the paper's "keep 1 % of the items"):
// the candidates come from the large-K selection, their exact scores from the gather-scoring pass of the explicit
// pre-filtering (candidate lists in place of a predicate), the top k from its merges.
// Queries are served in groups (the selection keeps a byte per item and query, so the group size bounds the
// workspace): as many as fit 2 GiB of such bytes, at least 8, at most 32.
// workspace: selection (8 queries) | query codes [B] | candidates [8][T] | their counts [8] u64 | thresholds [8] |
// search workspace of one group | 4 KB of counters
static uint32_t two_stage_group(const linr_index* ix, uint32_t B)
{
    uint64_t g = ((2ull << 30) / (ix->capacity ? ix->capacity : 1)) & ~7ull;
    if (g < 8) g = 8;
    if (g > 32) g = 32;
    return B < g ? B : (uint32_t)g;
}
struct two_stage_large_layout { uint64_t sel, off_q, off_cand, off_cnt, off_thr, off_inner, inner, off_vcnt, total; };
static int two_stage_large_plan(const linr_index* ix, uint32_t B, uint64_t T, uint32_t k, two_stage_large_layout* L)
{
    if (k > LINR_MAX_K) return LINR_E_K;
    const uint32_t G = two_stage_group(ix, B);
    int rc = linr_select_bits_workspace_bytes(ix, G, &L->sel);
    if (rc != LINR_OK) return rc;
    rc = group_workspace_bytes(ix, B, G, 1, k, &L->inner);
    if (rc != LINR_OK) return rc;
    uint64_t o = align_up(L->sel, 256);
    L->off_q = o; o += align_up((uint64_t)B * ix->bits_words * 8, 256);
    L->off_cand = o; o += align_up((uint64_t)G * T * 4, 256);
    L->off_cnt = o; o += align_up((uint64_t)G * 8, 256);
    L->off_thr = o; o += align_up((uint64_t)G * 4, 256);
    L->off_inner = o; o += align_up(L->inner, 256);
    L->off_vcnt = o; o += 4096;
    L->total = o;
    return LINR_OK;
}

// candidates up to this T are ranked first (linr_search_bits + rescore kernel); above it: selection + gather scoring
static uint32_t two_stage_rank_max()
{
    const uint32_t t = g_tuning.two_stage_rank_max ? g_tuning.two_stage_rank_max : 999u;
    return t < LINR_MAX_K ? t : LINR_MAX_K;
}

static int two_stage_large(const linr_index* ix, const void* Q, uint32_t B, const linr_filter* filters, uint64_t T, uint32_t k,
                           uint32_t* out_ids, float* out_scores, uint32_t* out_counts, void* workspace, uint64_t workspace_bytes,
                           void* hip_stream, uint32_t flags)
{
    hipStream_t st = (hipStream_t)hip_stream;
    if (T > ix->capacity) T = ix->capacity;
    two_stage_large_layout L;
    int rc = two_stage_large_plan(ix, B, T, k, &L);
    if (rc != LINR_OK) return rc;
    if (!workspace || (((uintptr_t)workspace) & 255u) || workspace_bytes < L.total) return LINR_E_WORKSPACE;
    if (((uintptr_t)Q) & 15u) return LINR_E_SHAPE;
    char* ws = (char*)workspace;
    uint64_t* qbits = (uint64_t*)(ws + L.off_q);
    uint32_t* cand = (uint32_t*)(ws + L.off_cand);
    unsigned long long* ccnt = (unsigned long long*)(ws + L.off_cnt);
    rc = linr_quantize_queries(ix, Q, B, qbits, hip_stream);
    if (rc != LINR_OK) return rc;
    linr_index v;
    {
        linr_index snap;
        v = *view_for(ix, st, true, &snap);
    }
    v.upd = nullptr;
    const uint32_t G = two_stage_group(ix, B);
    for (uint32_t b0 = 0; b0 < B; b0 += G) {
        const uint32_t Bg = (B - b0) < G ? (B - b0) : G;
        rc = linr_select_bits(ix, qbits + (uint64_t)b0 * ix->bits_words, Bg, filters + b0, T, cand, (uint64_t*)ccnt,
                              (int32_t*)(ws + L.off_thr), ws, L.sel, hip_stream, flags);
        if (rc != LINR_OK) return rc;
        rc = prefilter_group(v, nullptr, nullptr, nullptr, nullptr, 0, (const char*)Q + (uint64_t)b0 * v.row_bytes, nullptr, Bg, 1, k,
                             out_ids + (uint64_t)b0 * k, out_scores + (uint64_t)b0 * k, nullptr, out_counts + b0, ws + L.off_inner,
                             L.inner, (uint32_t*)(ws + L.off_vcnt), st, cand, ccnt, T);
        if (rc != LINR_OK) return rc;
    }
    return LINR_OK;
}

extern "C" int linr_search_two_stage_workspace_bytes(const linr_index* ix, uint32_t B, uint32_t T, uint32_t k, uint64_t* bytes)
{
    if (!ix || !bytes) return LINR_E_NULL;
    if (ix->dtype != LINR_F32 && ix->dtype != LINR_BF16) return LINR_E_DTYPE;
    if (k == 0 || k > T) return LINR_E_K;
    if (T > two_stage_rank_max()) {
        two_stage_large_layout L;
        int rc2 = two_stage_large_plan(ix, B ? B : 1, T > ix->capacity ? ix->capacity : T, k, &L);
        if (rc2 != LINR_OK) return rc2;
        *bytes = L.total;
        return LINR_OK;
    }
    uint64_t s1 = 0;
    int rc = linr_search_bits_workspace_bytes(ix, B, T, &s1);
    if (rc != LINR_OK) return rc;
    *bytes = align_up(s1, 256) + align_up((uint64_t)B * ix->bits_words * 8, 256) + 2 * align_up((uint64_t)B * T * 4, 256) +
             align_up((uint64_t)B * 4, 256);
    return LINR_OK;
}

extern "C" int linr_search_two_stage(const linr_index* ix, const void* Q, uint32_t B, const linr_filter* filters, uint32_t T,
                                     uint32_t k, uint32_t* out_ids, float* out_scores, uint32_t* out_counts, void* workspace,
                                     uint64_t workspace_bytes, void* hip_stream, uint32_t flags)
{
    if (!ix) return LINR_E_NULL;
    if (ix->dtype != LINR_F32 && ix->dtype != LINR_BF16) return LINR_E_DTYPE;
    if (k == 0 || k > T) return LINR_E_K;
    if (ix->n == 0 || !ix->emb || !ix->bits) return LINR_E_NOT_LOADED;
    if (B == 0) return LINR_OK;
    if (!Q || !filters || !out_ids || !out_scores || !out_counts) return LINR_E_NULL;
    if (T > two_stage_rank_max())
        return two_stage_large(ix, Q, B, filters, T, k, out_ids, out_scores, out_counts, workspace, workspace_bytes, hip_stream,
                               flags);
    uint64_t s1 = 0, total = 0;
    int rc = linr_search_bits_workspace_bytes(ix, B, T, &s1);
    if (rc != LINR_OK) return rc;
    rc = linr_search_two_stage_workspace_bytes(ix, B, T, k, &total);
    if (rc != LINR_OK) return rc;
    if (!workspace || (((uintptr_t)workspace) & 255u) || workspace_bytes < total) return LINR_E_WORKSPACE;
    char* w = (char*)workspace + align_up(s1, 256);
    uint64_t* qbits = (uint64_t*)w;              w += align_up((uint64_t)B * ix->bits_words * 8, 256);
    uint32_t* ids1 = (uint32_t*)w;               w += align_up((uint64_t)B * T * 4, 256);
    int32_t* m1 = (int32_t*)w;                   w += align_up((uint64_t)B * T * 4, 256);
    uint32_t* cnt1 = (uint32_t*)w;
    rc = linr_quantize_queries(ix, Q, B, qbits, hip_stream);
    if (rc != LINR_OK) return rc;
    rc = linr_search_bits(ix, qbits, B, filters, T, ids1, m1, cnt1, workspace, s1, hip_stream, flags);
    if (rc != LINR_OK) return rc;
    linr_rescore_args ra;
    memset(&ra, 0, sizeof(ra));
    ra.dtype = ix->dtype; ra.emb = ix->emb; ra.d = ix->d; ra.row_bytes = ix->row_bytes; ra.Q = Q; ra.B = B; ra.T = T; ra.k = k;
    ra.cand_ids = ids1; ra.cand_counts = cnt1; ra.out_ids = out_ids; ra.out_scores = out_scores; ra.out_counts = out_counts;
    HIP_TRY(linr_launch_rescore(ra, (hipStream_t)hip_stream));
    return LINR_OK;
}

// ---------------------------------------------------------------------------
// live updates (Sec. 4 "Model Live Update"; their cost for concurrent searches: Sec. 5.3, Table 5)
// ---------------------------------------------------------------------------
#define LINR_DEAD_BIT 0x80000000u

extern "C" int linr_index_enable_updates(linr_index* ix)
{
    if (!ix) return LINR_E_NULL;
    if (ix->n == 0 || !ix->emb) return LINR_E_NOT_LOADED;
    if (ix->upd) return LINR_OK;
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipSetDevice(ix->device));
    int rc = LINR_OK;
    // bit 31 of the masks becomes the library's "holds no item" mark: no resident item may carry it
    uint32_t* acc = nullptr;
    uint32_t host_acc = 0;
    hipError_t e = hipMalloc((void**)&acc, 256);
    if (e == hipSuccess) e = hipMemset(acc, 0, 4);
    if (e == hipSuccess) e = linr_launch_mask_or(ix->mask, ix->n, acc, nullptr);
    if (e == hipSuccess) e = hipMemcpy(&host_acc, acc, 4, hipMemcpyDeviceToHost);
    if (acc) (void)hipFree(acc);
    if (e != hipSuccess) { g_last_hip = (int)e; rc = LINR_E_HIP; }
    else if (host_acc & LINR_DEAD_BIT) rc = LINR_E_FILTER;
    if (rc == LINR_OK) {
        linr_update_state* u = new (std::nothrow) linr_update_state();
        if (!u) rc = LINR_E_HIP;
        else {
            u->n_pending = ix->n; u->stream = nullptr; u->pending = false; u->staging = nullptr; u->host_staging = nullptr; u->staging_bytes = 0;
            e = hipEventCreateWithFlags(&u->done, hipEventDisableTiming);
            if (e != hipSuccess) { g_last_hip = (int)e; rc = LINR_E_HIP; delete u; }
            else { ix->upd = u; ix->dead_bit = LINR_DEAD_BIT; }
        }
    }
    (void)hipSetDevice(dev);
    return rc;
}

// room for `bytes` in the staging buffer; waits for the update that may still read the old contents
static int staging_reserve(linr_update_state* u, uint64_t bytes)
{
    if (u->pending) HIP_TRY(hipEventSynchronize(u->done));
    if (bytes > u->staging_bytes) {
        if (u->staging) (void)hipFree(u->staging);
        if (u->host_staging) (void)hipHostFree(u->host_staging);
        u->staging = nullptr; u->host_staging = nullptr; u->staging_bytes = 0;
        const uint64_t want = align_up(bytes < 65536 ? 65536 : bytes, 65536);
        HIP_TRY(hipMalloc(&u->staging, want));
        HIP_TRY(hipHostMalloc(&u->host_staging, want, hipHostMallocDefault));
        u->staging_bytes = want;
    }
    return LINR_OK;
}

static int update_impl(linr_index* ix, const uint32_t* slots, uint32_t count, const void* emb, const float* row_scale,
                       const uint32_t* mask, const uint32_t* ts, int src, hipStream_t st, bool is_delete)
{
    if (!ix) return LINR_E_NULL;
    linr_update_state* u = ix->upd;
    if (!u) return LINR_E_STATE;
    if (count == 0) return LINR_OK;
    if (!slots) return LINR_E_NULL;
    if (!is_delete) {
        if (!emb || !mask || (ix->row_scale && !row_scale) || (ix->ts && !ts)) return LINR_E_NULL;
        if (src != LINR_SRC_HOST && src != LINR_SRC_DEVICE_COPY && src != LINR_SRC_DEVICE_BORROW) return LINR_E_SHAPE;
    }
    std::lock_guard<std::mutex> writer(u->writer);
    uint64_t mark;
    {
        std::lock_guard<std::mutex> g(u->mu);
        mark = u->pending ? u->n_pending : ix->n;
    }
    uint64_t top = 0;
    for (uint32_t i = 0; i < count; ++i) {
        if (slots[i] >= (is_delete ? mark : ix->capacity)) return LINR_E_CAPACITY;
        if ((uint64_t)slots[i] + 1 > top) top = (uint64_t)slots[i] + 1;
    }
    if (!is_delete) {                                   // two writers of one slot in one launch would tear its row
        std::vector<uint32_t> sorted(slots, slots + count);
        std::sort(sorted.begin(), sorted.end());
        if (std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end()) return LINR_E_SHAPE;
    }
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipSetDevice(ix->device));
    auto body = [&]() -> int {
        const bool host_rows = !is_delete && src == LINR_SRC_HOST;
        const uint64_t o_slots = 0;
        const uint64_t o_emb = align_up((uint64_t)count * 4, 256);
        const uint64_t o_mask = o_emb + (host_rows ? align_up((uint64_t)count * ix->row_bytes, 256) : 0);
        const uint64_t o_scale = o_mask + (host_rows ? align_up((uint64_t)count * 4, 256) : 0);
        const uint64_t o_ts = o_scale + (host_rows && ix->row_scale ? align_up((uint64_t)count * 4, 256) : 0);
        const uint64_t total = o_ts + (host_rows && ix->ts ? align_up((uint64_t)count * 4, 256) : 0);
        int rc = staging_reserve(u, total);
        if (rc != LINR_OK) return rc;
        char* sg = (char*)u->staging;
        char* hs = (char*)u->host_staging;
        memcpy(hs + o_slots, slots, (size_t)count * 4);
        if (host_rows) {
            memcpy(hs + o_emb, emb, (size_t)count * ix->row_bytes);
            memcpy(hs + o_mask, mask, (size_t)count * 4);
            if (ix->row_scale) memcpy(hs + o_scale, row_scale, (size_t)count * 4);
            if (ix->ts) memcpy(hs + o_ts, ts, (size_t)count * 4);
        }
        HIP_TRY(hipMemcpyAsync(sg, hs, (size_t)total, hipMemcpyHostToDevice, st));
        const uint32_t* d_slots = (const uint32_t*)(sg + o_slots);
        if (is_delete) {
            HIP_TRY(linr_launch_tombstone((uint32_t*)ix->mask, d_slots, count, ix->dead_bit, st));
        } else {
            linr_upsert_args a;
            memset(&a, 0, sizeof(a));
            a.slots = d_slots; a.count = count; a.row_bytes = ix->row_bytes; a.dead_bit = ix->dead_bit;
            a.emb = (void*)ix->emb; a.row_scale = (float*)ix->row_scale; a.mask = (uint32_t*)ix->mask; a.ts = (uint32_t*)ix->ts;
            if (host_rows) {
                a.src_emb = sg + o_emb; a.src_mask = (const uint32_t*)(sg + o_mask);
                a.src_scale = (const float*)(sg + o_scale); a.src_ts = (const uint32_t*)(sg + o_ts);
            } else {
                a.src_emb = emb; a.src_mask = mask; a.src_scale = row_scale; a.src_ts = ts;
            }
            // slots between the old mark and the new one that this batch does not write hold no item
            if (top > mark) HIP_TRY(linr_launch_fill_u32((uint32_t*)ix->mask + mark, top - mark, ix->dead_bit, st));
            HIP_TRY(linr_launch_upsert(a, st));
            if (ix->bits && ix->dtype != LINR_BITS)     // the quantised search's codes follow the rows
                HIP_TRY(linr_launch_sign_oporp_scatter(ix->dtype, a.src_emb, count, ix->d, ix->perm, ix->signs, ix->k_bits,
                                                       ix->bits_reps, ix->bits, d_slots, st));
            HIP_TRY(linr_launch_upsert_masks(a, st));   // last: the mask makes the slot visible
        }
        HIP_TRY(hipEventRecord(u->done, st));
        std::lock_guard<std::mutex> g(u->mu);
        u->n_pending = top > mark ? top : mark;
        u->stream = st;
        u->pending = true;
        return LINR_OK;
    };
    const int rc = body();
    (void)hipSetDevice(dev);
    return rc;
}

extern "C" int linr_index_upsert(linr_index* ix, const uint32_t* slots, uint32_t count, const void* emb, const float* row_scale,
                                 const uint32_t* mask, const uint32_t* ts, int src, void* hip_stream)
{
    return update_impl(ix, slots, count, emb, row_scale, mask, ts, src, (hipStream_t)hip_stream, false);
}

extern "C" int linr_index_delete(linr_index* ix, const uint32_t* slots, uint32_t count, void* hip_stream)
{
    return update_impl(ix, slots, count, nullptr, nullptr, nullptr, nullptr, LINR_SRC_HOST, (hipStream_t)hip_stream, true);
}

extern "C" int linr_index_sync_updates(linr_index* ix)
{
    if (!ix) return LINR_E_NULL;
    linr_update_state* u = ix->upd;
    if (!u) return LINR_E_STATE;
    std::lock_guard<std::mutex> writer(u->writer);
    bool pending;
    {
        std::lock_guard<std::mutex> g(u->mu);
        pending = u->pending;
    }
    if (pending) HIP_TRY(hipEventSynchronize(u->done));
    std::lock_guard<std::mutex> g(u->mu);
    if (u->pending) { ix->n = u->n_pending; u->pending = false; }
    return LINR_OK;
}

// ---------------------------------------------------------------------------
// attribute matching over clause lists (Sec. 3.1.1; the representation the benchmark of Sec. 5.3 uses)
// ---------------------------------------------------------------------------
extern "C" int linr_index_load_clauses(linr_index* ix, const uint64_t* values, const uint8_t* counts, uint32_t n_clauses,
                                       uint32_t row_width, uint32_t reverse, uint64_t n, int src)
{
    if (!ix || !values || !counts) return LINR_E_NULL;
    if (ix->n == 0 || !ix->emb) return LINR_E_NOT_LOADED;
    linr_index snap;
    const linr_index* cur = view_for(ix, nullptr, false, &snap);
    if (n != cur->n) return LINR_E_CAPACITY;
    if (n_clauses == 0 || n_clauses > LINR_MAX_CLAUSES || row_width == 0 || row_width > LINR_MAX_CLAUSE_ROW) return LINR_E_SHAPE;
    if (n_clauses < 32 && (reverse >> n_clauses) != 0) return LINR_E_SHAPE;
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipSetDevice(ix->device));
    if (ix->clause_values) (void)hipFree(ix->clause_values);
    if (ix->clause_counts) (void)hipFree(ix->clause_counts);
    ix->clause_values = nullptr; ix->clause_counts = nullptr; ix->clause_n = 0;
    const int fh = src == LINR_SRC_HOST;
    // for the whole capacity, like the other library-owned columns; slots beyond n list nothing
    const uint64_t cap = ix->capacity;
    int rc = copy_column((const void**)&ix->clause_values, values, n * row_width * 8, cap * row_width * 8, fh);
    if (rc == LINR_OK) rc = copy_column((const void**)&ix->clause_counts, counts, n * n_clauses, cap * n_clauses, fh);
    if (rc == LINR_OK && cap > n) {
        hipError_t e = hipMemset(ix->clause_counts + n * n_clauses, 0, (cap - n) * n_clauses);
        if (e != hipSuccess) { g_last_hip = (int)e; rc = LINR_E_HIP; }
    }
    if (rc == LINR_OK) { ix->n_clauses = n_clauses; ix->clause_width = row_width; ix->clause_reverse = reverse; ix->clause_n = n; }
    (void)hipSetDevice(dev);
    return rc;
}

// workspace of a clause search: the inner search of one group of <= 32 queries, then one word per item, then 32 filters
static int clause_layout(const linr_index* v, uint32_t B, uint32_t m, uint32_t k, uint64_t* inner, uint64_t* off_words,
                         uint64_t* off_filters, uint64_t* total)
{
    int rc = group_workspace_bytes(v, B, 32, m, k, inner);
    if (rc != LINR_OK) return rc;
    const uint64_t items = v->dead_bit ? v->capacity : v->n;
    *off_words = align_up(*inner, 256);
    *off_filters = align_up(*off_words + items * 4, 256);
    // + 32 counters (a 128-byte line each) of the pre-filtering strategy + the group's lists regrouped by clause
    *total = align_up(*off_filters + 32 * sizeof(linr_filter) + 4096 + linr_clause_entries_bytes(), 256);
    return LINR_OK;
}

extern "C" int linr_search_clauses_workspace_bytes(const linr_index* ix, uint32_t B, uint32_t m, uint32_t k, uint64_t* bytes)
{
    if (!ix || !bytes) return LINR_E_NULL;
    if (!ix->clause_values) return LINR_E_STATE;
    if (B == 0) { *bytes = 256; return LINR_OK; }
    linr_index snap;
    const linr_index* cur = view_for(ix, nullptr, false, &snap);
    uint64_t inner, ow, of;
    return clause_layout(cur, B, m, k, &inner, &ow, &of, bytes);
}

// Explicit pre-filtering (Sec. 3.1.2) for one group of <= 32 queries: only feasible (item, query) pairs are scored --
// feasibility from one word per item (`words`, clause searches) or from the bitmask / timestamp filters (`filters`,
// device) -- in phases (a small sample of the items, a merge that publishes the k-th key found, the next part against
// that bound, ...), the last merge being the final one.  `workspace` / `inner`: a search workspace for this group; vcnt: 4 KB of counters.
#define LINR_PREFILTER_THREE_PHASES (64ull << 20)      // items from which a third, smaller first sample pays
static int prefilter_group(const linr_index& v, const uint32_t* words, const linr_filter* filters, const uint32_t* item_mask,
                           const uint32_t* item_ts, uint32_t dead_bit, const void* Qg, const float* q_scale_g, uint32_t Bg,
                           uint32_t m, uint32_t k, uint32_t* out_ids, float* out_scores, int32_t* out_raw, uint32_t* out_counts,
                           void* workspace, uint64_t inner, uint32_t* vcnt, hipStream_t st, const uint32_t* cand,
                           const unsigned long long* cand_counts, uint64_t cand_T)
{
    if (m == 0 || m > LINR_MAX_M) return LINR_E_SHAPE;
    if (((uintptr_t)Qg) & 15u) return LINR_E_SHAPE;
    linr_plan pp;
    int rc = make_plan(&v, Bg, m, k, &pp);
    if (rc != LINR_OK) return rc;
    if (pp.total_bytes > inner) return LINR_E_WORKSPACE;
    char* ws = (char*)workspace;
    unsigned long long* tau = (unsigned long long*)(ws + pp.off_tau);
    uint32_t* cnt = (uint32_t*)(ws + pp.off_cnt);
    uint32_t* gcnt = (uint32_t*)(ws + pp.off_gcnt);
    uint32_t* fvalid = (uint32_t*)(ws + pp.off_fvalid);
    uint32_t* ccnt = (uint32_t*)(ws + pp.off_ccnt);
    HIP_TRY(linr_launch_init(tau, ccnt, gcnt, fvalid, cnt, (uint64_t)Bg * pp.nslots, Bg, st));
    linr_prefilter_args pa;
    memset(&pa, 0, sizeof(pa));
    pa.words = words; pa.mask = item_mask; pa.ts = item_ts; pa.filters = filters; pa.dead_bit = dead_bit;
    pa.n = v.n; pa.nq = Bg; pa.dtype = v.dtype; pa.vk = pp.vk; pa.emb = v.emb; pa.row_scale = v.row_scale;
    pa.row_bytes = v.row_bytes; pa.d = v.d; pa.Q = Qg; pa.m = m;
    pa.flat = (unsigned long long*)(ws + pp.off_flat); pa.flat_cap = pp.flat_cap;
    pa.seg = (unsigned long long*)(ws + pp.off_seg); pa.nslots = pp.nslots; pa.cap = pp.cap; pa.B = Bg;
    pa.vcnt = vcnt; pa.gcnt = gcnt; pa.fvalid = fvalid; pa.cnt = cnt;
    pa.cand = cand; pa.cand_counts = cand_counts; pa.cand_T = cand_T;
    pa.table_min = g_tuning.prefilter_table_min ? g_tuning.prefilter_table_min : LINR_PREFILTER_TABLE_MIN;
    linr_merge_args ma;
    memset(&ma, 0, sizeof(ma));
    ma.tau = tau; ma.cnt = cnt; ma.seg = pa.seg; ma.nslots = pp.nslots; ma.cap = pp.cap; ma.B = Bg; ma.k = k;
    ma.gcnt = gcnt; ma.fvalid = fvalid; ma.flat = pa.flat; ma.flat_cap = pp.flat_cap;
    ma.carry = (unsigned long long*)(ws + pp.off_carry); ma.ccnt = ccnt;
    ma.dtype = v.dtype; ma.vk = pp.vk; ma.emb = v.emb; ma.row_scale = v.row_scale; ma.row_bytes = v.row_bytes; ma.d = v.d;
    ma.Q = Qg; ma.q_scale = q_scale_g; ma.m = m;
    ma.out_ids = out_ids; ma.out_scores = out_scores; ma.out_raw = out_raw; ma.out_counts = out_counts;
    // 1/256 of the runs, then 15/256, then the rest (small indexes: 1/16, then the rest)
    static const uint32_t cuts3[4] = {0, 1, 16, 256}, cuts2[3] = {0, 1, 16};
    const bool three = !cand && (g_tuning.prefilter_phases ? g_tuning.prefilter_phases >= 3 : v.n >= LINR_PREFILTER_THREE_PHASES);
    const uint32_t* cuts = three ? cuts3 : cuts2;
    const int n_phases = three ? 3 : 2;
    for (int ph = 0; ph < n_phases; ++ph) {
        pa.mod = cuts[n_phases]; pa.lo = cuts[ph]; pa.hi = cuts[ph + 1];
        pa.tau = ph ? tau : nullptr;
        HIP_TRY(linr_launch_prefilter(pa, st));
        ma.final_level = ph + 1 == n_phases ? 1 : 0;
        HIP_TRY(linr_launch_merge(ma, st));
    }
    HIP_TRY(linr_launch_prefilter_overflow(vcnt, (uint64_t)pp.flat_cap + (uint64_t)pp.nslots * pp.cap, out_counts, Bg, st));
    return LINR_OK;
}

static int search_clauses_impl(const linr_index* ix, const void* Q, const float* q_scale, uint32_t B, uint32_t m,
                               const uint64_t* q_values, const uint8_t* q_counts, uint32_t q_width, uint32_t k,
                               uint32_t* out_ids, float* out_scores, int32_t* out_raw, uint32_t* out_counts, void* workspace,
                               uint64_t workspace_bytes, void* hip_stream, void** events, uint32_t* n_stages,
                               uint32_t* kinds, uint64_t* stage_items, bool prefilter = false)
{
    if (n_stages) *n_stages = 0;
    if (!ix) return LINR_E_NULL;
    hipStream_t st = (hipStream_t)hip_stream;
    linr_index v;
    {
        linr_index snap;
        v = *view_for(ix, st, true, &snap);
    }
    if (v.n == 0 || !v.emb) return LINR_E_NOT_LOADED;
    if (!v.clause_values) return LINR_E_STATE;                            // no clause columns
    if (v.clause_n != v.n && !v.dead_bit) return LINR_E_STATE;            // (only live updates change the item count)
    if (v.dtype == LINR_BITS) return LINR_E_DTYPE;
    if (k == 0 || k > LINR_MAX_K) return LINR_E_K;
    if (q_width == 0 || q_width > LINR_MAX_QUERY_ROW) return LINR_E_SHAPE;
    if (B == 0) return LINR_OK;
    if (!Q || !q_values || !q_counts || !out_ids || !out_scores || !out_counts) return LINR_E_NULL;
    uint64_t inner, ow, of, total;
    int rc = clause_layout(&v, B, m, k, &inner, &ow, &of, &total);
    if (rc != LINR_OK) return rc;
    if (!workspace || (((uintptr_t)workspace) & 255u) || workspace_bytes < total) return LINR_E_WORKSPACE;
    uint32_t* words = (uint32_t*)((char*)workspace + ow);
    linr_filter* filt = (linr_filter*)((char*)workspace + of);
    // the inner search ranks over the word column: "bit b set" is query b's whole predicate
    const uint32_t dead = v.dead_bit;
    const uint32_t* item_mask = v.mask;
    v.mask = words; v.ts = nullptr; v.dead_bit = 0; v.upd = nullptr;
    HIP_TRY(linr_launch_bit_filters(filt, 32, st));
    uint32_t stage = 0;
    for (uint32_t b0 = 0; b0 < B; b0 += 32) {
        const uint32_t Bg = (B - b0) < 32 ? (B - b0) : 32;
        linr_clause_args ca;
        memset(&ca, 0, sizeof(ca));
        ca.values = v.clause_values; ca.counts = v.clause_counts; ca.n_clauses = v.n_clauses; ca.width = v.clause_width;
        ca.reverse = v.clause_reverse; ca.n = v.n;
        ca.q_values = q_values + (uint64_t)b0 * q_width; ca.q_counts = q_counts + (uint64_t)b0 * v.n_clauses;
        ca.q_width = q_width; ca.nq = Bg; ca.mask = item_mask; ca.dead_bit = dead; ca.out = words;
        ca.entries = (char*)(filt + 32) + 4096;
        const bool rec = events && stage < LINR_MAX_STAGES;
        if (rec) HIP_TRY(hipEventRecord((hipEvent_t)events[2 * stage], st));
        HIP_TRY(linr_launch_clause_words(ca, st));
        if (rec) {
            HIP_TRY(hipEventRecord((hipEvent_t)events[2 * stage + 1], st));
            if (kinds) kinds[stage] = LINR_STAGE_FILTER;
            if (stage_items) stage_items[stage] = v.n;
            ++stage;
        }
        if (prefilter) {
            rc = prefilter_group(v, words, nullptr, nullptr, nullptr, 0, (const char*)Q + (uint64_t)b0 * m * v.row_bytes,
                                 q_scale ? q_scale + b0 : nullptr, Bg, m, k, out_ids + (uint64_t)b0 * k,
                                 out_scores + (uint64_t)b0 * k, out_raw ? out_raw + (uint64_t)b0 * k : nullptr, out_counts + b0,
                                 workspace, inner, (uint32_t*)(filt + 32), st, nullptr, nullptr, 0);
            if (rc != LINR_OK) return rc;
            continue;
        }
        uint32_t ns = 0;
        const bool more = events && stage < LINR_MAX_STAGES;
        rc = search_impl(&v, (const char*)Q + (uint64_t)b0 * m * v.row_bytes, q_scale ? q_scale + b0 : nullptr, Bg, m, filt, k,
                         out_ids + (uint64_t)b0 * k, out_scores + (uint64_t)b0 * k, out_raw ? out_raw + (uint64_t)b0 * k : nullptr,
                         out_counts + b0, workspace, inner, hip_stream, LINR_FILTERS_ON_DEVICE, more ? events + 2 * stage : nullptr,
                         more ? &ns : nullptr, more && kinds ? kinds + stage : nullptr, more && stage_items ? stage_items + stage : nullptr,
                         more ? LINR_MAX_STAGES - stage : 0);
        if (rc != LINR_OK) return rc;
        stage += ns;
    }
    if (n_stages) *n_stages = stage;
    return LINR_OK;
}

extern "C" int linr_search_clauses(const linr_index* ix, const void* Q, const float* q_scale, uint32_t B, uint32_t m,
                                   const uint64_t* q_values, const uint8_t* q_counts, uint32_t q_width, uint32_t k,
                                   uint32_t* out_ids, float* out_scores, int32_t* out_raw, uint32_t* out_counts, void* workspace,
                                   uint64_t workspace_bytes, void* hip_stream)
{
    return search_clauses_impl(ix, Q, q_scale, B, m, q_values, q_counts, q_width, k, out_ids, out_scores, out_raw, out_counts,
                               workspace, workspace_bytes, hip_stream, nullptr, nullptr, nullptr, nullptr);
}

extern "C" int linr_search_clauses_timed(const linr_index* ix, const void* Q, const float* q_scale, uint32_t B, uint32_t m,
                                         const uint64_t* q_values, const uint8_t* q_counts, uint32_t q_width, uint32_t k,
                                         uint32_t* out_ids, float* out_scores, int32_t* out_raw, uint32_t* out_counts,
                                         void* workspace, uint64_t workspace_bytes, void* hip_stream, void** events,
                                         uint32_t* n_stages, uint32_t* kinds, uint64_t* stage_items)
{
    return search_clauses_impl(ix, Q, q_scale, B, m, q_values, q_counts, q_width, k, out_ids, out_scores, out_raw, out_counts,
                               workspace, workspace_bytes, hip_stream, events, n_stages, kinds, stage_items);
}

extern "C" int linr_search_clauses_prefilter(const linr_index* ix, const void* Q, const float* q_scale, uint32_t B, uint32_t m,
                                             const uint64_t* q_values, const uint8_t* q_counts, uint32_t q_width, uint32_t k,
                                             uint32_t* out_ids, float* out_scores, int32_t* out_raw, uint32_t* out_counts,
                                             void* workspace, uint64_t workspace_bytes, void* hip_stream)
{
    return search_clauses_impl(ix, Q, q_scale, B, m, q_values, q_counts, q_width, k, out_ids, out_scores, out_raw, out_counts,
                               workspace, workspace_bytes, hip_stream, nullptr, nullptr, nullptr, nullptr, true);
}

extern "C" int linr_index_upsert_clauses(linr_index* ix, const uint32_t* slots, uint32_t count, const uint64_t* values,
                                         const uint8_t* counts, int src, void* hip_stream)
{
    if (!ix) return LINR_E_NULL;
    linr_update_state* u = ix->upd;
    if (!u || !ix->clause_values) return LINR_E_STATE;
    if (count == 0) return LINR_OK;
    if (!slots || !values || !counts) return LINR_E_NULL;
    if (src != LINR_SRC_HOST && src != LINR_SRC_DEVICE_COPY && src != LINR_SRC_DEVICE_BORROW) return LINR_E_SHAPE;
    hipStream_t st = (hipStream_t)hip_stream;
    std::lock_guard<std::mutex> writer(u->writer);
    for (uint32_t i = 0; i < count; ++i)
        if (slots[i] >= ix->capacity) return LINR_E_CAPACITY;
    {
        std::vector<uint32_t> sorted(slots, slots + count);
        std::sort(sorted.begin(), sorted.end());
        if (std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end()) return LINR_E_SHAPE;
    }
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipSetDevice(ix->device));
    auto body = [&]() -> int {
        const bool host_rows = src == LINR_SRC_HOST;
        const uint32_t W = ix->clause_width, C = ix->n_clauses;
        const uint64_t o_val = align_up((uint64_t)count * 4, 256);
        const uint64_t o_cnt = o_val + (host_rows ? align_up((uint64_t)count * W * 8, 256) : 0);
        const uint64_t total = o_cnt + (host_rows ? align_up((uint64_t)count * C, 256) : 0);
        int rc = staging_reserve(u, total);
        if (rc != LINR_OK) return rc;
        char* sg = (char*)u->staging;
        char* hs = (char*)u->host_staging;
        memcpy(hs, slots, (size_t)count * 4);
        if (host_rows) {
            memcpy(hs + o_val, values, (size_t)count * W * 8);
            memcpy(hs + o_cnt, counts, (size_t)count * C);
        }
        HIP_TRY(hipMemcpyAsync(sg, hs, (size_t)total, hipMemcpyHostToDevice, st));
        HIP_TRY(linr_launch_upsert_clauses((const uint32_t*)sg, count, host_rows ? (const uint64_t*)(sg + o_val) : values,
                                           host_rows ? (const uint8_t*)(sg + o_cnt) : counts, ix->clause_values, ix->clause_counts,
                                           W, C, st));
        HIP_TRY(hipEventRecord(u->done, st));
        std::lock_guard<std::mutex> g(u->mu);
        if (!u->pending) u->n_pending = ix->n;
        u->stream = st;
        u->pending = true;
        return LINR_OK;
    };
    const int rc = body();
    (void)hipSetDevice(dev);
    return rc;
}

// ---------------------------------------------------------------------------
// explicit pre-filtering for the bitmask / timestamp filters of linr_search_filtered
// ---------------------------------------------------------------------------
extern "C" int linr_search_prefilter_workspace_bytes(const linr_index* ix, uint32_t B, uint32_t m, uint32_t k, uint64_t* bytes)
{
    if (!ix || !bytes) return LINR_E_NULL;
    if (B == 0) { *bytes = 256; return LINR_OK; }
    uint64_t inner = 0;
    int rc = group_workspace_bytes(ix, B, 32, m, k, &inner);
    if (rc != LINR_OK) return rc;
    *bytes = align_up(inner, 256) + 4096;
    return LINR_OK;
}

static int prefilter_impl(const linr_index* ix, const void* Q, const float* q_scale, uint32_t B, uint32_t m,
                          const linr_filter* filters, uint32_t k, uint32_t* out_ids, float* out_scores,
                          int32_t* out_raw, uint32_t* out_counts, void* workspace, uint64_t workspace_bytes,
                          void* hip_stream, uint32_t flags)
{
    if (!ix) return LINR_E_NULL;
    hipStream_t st = (hipStream_t)hip_stream;
    linr_index v;
    {
        linr_index snap;
        v = *view_for(ix, st, true, &snap);
    }
    v.upd = nullptr;
    if (k == 0 || k > LINR_MAX_K) return LINR_E_K;
    if (m == 0 || m > LINR_MAX_M) return LINR_E_SHAPE;
    if (v.n == 0 || !v.emb) return LINR_E_NOT_LOADED;
    if (v.dtype == LINR_BITS) return LINR_E_DTYPE;
    if (B == 0) return LINR_OK;
    if (!Q || !filters || !out_ids || !out_scores || !out_counts) return LINR_E_NULL;
    if (flags & LINR_FILTERS_ON_HOST)
        for (uint32_t b = 0; b < B; ++b) {
            if (filters[b].n_any > LINR_MAX_ANY) return LINR_E_FILTER;
            if (filters[b].ts_min > filters[b].ts_max) return LINR_E_FILTER;
        }
    uint64_t inner = 0, total = 0;
    int rc = group_workspace_bytes(&v, B, 32, m, k, &inner);
    if (rc != LINR_OK) return rc;
    rc = linr_search_prefilter_workspace_bytes(&v, B, m, k, &total);
    if (rc != LINR_OK) return rc;
    if (!workspace || (((uintptr_t)workspace) & 255u) || workspace_bytes < total) return LINR_E_WORKSPACE;
    uint32_t* vcnt = (uint32_t*)((char*)workspace + align_up(inner, 256));
    for (uint32_t b0 = 0; b0 < B; b0 += 32) {
        const uint32_t Bg = (B - b0) < 32 ? (B - b0) : 32;
        const linr_filter* use = filters + b0;
        if (flags & LINR_FILTERS_ON_HOST) {
            linr_plan pp;
            rc = make_plan(&v, Bg, m, k, &pp);
            if (rc != LINR_OK) return rc;
            linr_filter* dfilt = (linr_filter*)((char*)workspace + pp.off_filters);
            HIP_TRY(hipMemcpyAsync(dfilt, filters + b0, (size_t)Bg * sizeof(linr_filter), hipMemcpyHostToDevice, st));
            use = dfilt;
        }
        rc = prefilter_group(v, nullptr, use, v.mask, v.ts, v.dead_bit, (const char*)Q + (uint64_t)b0 * m * v.row_bytes,
                             q_scale ? q_scale + b0 : nullptr, Bg, m, k, out_ids + (uint64_t)b0 * k, out_scores + (uint64_t)b0 * k,
                             out_raw ? out_raw + (uint64_t)b0 * k : nullptr, out_counts + b0, workspace, inner, vcnt, st, nullptr, nullptr, 0);
        if (rc != LINR_OK) return rc;
    }
    return LINR_OK;
}

extern "C" int linr_search_filtered_prefilter(const linr_index* ix, const void* Q, const float* q_scale, uint32_t B, uint32_t m,
                                              const linr_filter* filters, uint32_t k, uint32_t* out_ids, float* out_scores,
                                              int32_t* out_raw, uint32_t* out_counts, void* workspace, uint64_t workspace_bytes,
                                              void* hip_stream, uint32_t flags)
{
    return prefilter_impl(ix, Q, q_scale, B, m, filters, k, out_ids, out_scores, out_raw, out_counts, workspace, workspace_bytes,
                          hip_stream, flags);
}
