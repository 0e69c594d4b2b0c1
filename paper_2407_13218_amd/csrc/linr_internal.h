// Internal declarations shared by the host-side C ABI (linr_api.cpp) and the HIP
// kernels (linr_kernels.hip).  Not installed; the public interface is include/linr.h.
#pragma once
#include <stdint.h>
#include <hip/hip_runtime.h>
#include "linr.h"

#define LINR_WAVES_PER_BLOCK 4
#define LINR_MAX_LEVELS 12
#define LINR_MAX_SLOTS 4096          // merge kernel keeps one prefix entry per slot in LDS
#define LINR_MAX_NSPLIT 16
#define LINR_WIDE_QCAP 320            // keys a wave of the 32x32-tile kernel queues in LDS before writing them out
#define LINR_DENSE_SLACK 320          // large-batch int8 kernel: a segment holds k keys + its wave's queue (192) + one chunk's appends (128)
#define LINR_FLAT_REGIONS 64          // independently counted regions of a query's flat candidate array
#define LINR_COUNTER_STRIDE 16        // words between two region counters (one 64-byte line each)

// how the ranking value is held in the scan's accumulators
enum { LINR_VK_FLOAT = 0,       // fp32 / bf16: fp32 accumulator is the ranking value
       LINR_VK_I8_SCALED = 1,   // int8: (float)int32 * row_scale
       LINR_VK_I8_RAW = 2 };    // int8: the int32 itself

struct linr_index {
    int device;
    int dtype;
    uint32_t d;
    uint32_t row_bytes;
    uint64_t capacity;
    uint64_t n;
    const void* emb;
    const float* row_scale;
    const uint32_t* mask;
    const uint32_t* ts;
    int owned;                  // library allocated the four columns
    float* scale_stats;         // scaled int8: min of 1/scale, 127/span, span/127, mean of 1/scale (+ reduction scratch); always owned
    uint8_t* scale_code;        // scaled int8: E_i of every item, padded to a multiple of 256 items; always owned
    // quantised search: Sign-OPORP codes [n][bits_words] (owned), k_bits, and the device copies of perm / signs
    uint64_t* bits;
    uint32_t k_bits, bits_words;
    uint32_t bits_reps;         // independent (permutation, signs) draws the code is made of: perm / signs are [bits_reps][d]
    uint32_t* perm;
    int8_t* signs;
    int num_cu;
    // live updates: the mask bit that marks a slot as holding no item (0 until updates are enabled) and the
    // host-side bookkeeping of updates in flight (linr_api.cpp)
    uint32_t dead_bit;
    struct linr_update_state* upd;
    // attribute matching over clause lists: values [clause_n][clause_width], counts [clause_n][n_clauses] (owned)
    uint64_t* clause_values;
    uint8_t* clause_counts;
    uint32_t n_clauses, clause_width, clause_reverse;
    uint64_t clause_n;
    // planner (masking or explicit pre-filtering): share of the items that have each mask bit set, from a sample
    // taken when the columns were loaded (host copy; live updates do not refresh it)
    float bit_freq[32];
    int have_bit_freq;
};

// Launch plan of one search pass (at most max_batch queries).
struct linr_plan {
    int vk;                     // LINR_VK_*
    uint32_t ks;                // 64-byte K-steps per row (1, 2, 4 or 8)
    uint32_t tpc;               // 16-item tiles per chunk (8 / ks)
    uint32_t chunk_items;       // 16 * tpc
    uint32_t qg;                // 16-query groups held per wave
    uint32_t nsplit;            // waves that share a chunk and split the query groups
    uint32_t generic;           // 1 = queries streamed from LDS
    uint32_t coop;              // 1 = the four waves of a workgroup share each chunk and split the query groups
    uint32_t wide;              // 1 = coop with 32x32 tiles; qg then counts 32-query groups per wave
    uint32_t dense;             // 1 = large-batch int8 kernel (queries as the row operand, bounds through the accumulator
                                //     input); qg groups per wave, nsplit query sets per workgroup, nslots = grid * 4 / nsplit
    uint32_t bits;              // 1 = bit-matching kernel over 1-bit codes (ks = 64-bit words per code)
    uint32_t grid;              // workgroups of LINR_WAVES_PER_BLOCK waves
    uint32_t nslots;            // chunk-slots = waves / nsplit
    uint32_t cap;               // entries per (slot, query) candidate segment
    uint32_t max_batch;         // queries per pass
    uint32_t nlevels;
    uint32_t stride[LINR_MAX_LEVELS];   // sweep l visits chunks c = lc * stride[l]; the last stride is 1
    uint32_t skip_mod[LINR_MAX_LEVELS]; // ... except level indices lc that are multiples of this (0: visit all)
    uint64_t n_chunks;
    // workspace layout (byte offsets)
    uint32_t flat_cap;          // keys per query in the flat candidate array
    uint64_t off_tau, off_ccnt, off_carry, off_gcnt, off_fvalid, off_cnt, off_filters, off_order, off_flat, off_seg, total_bytes;
};

struct linr_scan_args {
    const void* emb; const float* row_scale; const uint32_t* mask; const uint32_t* ts;
    const float* scale_stats;   // see linr_index (read by the 32x32-tile kernel only)
    const uint8_t* scale_code;
    uint64_t n; uint32_t row_bytes;
    const void* Q; uint32_t B; uint32_t m;
    const linr_filter* filters;
    unsigned long long* tau;     // [B] best-known lower bound of each query's k-th key (0 = none)
    uint32_t* cnt;              // [B][nslots]: sizes of per-slot segments that could not be flushed
    uint32_t* gcnt;             // [B][REGIONS] (strided) keys flushed into each region of the query's flat array
    uint32_t* fvalid;           // [B][REGIONS] (strided) end of the valid part of a region if a wave could not flush, else ~0
    unsigned long long* flat;   // [B][REGIONS][flat_cap / REGIONS]
    uint32_t flat_cap;
    unsigned long long* seg;     // [nslots][B][cap] per-(slot, query) candidate segments
    uint32_t nslots, cap, nsplit, k;
    uint64_t n_dense;           // chunks this sweep visits
    uint32_t stride;            // chunk stride of this sweep
    uint32_t skip_mod;          // level indices that are multiples of this were visited by earlier sweeps (0: none)
    uint32_t k_bits;            // bit-matching kernel: bits per code
    uint32_t dead_bit;          // mask bit no feasible item may carry (live updates), or 0
    const uint32_t* qorder;     // large-batch int8 kernel: the batch's queries in ascending order of their bounds, or nullptr
};

struct linr_merge_args {
    unsigned long long* tau; uint32_t* cnt; unsigned long long* seg;
    uint32_t* gcnt; uint32_t* fvalid; unsigned long long* flat; uint32_t flat_cap;
    unsigned long long* carry;  // [B][k] best keys of the sweeps so far
    uint32_t* ccnt;             // [B] how many of them
    uint32_t nslots, cap, B, k;
    int final_level;
    // finalisation (final level only)
    int dtype, vk;
    const void* emb; const float* row_scale; uint32_t row_bytes, d;
    const void* Q; const float* q_scale; uint32_t m;
    uint32_t* out_ids; float* out_scores; int32_t* out_raw; uint32_t* out_counts;
};

// kernels' host launchers (linr_kernels.hip)
hipError_t linr_launch_init(unsigned long long* tau, uint32_t* ccnt, uint32_t* gcnt, uint32_t* fvalid, uint32_t* cnt,
                            uint64_t n_cnt, uint32_t B, hipStream_t s);
hipError_t linr_launch_scan(const linr_plan& p, int dtype, const linr_scan_args& a, hipStream_t s);
hipError_t linr_launch_merge(const linr_merge_args& a, hipStream_t s);
// quantised search helpers: codes of `n` rows (fp32 / bf16, row-major [n][d]); rescoring of T candidates per query
hipError_t linr_launch_sign_oporp(int dtype, const void* x, uint64_t n, uint32_t d, const uint32_t* perm, const int8_t* signs,
                                  uint32_t k_bits, uint32_t reps, uint64_t* out, hipStream_t s);
// codes of rows written by an update: row r of x goes to out[scatter[r]] (scatter == nullptr: out[r])
hipError_t linr_launch_sign_oporp_scatter(int dtype, const void* x, uint64_t n, uint32_t d, const uint32_t* perm,
                                          const int8_t* signs, uint32_t k_bits, uint32_t reps, uint64_t* out,
                                          const uint32_t* scatter, hipStream_t s);
// live updates: row / side-column scatter into slots, tombstones, mask fill, OR over all masks
struct linr_upsert_args {
    const uint32_t* slots; uint32_t count; uint32_t row_bytes;       // row_bytes: a multiple of 8
    const void* src_emb; const float* src_scale; const uint32_t* src_mask; const uint32_t* src_ts;
    void* emb; float* row_scale; uint32_t* mask; uint32_t* ts;
    uint32_t dead_bit;
};
hipError_t linr_launch_upsert(const linr_upsert_args& a, hipStream_t s);          // rows, row scales, timestamps
hipError_t linr_launch_upsert_masks(const linr_upsert_args& a, hipStream_t s);    // masks (launched last)
// clause lists of `count` slots: values rows of `width` words and counts rows of `n_clauses` bytes
hipError_t linr_launch_upsert_clauses(const uint32_t* slots, uint32_t count, const uint64_t* src_values, const uint8_t* src_counts,
                                      uint64_t* values, uint8_t* counts, uint32_t width, uint32_t n_clauses, hipStream_t s);
hipError_t linr_launch_tombstone(uint32_t* mask, const uint32_t* slots, uint32_t count, uint32_t dead_bit, hipStream_t s);
hipError_t linr_launch_fill_u32(uint32_t* dst, uint64_t n, uint32_t value, hipStream_t s);
hipError_t linr_launch_mask_or(const uint32_t* mask, uint64_t n, uint32_t* out, hipStream_t s);   // *out |= OR of mask[0..n)
// clause lists -> one word per item whose bit b says "item satisfies every clause of query b" (b < nq <= 32)
struct linr_clause_args {
    const uint64_t* values; const uint8_t* counts; uint32_t n_clauses, width, reverse; uint64_t n;
    const uint64_t* q_values; const uint8_t* q_counts; uint32_t q_width, nq;
    const uint32_t* mask; uint32_t dead_bit;           // live updates: slots whose mask carries dead_bit satisfy nothing
    uint32_t* out;                                      // [n]
    void* entries;                                      // device scratch of linr_clause_entries_bytes(), 8-byte aligned
};
hipError_t linr_launch_clause_words(const linr_clause_args& a, hipStream_t s);
uint32_t linr_clause_entries_bytes(void);
// filters[b] = "bit b of the mask is set", b < nq
hipError_t linr_launch_bit_filters(linr_filter* filters, uint32_t nq, hipStream_t s);
// explicit pre-filtering (Sec. 3.1.2): score only the items whose feasibility word has a bit set, append their keys
// to the query's flat candidate array (first flat_cap keys) and, beyond that, to the per-slot segments
#define LINR_PREFILTER_TABLE_MIN 6     // queries per group from which the clause table beats the query-by-query test (measured at 1e9 items)
struct linr_prefilter_args {
    const uint32_t* words; uint64_t n; uint32_t nq;   // words == nullptr: feasibility from the filters below instead
    const uint32_t* mask; const uint32_t* ts; const linr_filter* filters; uint32_t dead_bit;
    int dtype, vk; const void* emb; const float* row_scale; uint32_t row_bytes, d; const void* Q; uint32_t m;
    unsigned long long* flat; uint32_t flat_cap; unsigned long long* seg; uint32_t nslots, cap, B;
    uint32_t* vcnt;             // [32 x 32 words] per query, a 128-byte line each: word 0 keys appended in this phase,
                                // word 1 sticky "the candidate arrays were too small"
    uint32_t* gcnt; uint32_t* fvalid; uint32_t* cnt;      // the merge's view of where the keys are
    // phases, as the scans' sweeps: a phase scores the runs of 512 items whose number modulo `mod` lies in [lo, hi); the
    // first (lo == 0) takes a small sample, a merge publishes the k-th key found (tau), and the later phases keep only
    // keys that are not below it
    uint32_t mod, lo, hi; const unsigned long long* tau;
    // candidate lists instead of a predicate (two-stage search with many candidates): cand [nq][cand_T] item ids,
    // cand_counts [nq] how many of each row are valid
    const uint32_t* cand; const unsigned long long* cand_counts; uint64_t cand_T;
    uint32_t vec16;             // (set by the launcher) the word / mask / timestamp columns are 16-byte aligned
    uint32_t table_min;         // bitmask filters are looked up byte by byte in a table from this many queries on (0: never)
};
hipError_t linr_launch_prefilter(const linr_prefilter_args& a, hipStream_t s);   // one phase: zero, score, counts
// out_counts[b] = 0xFFFFFFFF where vcnt[b] > capacity (run behind the merge)
hipError_t linr_launch_prefilter_overflow(const uint32_t* vcnt, uint64_t capacity, uint32_t* out_counts, uint32_t nq, hipStream_t s);
// large-K selection by bit matching (counting: the number of differing bits takes k_bits + 1 values)
#define LINR_SELECT_BINS 520           // row length of the global counts (k_bits <= 512 -> 513 values)
struct linr_select_cut { uint32_t t_diff, pad_; uint64_t need_eq; };  // every item with fewer differing bits; the first need_eq with t_diff
struct linr_select_args {
    const unsigned long long* bits; uint32_t words, k_bits; const uint32_t* mask; const uint32_t* ts; uint32_t dead_bit;
    uint64_t n; uint32_t id_base, n_seg, B;
    uint32_t seg_items;                // items whose counts are kept together (one workgroup per segment and query):
                                       // a multiple of 4096, at most 65536 (16-bit counts per lane in LDS)
    const unsigned long long* q_codes; const linr_filter* filters; uint64_t K;
    unsigned long long* hist;          // [B][LINR_SELECT_BINS], zero on entry
    uint32_t* seg_hist;                // [B][n_seg][k_bits + 1]
    unsigned long long* gt_base; unsigned long long* eq_base;     // [B][n_seg]
    linr_select_cut* cut;              // [B]
    uint8_t* dcache;                   // [B][n_seg * seg_items] differing bits per item (255: infeasible, or 255 and more), or nullptr: recompute
    uint32_t* out_ids; unsigned long long* out_counts; int32_t* out_thresholds;
};
hipError_t linr_launch_select(const linr_select_args& a, hipStream_t s);
struct linr_rescore_args {
    int dtype; const void* emb; uint32_t d; uint32_t row_bytes; const void* Q; uint32_t B, T, k;
    const uint32_t* cand_ids; const uint32_t* cand_counts;
    uint32_t* out_ids; float* out_scores; uint32_t* out_counts;
};
hipError_t linr_launch_rescore(const linr_rescore_args& a, hipStream_t s);
// device address of the fixed scratch array (LINR_NOALLOC_SCRATCH_BYTES) of the GPU `device`, which must be current
hipError_t linr_static_scratch(int device, void** ptr);
// 1 if a register-resident-query scan kernel exists for this shape
int linr_fast_variant_exists(int dtype, int vk, uint32_t ks, uint32_t m, uint32_t qg);
int linr_coop_variant_exists(int dtype, int vk, uint32_t ks, uint32_t m, uint32_t qg);
int linr_wide_variant_exists(int dtype, int vk, uint32_t ks, uint32_t m, uint32_t qw);
int linr_bits_mfma_variant_exists(uint32_t words, uint32_t qg);
// large-batch int8 kernel (linr_kernels_dense.hip).  what: 0 = does the variant exist, 1 = workgroups per compute unit
// (*blocks_per_cu), 2 = launch `grid` workgroups on stream s.  ng: 16-query groups per wave (4, 8 or 16).
// order[0 .. B) = the queries of a pass (B <= 1024) in ascending order of their current bounds tau (none first)
hipError_t linr_launch_dense_order(const unsigned long long* tau, uint32_t B, uint32_t* order, hipStream_t s);
hipError_t linr_dense_dispatch(int what, int vk, uint32_t ng, bool ts, uint32_t grid, hipStream_t s, const linr_scan_args* a,
                               int* blocks_per_cu);
hipError_t linr_dense_bf16_dispatch(int what, uint32_t ks, uint32_t ng, uint32_t m, bool ts, uint32_t grid, hipStream_t s,
                                    const linr_scan_args* a, int* blocks_per_cu);      // matrix-core bit matching (plan.bits == 2)
// statistics of 1/row_scale of a scaled int8 index (out[3]; part: 4 * LINR_SCALE_STAT_BLOCKS floats of scratch) and the
// per-item codes derived from them (codes: n_pad bytes)
#define LINR_SCALE_STAT_BLOCKS 1024
// out[b] += number of sampled items (every `step`-th of the n) whose mask has bit b, b < 32; out[32] += items sampled
hipError_t linr_launch_mask_bit_counts(const uint32_t* mask, uint64_t n, uint64_t step, unsigned long long* out, hipStream_t s);
hipError_t linr_launch_scale_stats(const float* row_scale, uint64_t n, uint64_t n_pad, float* part, float* out, uint8_t* codes,
                                   hipStream_t s);
// workgroups of the planned scan kernel resident per compute unit (0 if unknown)
int linr_scan_blocks_per_cu(const linr_plan& p, int dtype, uint32_t B, uint32_t m, int has_ts);
// dynamic LDS bytes of the LDS-streamed scan kernel for a pass of B queries
uint32_t linr_lds_scan_dynamic_bytes(uint32_t B, uint32_t m, uint32_t ks);
#define LINR_LDS_SCAN_BUDGET 120000u  // bytes of dynamic LDS next to 38 KB of per-wave chunk staging
