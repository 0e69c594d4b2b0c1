/*
 * linr.h -- C ABI of the MI355X-native exhaustive filtered top-k retrieval path
 * (LiNR, arXiv 2407.13218: Sec. 3.1 "Exhaustive Search with Attribute-Based
 * Matching").
 *
 * The library keeps an item index resident in GPU memory (Sec. 4.2: the corpus
 * and its filter attributes live wholly on the device) and answers batches of
 * queries: every item is scored against every query (Sec. 3.1.1), an item may
 * enter a query's result only if it satisfies all of that query's clauses
 * (Sec. 3.1.1 feasibility rule, applied as a pre-filter in the sense of
 * Sec. 3.1.2), and the exact top-k of the feasible items is returned.
 *
 * Conventions for every entry point
 *   - returns LINR_OK (0) or a negative LINR_E_* code; never aborts or throws;
 *   - arguments are validated on the host before any device work is enqueued;
 *     on error no output buffer has been touched;
 *   - "device" pointers are HIP device memory of the index's GPU, "host"
 *     pointers are ordinary process memory;
 *   - linr_search_filtered only enqueues work on the caller's stream; results are
 *     valid once that stream has been synchronised.  It allocates nothing.
 */
#ifndef LINR_H
#define LINR_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

typedef struct linr_index linr_index;       /* opaque; created/destroyed by the library */

enum { LINR_F32 = 0, LINR_BF16 = 1, LINR_I8 = 2,            /* element type of the index */
       LINR_BITS = 3 };                                      /* 1-bit codes only (see the quantised search below) */

enum {
    LINR_OK = 0,
    LINR_E_NULL = -1,        /* a required pointer is NULL                                 */
    LINR_E_SHAPE = -2,       /* d / m / B / alignment not supported                        */
    LINR_E_DTYPE = -3,       /* loader or query type does not match the index type         */
    LINR_E_K = -4,           /* k == 0 or k > LINR_MAX_K                                   */
    LINR_E_CAPACITY = -5,    /* n exceeds the capacity given at creation, or id space      */
    LINR_E_NOT_LOADED = -6,  /* search on an index that holds no items yet                 */
    LINR_E_WORKSPACE = -7,   /* workspace NULL, misaligned or smaller than required        */
    LINR_E_HIP = -8,         /* a HIP runtime call failed (see linr_last_hip_error)        */
    LINR_E_FILTER = -9,      /* malformed filter (host filters only are checked)           */
    LINR_E_STATE = -10,      /* the index is not in the state the call needs               */
    LINR_E_TOO_LARGE = -11   /* the search needs more scratch than the fixed array of
                                linr_search_filtered_noalloc holds                         */
};

/* where the loader's source arrays live and who owns the resident copy */
enum {
    LINR_SRC_HOST = 0,           /* host arrays, copied into library-owned device memory   */
    LINR_SRC_DEVICE_COPY = 1,    /* device arrays, copied into library-owned device memory */
    LINR_SRC_DEVICE_BORROW = 2   /* device arrays used in place; the caller keeps them
                                    alive and unchanged for the life of the index          */
};

/* flags of linr_search_filtered */
enum {
    LINR_FILTERS_ON_DEVICE = 0,  /* default: `filters` is a device pointer                 */
    LINR_FILTERS_ON_HOST = 1,    /* `filters` is a host pointer: validated, then copied    */
    LINR_PLAN_MASKING = 2,       /* score every item, filter folded into the scan          */
    LINR_PLAN_PREFILTER = 4      /* explicit pre-filtering (linr_search_filtered_prefilter) */
};

/* the two ways of answering a filtered search (Sec. 3.1.2) */
enum { LINR_STRATEGY_MASKING = 0, LINR_STRATEGY_PREFILTER = 1 };

#define LINR_MAX_ANY 4
#define LINR_MAX_K   8192
#define LINR_MAX_M   8
#define LINR_NO_ID   0xFFFFFFFFu

/*
 * One query's predicate over an item's 32-bit attribute mask and optional
 * 32-bit timestamp (40 bytes, plain data).  Sec. 3.1.1: an item is feasible iff
 * every clause holds; a clause with several attributes holds if at least one of
 * them is present; a reverse clause holds on mismatch.
 *   all_bits  : union of the single-attribute clauses -- each bit must be set;
 *   none_bits : reverse clauses -- none of these bits may be set;
 *   any_bits[g], g < n_any : a multi-attribute clause -- at least one bit set;
 *   ts_min..ts_max : inclusive unsigned window on the item timestamp, evaluated
 *                    only when the index has a timestamp column.
 * The all-zero filter with ts window (0, 0xFFFFFFFF) passes every item.
 */
typedef struct {
    uint32_t all_bits;
    uint32_t none_bits;
    uint32_t any_bits[LINR_MAX_ANY];
    uint32_t n_any;
    uint32_t ts_min, ts_max;
    uint32_t _pad;
} linr_filter;

/*
 * Create an empty index for up to `capacity` items of `d` dimensions on HIP
 * device `device`.  d * sizeof(element) must be a multiple of 16 and at most 512
 * bytes.  capacity <= 2^32 - 2 (item ids are uint32 row numbers).
 * The handle is owned by the library until linr_index_destroy.
 */
int linr_index_create(linr_index** out, uint64_t capacity, uint32_t d, int dtype, int device);

/*
 * Make `n` items resident (Sec. 4.2: embeddings plus filter attributes form the
 * served model).  Row i of `emb` ([n][d], row-major, 16-byte aligned) becomes
 * item id i.  `mask` is [n]; `ts` is [n] or NULL (no timestamp column).
 * A later load replaces the previous contents (and ends live updates, clause columns
 * and 1-bit codes of the previous contents).  `src` is a LINR_SRC_* value (columns used in
 * place, LINR_SRC_DEVICE_BORROW, must all be 16-byte aligned); columns the
 * library copies are allocated for the whole capacity, so that live updates can add
 * items in place.  bf16 values are passed as their 16-bit patterns.
 * int8: symmetric codes with one positive fp32 scale per row; row_scale == NULL
 * selects raw ranking (see linr_search_filtered).  This quantised layout is this
 * library's memory-saving representation (the paper's own is the 1-bit code of
 * Sec. 3.2); it keeps a 1e9 x 64 index at 72 GB.  With row scales the index also
 * owns one code byte per item derived from them (library-allocated at load, in every
 * LINR_SRC_* mode; used by the 32x32-tile kernel).  The loaders allocate device
 * memory and synchronise; the search never does.
 */
int linr_index_load_fp32(linr_index*, const float* emb, const uint32_t* mask, const uint32_t* ts,
                         uint64_t n, int src);
int linr_index_load_bf16(linr_index*, const uint16_t* emb, const uint32_t* mask, const uint32_t* ts,
                         uint64_t n, int src);
int linr_index_load_int8(linr_index*, const int8_t* emb, const float* row_scale, const uint32_t* mask,
                         const uint32_t* ts, uint64_t n, int src);

/* Bytes of device workspace linr_search_filtered needs for (B, m, k) on this index. */
int linr_search_workspace_bytes(const linr_index*, uint32_t B, uint32_t m, uint32_t k, uint64_t* bytes);

/*
 * Exhaustive filtered top-k (Sec. 3.1.1 scoring, Sec. 3.1.2 pre-filter semantics,
 * Sec. 5.3.2: each query of the batch has its own filter).
 *
 *   Q        device [B][m][d] of the index element type; m embeddings per query,
 *            an item's score for the query is the maximum over the m dot products;
 *   q_scale  device [B] or NULL (= 1.0f); int8 only;
 *   filters  [B] linr_filter, device or host per `flags`;
 *   out_ids  device [B][k]; out_scores device [B][k]; out_raw device [B][k] or NULL
 *            (int8 only: the int32 dot product); out_counts device [B];
 *   workspace  device, 256-byte aligned, >= linr_search_workspace_bytes; contents
 *            need not be initialised and are garbage afterwards.  Two searches
 *            that may overlap in time need separate workspaces;
 *   hip_stream  a hipStream_t (NULL = the default stream).
 *
 * Ranking value of item i for query b:
 *   fp32/bf16 : max_e <Q[b][e], emb[i]> accumulated in fp32;
 *   int8, row_scale given : (float)raw * row_scale[i], raw = max_e int32 dot, one
 *               round-to-nearest fp32 product; out_scores = that * q_scale[b];
 *   int8, no row_scale    : raw itself; out_scores = (float)raw * q_scale[b].
 * Row b of the outputs holds counts[b] = min(k, #feasible items) entries sorted by
 * (ranking value descending, item id ascending); the tail is padded with
 * LINR_NO_ID, -INFINITY and INT32_MIN.  Inputs must be finite.
 * B == 0 is a no-op.  Errors: LINR_E_K, LINR_E_SHAPE (m == 0 or m > LINR_MAX_M),
 * LINR_E_NOT_LOADED, LINR_E_WORKSPACE, LINR_E_NULL, LINR_E_FILTER (host filters:
 * n_any > LINR_MAX_ANY, ts_min > ts_max), LINR_E_HIP.
 *
 * Strategy (Sec. 3.1.2; the trade-off of Sec. 5.3.1 - 5.3.2): the search either scores every
 * item with the filter folded into the scan ("masking") or decides feasibility first and
 * scores only the feasible (item, query) pairs (explicit pre-filtering, the path of
 * linr_search_filtered_prefilter, whose notes on LINR_COUNT_OVERFLOW then apply).  Results
 * are identical.  LINR_PLAN_MASKING / LINR_PLAN_PREFILTER force one.  With neither flag the
 * library decides -- linr_plan_filtered's choice -- where it can read the filters
 * (LINR_FILTERS_ON_HOST) and `workspace_bytes` also covers
 * linr_search_prefilter_workspace_bytes; otherwise it masks.
 */
int linr_search_filtered(const linr_index*, const void* Q, const float* q_scale, uint32_t B, uint32_t m,
                         const linr_filter* filters, uint32_t k,
                         uint32_t* out_ids, float* out_scores, int32_t* out_raw, uint32_t* out_counts,
                         void* workspace, uint64_t workspace_bytes, void* hip_stream, uint32_t flags);

/*
 * The planner behind linr_search_filtered.  From the share of items that carry each mask bit
 * (sampled when the index was loaded; live updates do not refresh the sample) it estimates each
 * filter's pass rate, taking attributes as independent and timestamp windows as open, and from
 * that the cost of both strategies with constants fitted to measurements on an MI355X (a
 * 1e9 x 64-byte index: pre-filtering wins below about 2.5e8 ... 5e8 feasible pairs for up to 32
 * queries, below a pass rate of about 0.6 % for hundreds).  *strategy = LINR_STRATEGY_*;
 * *est_pairs (may be NULL) = estimated feasible (item, query) pairs.  `host_filters` is a
 * host pointer.  Nothing is launched.
 */
int linr_plan_filtered(const linr_index*, const linr_filter* host_filters, uint32_t B, uint32_t m, uint32_t k,
                       int* strategy, double* est_pairs);

/*
 * linr_search_filtered for callers that cannot allocate device memory or carry a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * (without the workspace), same kernels and bit-identical results; the scratch memory is a fixed
 * array of LINR_NOALLOC_SCRATCH_BYTES inside the library, one copy per GPU, held from the time the
 * library is loaded until the process ends.  The call allocates and frees nothing (the very first
 * search of a process loads the kernels, as any first launch does: make one call before capturing).
 * A search whose linr_search_workspace_bytes(B, m, k) exceeds LINR_NOALLOC_SCRATCH_BYTES is
 * rejected with LINR_E_TOO_LARGE before anything is enqueued (one query with k <= 1000 fits at
 * any index size; so does B = 4 with k <= 100).  All calls on one GPU share that GPU's array: two
 * such searches that may overlap in time (different streams, different host threads) race -- keep
 * them on one stream, or use linr_search_filtered with separate workspaces.  The array keeps the
 * last call's contents; every counter a search relies on is reset by the search's own first
 * kernel.  The index's device is made current for the duration of the call.
 */
#define LINR_NOALLOC_SCRATCH_BYTES (64u << 20)
int linr_search_filtered_noalloc(const linr_index*, const void* Q, const float* q_scale, uint32_t B, uint32_t m,
                                 const linr_filter* filters, uint32_t k,
                                 uint32_t* out_ids, float* out_scores, int32_t* out_raw, uint32_t* out_counts,
                                 void* hip_stream, uint32_t flags);

/*
 * The same search by explicit pre-filtering (Sec. 3.1.2 "KNN with Explicit Pre-Filtering"):
 * one pass over the mask (and timestamp) column decides feasibility, only the feasible
 * (item, query) pairs are scored -- their rows gathered with 16-byte loads -- and one
 * selection over their keys gives the top k; the embeddings of infeasible items are never
 * read.  Same arguments and results as linr_search_filtered (fp32 / bf16 scores within the
 * usual tolerance of it, int8 bit-identical); workspace from
 * linr_search_prefilter_workspace_bytes.  Queries are answered in groups of 32.  Faster
 * when few (item, query) pairs are feasible (1e9 items, 0.1 % feasible, one query: a
 * thirteenth of the time), slower when many are: the caller chooses, as between the paper's two
 * variants.  A
 * query with more feasible items than the candidate arrays of the workspace hold is not
 * answered: out_counts[b] = LINR_COUNT_OVERFLOW, its other outputs are undefined.
 */
#define LINR_COUNT_OVERFLOW 0xFFFFFFFFu
int linr_search_prefilter_workspace_bytes(const linr_index*, uint32_t B, uint32_t m, uint32_t k, uint64_t* bytes);
int linr_search_filtered_prefilter(const linr_index*, const void* Q, const float* q_scale, uint32_t B, uint32_t m,
                                   const linr_filter* filters, uint32_t k,
                                   uint32_t* out_ids, float* out_scores, int32_t* out_raw, uint32_t* out_counts,
                                   void* workspace, uint64_t workspace_bytes, void* hip_stream, uint32_t flags);

int linr_index_destroy(linr_index*);

/*
 * Quantised search (Sec. 3.2 "Quantized KNN" and the figure "KNN with Quantized
 * Filtering").  An embedding is compressed to k_bits one-bit values by Sign-OPORP:
 *     sketch[j] = sum_{t < L} signs[j*L+t] * x[perm[j*L+t]],  L = d / k_bits,
 *     bit[j]    = sketch[j] > 0
 * (perm: a permutation of 0..d-1; signs: +1 / -1; both drawn once by the caller and
 * shared by items and queries; sums in double precision, t ascending).  Bit j is bit
 * j%64 of 64-bit word j/64; a code is W = ceil(k_bits/64) words.  The similarity of two
 * codes is their number of equal bits.  Codes longer than one pass over the coordinates
 * gives (Sec. 5.3.1 uses 512 bits for d = 128) are R independent draws of (perm, signs),
 * k_bits / R bits each with L = d * R / k_bits, one after the other: bit r * (k_bits / R) + j
 * is bit j of draw r (draws add information only with bins of two or more coordinates:
 * with L = 1 every draw is the same sign quantisation).  Limits: k_bits <= 512 with W in {1, 2, 3, 4, 6, 8}; k_bits % R == 0;
 * d % (k_bits / R) == 0; R <= 64.
 *
 * linr_index_build_bits  derives the codes of every resident item of an fp32 / bf16
 *     index (library-owned, n * W * 8 bytes); perm [d] and signs [d] are host arrays
 *     (src == LINR_SRC_HOST) or device arrays (any other LINR_SRC_* value); copied.
 * linr_index_build_bits_rep  the same with `reps` = R draws: perm [R][d], signs [R][d].
 * linr_index_load_bits   fills an index created with dtype LINR_BITS (d = k_bits) with
 *     ready-made codes [n][W] plus mask / ts: a codes-only index (8 bytes per item at
 *     64 bits) for when memory is the concern.  `src` as for the other loaders.
 * linr_quantize_queries  codes of B query embeddings (device [B][d], index element
 *     type) with the index's perm / signs -> device qbits [B][W].
 * linr_search_bits       per query the T feasible items with the most matching bits,
 *     ties to the lower id: out_ids / out_matches device [B][T] (padding LINR_NO_ID /
 *     INT32_MIN), out_counts device [B] = min(T, #feasible).  qbits device [B][W],
 *     16-byte aligned.  T <= LINR_MAX_K.  Exact with respect to the codes.
 * linr_search_two_stage  quantises the queries, takes the top T by matching bits, scores
 *     those T items with the full-precision embeddings (fp32 accumulation) and returns
 *     the top k <= T by (score descending, id ascending): out_ids / out_scores device
 *     [B][k], out_counts device [B] = min(k, T, #feasible).  m = 1.  An approximation of
 *     linr_search_filtered whose recall grows with T; it equals it when T >= #feasible.
 *     T may exceed LINR_MAX_K (the paper's experiment keeps 1 % of the items): from
 *     T = 1000 on the candidates come from linr_select_bits and are scored by the gather
 *     pass of the explicit pre-filtering (faster than ranking them first; same results);
 *     k <= LINR_MAX_K; a query whose sampled candidates overflow the workspace's
 *     candidate arrays gets out_counts[b] = LINR_COUNT_OVERFLOW.
 * Workspaces: device, 256-byte aligned, sizes from the *_workspace_bytes calls; filters,
 * hip_stream and flags as for linr_search_filtered.  Errors as there, plus LINR_E_DTYPE
 * (index kind does not fit the call) and LINR_E_NOT_LOADED (no codes built yet).
 */
int linr_index_build_bits(linr_index*, const uint32_t* perm, const int8_t* signs, uint32_t k_bits, int src);
int linr_index_build_bits_rep(linr_index*, const uint32_t* perm, const int8_t* signs, uint32_t k_bits, uint32_t reps, int src);
int linr_index_load_bits(linr_index*, const uint64_t* bits, const uint32_t* mask, const uint32_t* ts, uint64_t n, int src);
int linr_quantize_queries(const linr_index*, const void* Q, uint32_t B, uint64_t* qbits, void* hip_stream);
int linr_search_bits_workspace_bytes(const linr_index*, uint32_t B, uint32_t T, uint64_t* bytes);
int linr_search_bits(const linr_index*, const uint64_t* qbits, uint32_t B, const linr_filter* filters, uint32_t T,
                     uint32_t* out_ids, int32_t* out_matches, uint32_t* out_counts,
                     void* workspace, uint64_t workspace_bytes, void* hip_stream, uint32_t flags);
/*
 * Large-K selection by bit matching (Sec. 3.2: the quantised module used without the
 * full-precision stage "when K is large"; the notification use case of Sec. 5.3, the top
 * 50 million of a billion members by 64-bit codes).  Per query the K feasible items with
 * the most matching bits, ties to the lower id -- the first K of the ranking that
 * linr_search_bits returns -- as a set: out_ids device [B][K], row b holding
 * out_counts[b] = min(K, #feasible) ids in ascending order (the rest of the row is not
 * written); out_thresholds[b] = the fewest matching bits among the selected (-1 if none).
 * out_counts device uint64 [B], out_thresholds device int32 [B].  Any K >= 1 (K beyond
 * the item count selects every feasible item).  qbits device [B][W], 16-byte aligned;
 * filters / flags / hip_stream as for linr_search_filtered; B <= 65535.  Exact: a match
 * count takes k_bits + 1 values only, so two streaming passes (counts per segment of
 * items, then the ids) replace a sort.  Works on a codes-only index and on
 * the codes built for an fp32 / bf16 index, also next to live updates.  Workspace: about one
 * byte per item (of the capacity) and query, plus a few MB of counts; a group of queries
 * none of which looks at the attributes does not read the mask column.
 */
int linr_select_bits_workspace_bytes(const linr_index*, uint32_t B, uint64_t* bytes);
int linr_select_bits(const linr_index*, const uint64_t* qbits, uint32_t B, const linr_filter* filters, uint64_t K,
                     uint32_t* out_ids, uint64_t* out_counts, int32_t* out_thresholds,
                     void* workspace, uint64_t workspace_bytes, void* hip_stream, uint32_t flags);
int linr_search_two_stage_workspace_bytes(const linr_index*, uint32_t B, uint32_t T, uint32_t k, uint64_t* bytes);
int linr_search_two_stage(const linr_index*, const void* Q, uint32_t B, const linr_filter* filters, uint32_t T, uint32_t k,
                          uint32_t* out_ids, float* out_scores, uint32_t* out_counts,
                          void* workspace, uint64_t workspace_bytes, void* hip_stream, uint32_t flags);

/*
 * Attribute matching over clause lists (Sec. 3.1.1 "KNN with Similarity Masking" and its
 * figure; the datasets of Sec. 5.3 carry one 64-bit attribute per clause).  There are
 * n_clauses clauses; item i lists counts[i][c] attributes (64-bit ids) for clause c, all
 * lists of an item back to back, clause 0 first, in row i of values [n][row_width] (entries
 * behind the last list are ignored; lists need not be sorted, the kernel stops at the
 * first match anyway).  A query carries lists in the same layout.  A clause is satisfied
 * when the two lists share an attribute -- a REVERSE clause (bit c of `reverse`) when they
 * share none -- and an item is feasible when every clause is; a clause for which the query
 * lists nothing places no constraint.  This predicate replaces the bitmask filter of
 * linr_search_filtered; scoring, ranking, ties, outputs and errors are the same.
 *
 * linr_index_load_clauses  attaches clause columns to a loaded fp32 / bf16 / int8 index:
 *     values [n][row_width] uint64, counts [n][n_clauses] uint8, host or device per `src`
 *     (always copied); n must equal the number of resident items (LINR_E_CAPACITY).
 *     Limits: n_clauses <= LINR_MAX_CLAUSES, row_width <= LINR_MAX_CLAUSE_ROW.
 * linr_search_clauses  q_values device [B][q_width] uint64, q_counts device [B][n_clauses]
 *     uint8, q_width <= LINR_MAX_QUERY_ROW.  Queries are answered in groups of 32: one pass
 *     over the clause columns writes, per item, a word whose bit b says "feasible for query
 *     b of the group", and the exhaustive search then runs with that bit as the predicate.
 *     On an index with live updates, deleted slots are infeasible.
 * linr_index_upsert_clauses  (live updates) writes the lists of `count` slots (host array,
 *     distinct, each < capacity): values [count][row_width], counts [count][n_clauses], host
 *     (copied before the call returns) or device per `src`.  The clause columns span the
 *     capacity; a slot that never received lists lists nothing (it fails every constrained
 *     forward clause and satisfies every reverse clause).  For a new item call this before
 *     linr_index_upsert on the same stream: the slot is not visible yet, so no search can
 *     see the item with someone else's lists.  Enqueues only, like linr_index_upsert.
 * Workspace from linr_search_clauses_workspace_bytes.  LINR_E_STATE without clause columns
 * (and for linr_index_upsert_clauses without live updates).
 */
#define LINR_MAX_CLAUSES 8
#define LINR_MAX_CLAUSE_ROW 32
#define LINR_MAX_QUERY_ROW 64
int linr_index_load_clauses(linr_index*, const uint64_t* values, const uint8_t* counts, uint32_t n_clauses,
                            uint32_t row_width, uint32_t reverse, uint64_t n, int src);
int linr_index_upsert_clauses(linr_index*, const uint32_t* slots, uint32_t count, const uint64_t* values,
                              const uint8_t* counts, int src, void* hip_stream);
int linr_search_clauses_workspace_bytes(const linr_index*, uint32_t B, uint32_t m, uint32_t k, uint64_t* bytes);
int linr_search_clauses(const linr_index*, const void* Q, const float* q_scale, uint32_t B, uint32_t m,
                        const uint64_t* q_values, const uint8_t* q_counts, uint32_t q_width, uint32_t k,
                        uint32_t* out_ids, float* out_scores, int32_t* out_raw, uint32_t* out_counts,
                        void* workspace, uint64_t workspace_bytes, void* hip_stream);

/*
 * The same search by explicit pre-filtering (Sec. 3.1.2 "KNN with Explicit Pre-Filtering"):
 * after the pass over the clause columns only the feasible (item, query) pairs are scored
 * (rows gathered with 16-byte loads, 4 to 16 lanes per pair) and one selection over their keys
 * gives the top k -- the embeddings of infeasible items are never read.  Same arguments,
 * workspace and results as linr_search_clauses (fp32 / bf16 scores within the usual
 * tolerance of each other, int8 bit-identical).  Faster when few items are feasible,
 * slower when many are (the caller chooses, as between the paper's two variants).  A query
 * with more feasible items than the candidate arrays of the workspace hold (several
 * million) is not answered: out_counts[b] = LINR_COUNT_OVERFLOW, its other outputs are undefined.
 */
int linr_search_clauses_prefilter(const linr_index*, const void* Q, const float* q_scale, uint32_t B, uint32_t m,
                                  const uint64_t* q_values, const uint8_t* q_counts, uint32_t q_width, uint32_t k,
                                  uint32_t* out_ids, float* out_scores, int32_t* out_raw, uint32_t* out_counts,
                                  void* workspace, uint64_t workspace_bytes, void* hip_stream);

/*
 * Live updates (Sec. 4 "Model Live Update": Upsert and Delete calls on columns that are
 * pre-allocated larger than the initial index, a high-water mark for the working set, and
 * updates that run next to searches; their cost for searches is the subject of Sec. 5.3,
 * "Impact of Live Model Update on Inference").
 *
 * An item lives in a slot; the slot number is the id a search returns (the mapping from
 * document keys to slots belongs to the caller's ingestor).  The index holds `capacity`
 * slots (linr_index_create); slots [0, n) below the high-water mark n are scanned.
 *
 * linr_index_enable_updates  call once after a load.  From then on bit 31 of every item
 *     mask belongs to the library (set = the slot holds no item) and 31 attribute bits
 *     remain: LINR_E_FILTER if a resident mask carries bit 31.  A filter that requires
 *     bit 31 matches nothing.  Library-owned columns already span the capacity; borrowed
 *     columns (LINR_SRC_DEVICE_BORROW) must do so too -- updates write into them.
 *     linr_search_workspace_bytes then answers for a full index.  A later load ends it.
 * linr_index_upsert  writes `count` items into the given slots (host array, distinct,
 *     each < capacity; LINR_E_CAPACITY / LINR_E_SHAPE otherwise): emb [count][d] (codes
 *     [count][W] for LINR_BITS), mask, and row_scale / ts where the index has them, host
 *     (src == LINR_SRC_HOST; copied before the call returns) or device (any other value;
 *     read when the stream gets there).  Bit 31 of the new masks is ignored.  The slot may
 *     be fresh, deleted or live.  The mark rises to max(slot) + 1; skipped slots below it
 *     stay empty.  Codes made by linr_index_build_bits are refreshed for the new rows.
 * linr_index_delete  marks the slots (host array, each below the mark) as empty; a slot
 *     that is already empty stays so.
 * linr_index_sync_updates  waits for every enqueued update and publishes the mark.
 *
 * Both calls only enqueue work on `hip_stream` (a copy from a pinned staging area and a
 * few small kernels) and return; they wait only for the previous update, whose staging
 * area they reuse.  Any number of host threads may search while one thread at a time
 * updates (updaters are serialised by a lock; searches take a lock for a few loads only).
 * Visibility: a search enqueued on the update's own stream sees it (stream order).  For
 * searches on other streams a delete takes effect when its kernel runs (one atomic word
 * per slot), and items upserted into slots at or above the published mark appear, whole,
 * in searches enqueued after the update has finished on the device: the mark is published
 * by the first call that finds the update's event complete.  Rewriting a slot below the
 * published mark -- a live one, or a DELETED one that is being recycled -- while searches on
 * other streams are running is not atomic: the writer stores the row first and the mask
 * last, but nothing orders a reader's loads of the two against them across streams, so
 * such a search may pair the slot's new mask with its old row.  Give new versions fresh slots (at or above the mark) and
 * delete the old ones; recycle deleted slots from the searches' own stream, or while no
 * search is in flight.
 * Errors: LINR_E_STATE (updates not enabled), LINR_E_NULL, LINR_E_CAPACITY, LINR_E_SHAPE,
 * LINR_E_HIP.
 */
int linr_index_enable_updates(linr_index*);
int linr_index_upsert(linr_index*, const uint32_t* slots, uint32_t count, const void* emb, const float* row_scale,
                      const uint32_t* mask, const uint32_t* ts, int src, void* hip_stream);
int linr_index_delete(linr_index*, const uint32_t* slots, uint32_t count, void* hip_stream);
int linr_index_sync_updates(linr_index*);

/* number of items currently resident (the published high-water mark) / element type / dimensions */
int linr_index_info(const linr_index*, uint64_t* n, uint32_t* d, int* dtype, int* has_ts, int* has_row_scale);

const char* linr_strerror(int code);
/* hipError_t value of the last failing HIP call on this thread (0 if none) */
int linr_last_hip_error(void);

/*
 * Launch-shape knobs for tests and tuning (process-wide; 0 = library default).
 *   sample_ratio   : factor between the item counts covered after successive early
 *                    sweeps (power of two >= 2);
 *   min_sample     : smallest first sweep, in items;
 *   blocks_per_cu  : persistent workgroups per compute unit for the scan;
 *   max_levels     : upper bound on the number of sweeps (1 = single full sweep);
 *   force_generic  : 1 = always use the kernel that streams queries from LDS (searches over 1-bit codes: always
 *                    the matrix-core bit-matching kernel);
 *   max_qg         : cap on the 16-query groups one wave keeps in registers (larger
 *                    batches are then split over several waves per chunk);
 *   no_coop        : 1 = never use the workgroup-cooperative scan kernel (1-bit codes: always the popcount kernel);
 *   coop_min_groups: use that kernel for batches of more than this many 16-query groups;
 *   no_top_split   : 1 = do not split the last sweep into the finer 1/8, 3/8, 1/2 sweeps;
 *   prefilter_phases: 2 or 3 = the explicit pre-filtering searches take that many phases (1/16 of the items, the
 *                    rest; or 1/256, 15/256, the rest) whatever the index size; 0 = three from 2^26 items on;
 *   two_stage_rank_max: linr_search_two_stage ranks its candidates (linr_search_bits + re-scoring kernel) up to this
 *                    T and takes the selection path (linr_select_bits + gather scoring) above it; 0 = 999;
 *   wide_min_batch : use the 32x32-tile kernel (int8, m = 1, rows of 64 / 128 / 256 bytes) for batches of at
 *                    least this many queries; 0 = never (the default: it does not beat the other kernels yet);
 *   no_dense       : 1 = never use the large-batch kernels (int8 rows of exactly 64 bytes or bf16 rows of 256 bytes with
 *                    m = 1: the default for batches of 65 queries or more; bf16 rows of 128 bytes with m = 8: from 24
 *                    queries on), so that the older kernels can still be exercised;
 *   dense_min_batch: use those kernels from this batch size on; 0 = 65 (m = 8: 24);
 *   dense_groups   : 16-query groups a wave of that kernel keeps in registers (4, 8 or 16); 0 = chosen by batch size.
 *   top_ratios     : factors of the last sweeps when they are split, one hexadecimal digit each (2, 4 or 8), the
 *                    last sweep's in the lowest digit: 0x442 = the last sweep visits 1/2 of the chunks, the one before
 *                    3/8, the one before that 3/32; 0 = chosen by batch size.
 *   prefilter_table_min: the explicit pre-filtering searches evaluate the all / none clauses of a group of queries by
 *                    table look-up (one AND of four entries per item, whatever the number of queries) from this many
 *                    queries per group on, query by query below; 0 = 6, 33 or more = never.
 *   select_seg_items: items per segment of the large-K selection (4096, 16384 or 65536; one workgroup counts a segment
 *                    for up to eight queries); 0 = chosen from the capacity, the batch and the code length.
 * The settings are process-wide and read by every search while it plans its launches: change them only while no
 * other thread is inside a call of this library.
 */
typedef struct {
    uint32_t sample_ratio, min_sample, blocks_per_cu, max_levels, force_generic, max_qg, no_coop, coop_min_groups;
    uint32_t no_top_split, prefilter_phases, wide_min_batch, two_stage_rank_max;
    uint32_t no_dense, dense_min_batch, dense_groups, top_ratios, prefilter_table_min, select_seg_items;
} linr_tuning;
int linr_set_tuning(const linr_tuning*);

/*
 * Per-stage timing of a search, for benchmarks (Sec. 5.3 reports latency per batch;
 * this breaks one batch down by launch).  `events` holds 2 * LINR_MAX_STAGES
 * hipEvent_t made by linr_events_create; stage s of this search records
 * events[2s] / events[2s+1] around its launch on the search stream.  Nothing is
 * synchronised: read the times with linr_events_elapsed_ms after the stream has
 * finished.  *n_stages receives the number of stages, kinds[s] a LINR_STAGE_* value
 * and stage_items[s] the number of items a scan stage visits.
 */
#define LINR_MAX_STAGES 160
enum { LINR_STAGE_INIT = 0, LINR_STAGE_SCAN = 1, LINR_STAGE_MERGE = 2, LINR_STAGE_FILTER = 3 };
int linr_search_filtered_timed(const linr_index*, const void* Q, const float* q_scale, uint32_t B, uint32_t m,
                         const linr_filter* filters, uint32_t k,
                         uint32_t* out_ids, float* out_scores, int32_t* out_raw, uint32_t* out_counts,
                         void* workspace, uint64_t workspace_bytes, void* hip_stream, uint32_t flags,
                         void** events, uint32_t* n_stages, uint32_t* kinds, uint64_t* stage_items);
/* the same per-stage timing for linr_search_bits (Sec. 3.2) */
int linr_search_bits_timed(const linr_index*, const uint64_t* qbits, uint32_t B, const linr_filter* filters, uint32_t T,
                           uint32_t* out_ids, int32_t* out_matches, uint32_t* out_counts,
                           void* workspace, uint64_t workspace_bytes, void* hip_stream, uint32_t flags,
                           void** events, uint32_t* n_stages, uint32_t* kinds, uint64_t* stage_items);
/* ... and for linr_search_clauses (LINR_STAGE_FILTER = the pass over the clause columns) */
int linr_search_clauses_timed(const linr_index*, const void* Q, const float* q_scale, uint32_t B, uint32_t m,
                              const uint64_t* q_values, const uint8_t* q_counts, uint32_t q_width, uint32_t k,
                              uint32_t* out_ids, float* out_scores, int32_t* out_raw, uint32_t* out_counts,
                              void* workspace, uint64_t workspace_bytes, void* hip_stream,
                              void** events, uint32_t* n_stages, uint32_t* kinds, uint64_t* stage_items);
/* hipEvent_t helpers for callers without direct access to the HIP runtime (host arrays) */
int linr_events_create(void** events, uint32_t n);
int linr_events_destroy(void** events, uint32_t n);
/* ms[i] = time from events[2i] to events[2i+1], i < n_pairs; the events must have completed */
int linr_events_elapsed_ms(void** events, uint32_t n_pairs, float* ms);

#ifdef __cplusplus
}
#endif
#endif
