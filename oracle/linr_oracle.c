/*
 * linr_oracle.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * Plain, slow CPU statement of what the retrieval hot path computes: for each
 * query, visit every item, keep the items that satisfy the query's attribute
 * clauses, score them against the query, sort ALL feasible items by
 * (score descending, item id ascending) and emit the first k.
 *
 * This file shares no code, header, table or helper with the HIP library.
 * Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may
 * load it.  It is never tuned: it is the definition, written out.
 *
 * What it follows (LiNR, arXiv 2407.13218):
 *   - Sec. 3.1.1 "KNN with Similarity Masking": the query embedding is scored
 *     against ALL item embeddings; an item is feasible iff EVERY clause of the
 *     query is satisfied; a clause holding several attributes is satisfied by
 *     ANY one of them; reverse clauses pass on mismatch.
 *   - Sec. 3.1.2 "KNN with Explicit Pre-Filtering": infeasible items are
 *     removed before scoring/top-K, so they can never occupy a result slot
 *     (the reading taken here; the masking variant's "score := 0" would let an
 *     infeasible item outrank a feasible one with a negative score).
 *   - Sec. 1 / Sec. 3.2: similarity is the dot product of (already normalised)
 *     embeddings; the search is exhaustive, hence exact.
 *   - Sec. 5.3.2: queries of one batch carry their own filters and are
 *     answered independently.
 * Not in the paper, fixed by this build's problem statement: attributes are a
 * 32-bit mask plus an optional 32-bit timestamp per item; int8 codes with one
 * fp32 scale per row and exact int32 accumulation; ties go to the lower id;
 * several embeddings per query aggregate by max.
 *
 * Arithmetic:
 *   int8 : raw = sum_j (int32)q[j]*(int32)x[j]            (exact)
 *          rank = raw                         if no row scale is given
 *          rank = (float)raw * row_scale[i]   one round-to-nearest fp32 product
 *          out_score = rank * q_scale[b]      one more fp32 product (winners only)
 *   bf16 : every bf16 is widened exactly to fp32; products and the running sum
 *          are fp32, j ascending, no fused multiply-add.
 *   fp32 : the same without widening.
 *   m > 1: rank uses max over the m embeddings of the query (raw for int8).
 *
 * Every function below is pinned by tests/test_oracle_*.py (hand-worked example,
 * numpy matmul + stable argsort, brute-force enumeration, invariants), so the
 * header has no "parity unpinned" entry.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#include <pthread.h>

#define ORACLE_F32 0
#define ORACLE_BF16 1
#define ORACLE_I8 2
#define ORACLE_MAX_ANY 4
#define ORACLE_NO_ID 0xFFFFFFFFu

/* One query's predicate; 40 bytes, same field order as the input generator writes. */
typedef struct {
    uint32_t all_bits;               /* single-attribute clauses: every bit must be present  */
    uint32_t none_bits;              /* reverse clauses: none of these bits may be present   */
    uint32_t any_bits[ORACLE_MAX_ANY]; /* multi-attribute clauses: at least one bit present   */
    uint32_t n_any;                  /* how many any_bits[] entries are in use               */
    uint32_t ts_min, ts_max;         /* inclusive timestamp window                            */
    uint32_t pad_;
} oracle_filter;

/* Sec. 3.1.1 feasibility rule over the bitmask / timestamp attribute space. */
int linr_oracle_pass(const oracle_filter* f, uint32_t mask, int has_ts, uint32_t ts)
{
    if ((mask & f->all_bits) != f->all_bits) return 0;
    if ((mask & f->none_bits) != 0) return 0;
    for (uint32_t g = 0; g < f->n_any && g < ORACLE_MAX_ANY; ++g)
        if ((mask & f->any_bits[g]) == 0) return 0;
    if (has_ts) {
        if (ts < f->ts_min) return 0;
        if (ts > f->ts_max) return 0;
    }
    return 1;
}

static float bf16_to_f32(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* fp32-accumulated dot product, j ascending (file is built with -ffp-contract=off). */
static float dot_f32(const float* q, const float* x, uint32_t d)
{
    float s = 0.0f;
    for (uint32_t j = 0; j < d; ++j) { float p = q[j] * x[j]; s = s + p; }
    return s;
}
static float dot_bf16(const uint16_t* q, const uint16_t* x, uint32_t d)
{
    float s = 0.0f;
    for (uint32_t j = 0; j < d; ++j) { float p = bf16_to_f32(q[j]) * bf16_to_f32(x[j]); s = s + p; }
    return s;
}
static int32_t dot_i8(const int8_t* q, const int8_t* x, uint32_t d)
{
    int32_t s = 0;
    for (uint32_t j = 0; j < d; ++j) s += (int32_t)q[j] * (int32_t)x[j];
    return s;
}

static size_t elt_size(int dtype) { return dtype == ORACLE_F32 ? 4 : dtype == ORACLE_BF16 ? 2 : 1; }

/* Score of one (query b, item i) pair.  *raw_out receives the int32 value for int8. */
static double pair_rank(int dtype, const void* emb, const float* row_scale, uint32_t d,
                        const void* Q, uint32_t m, uint32_t b, uint64_t i, int32_t* raw_out)
{
    size_t es = elt_size(dtype);
    const char* x = (const char*)emb + (size_t)i * d * es;
    if (dtype == ORACLE_I8) {
        int32_t best = INT32_MIN;
        for (uint32_t e = 0; e < m; ++e) {
            const int8_t* q = (const int8_t*)Q + ((size_t)b * m + e) * d;
            int32_t r = dot_i8(q, (const int8_t*)x, d);
            if (r > best) best = r;
        }
        *raw_out = best;
        if (row_scale) { float rf = (float)best * row_scale[i]; return (double)rf; }
        return (double)best;
    }
    float best = -INFINITY;
    for (uint32_t e = 0; e < m; ++e) {
        float r;
        if (dtype == ORACLE_F32) r = dot_f32((const float*)Q + ((size_t)b * m + e) * d, (const float*)x, d);
        else r = dot_bf16((const uint16_t*)Q + ((size_t)b * m + e) * d, (const uint16_t*)x, d);
        if (r > best) best = r;
    }
    *raw_out = 0;
    return (double)best;
}

typedef struct { double rank; uint64_t id; int32_t raw; } cand_t;

/* (rank descending, id ascending).  -0.0 == +0.0 here, so the id decides between them. */
static int cand_cmp(const void* a, const void* b)
{
    const cand_t* x = (const cand_t*)a;
    const cand_t* y = (const cand_t*)b;
    if (x->rank > y->rank) return -1;
    if (x->rank < y->rank) return 1;
    if (x->id < y->id) return -1;
    if (x->id > y->id) return 1;
    return 0;
}

typedef struct {
    int dtype; const void* emb; const float* row_scale; const uint32_t* mask; const uint32_t* ts;
    uint32_t d; const void* Q; uint32_t m; uint32_t b; const oracle_filter* f;
    uint64_t lo, hi;           /* item range of this worker */
    cand_t* out; size_t n_out, cap; int oom;
} work_t;

static void* scan_range(void* arg)
{
    work_t* w = (work_t*)arg;
    for (uint64_t i = w->lo; i < w->hi; ++i) {
        if (!linr_oracle_pass(w->f, w->mask[i], w->ts != NULL, w->ts ? w->ts[i] : 0)) continue;
        if (w->n_out == w->cap) {
            size_t nc = w->cap ? w->cap * 2 : 1024;
            cand_t* p = (cand_t*)realloc(w->out, nc * sizeof(cand_t));
            if (!p) { w->oom = 1; return NULL; }
            w->out = p; w->cap = nc;
        }
        cand_t c;
        c.rank = pair_rank(w->dtype, w->emb, w->row_scale, w->d, w->Q, w->m, w->b, i, &c.raw);
        c.id = i;
        w->out[w->n_out++] = c;
    }
    return NULL;
}

/*
 * Exhaustive filtered top-k.  All pointers are host memory.
 *   emb [n][d] row-major of dtype; row_scale [n] or NULL (int8 only); mask [n]; ts [n] or NULL
 *   Q [B][m][d] of dtype; q_scale [B] or NULL (int8 only; NULL = 1.0f)
 *   out_ids/out_scores/out_raw [B][k], out_counts [B]; out_raw may be NULL.
 *   id_base is added to the row index to form the reported id (for sharded use by tests).
 * Rows of the outputs beyond counts[b] are padded with NO_ID / -inf / INT32_MIN.
 * Returns 0, or -1 on bad arguments / out of memory.
 */
int linr_oracle_search(int dtype, const void* emb, const float* row_scale, const uint32_t* mask,
                       const uint32_t* ts, uint64_t n, uint32_t d, uint64_t id_base,
                       const void* Q, const float* q_scale, uint32_t B, uint32_t m,
                       const oracle_filter* filters, uint32_t k,
                       uint32_t* out_ids, float* out_scores, int32_t* out_raw, uint32_t* out_counts,
                       int nthreads)
{
    if (!mask || !Q || !filters || !out_ids || !out_scores || !out_counts) return -1;
    if (n > 0 && !emb) return -1;
    if (dtype < 0 || dtype > 2 || d == 0 || m == 0 || k == 0) return -1;
    if (nthreads < 1) nthreads = 1;
    if (nthreads > 256) nthreads = 256;
    for (uint32_t b = 0; b < B; ++b) {
        work_t w[256];
        pthread_t th[256];
        uint64_t per = (n + (uint64_t)nthreads - 1) / (uint64_t)nthreads;
        for (int t = 0; t < nthreads; ++t) {
            memset(&w[t], 0, sizeof(work_t));
            w[t].dtype = dtype; w[t].emb = emb; w[t].row_scale = row_scale; w[t].mask = mask; w[t].ts = ts;
            w[t].d = d; w[t].Q = Q; w[t].m = m; w[t].b = b; w[t].f = &filters[b];
            w[t].lo = per * (uint64_t)t < n ? per * (uint64_t)t : n;
            w[t].hi = per * (uint64_t)(t + 1) < n ? per * (uint64_t)(t + 1) : n;
        }
        if (nthreads == 1) scan_range(&w[0]);
        else {
            for (int t = 0; t < nthreads; ++t) pthread_create(&th[t], NULL, scan_range, &w[t]);
            for (int t = 0; t < nthreads; ++t) pthread_join(th[t], NULL);
        }
        size_t total = 0; int oom = 0;
        for (int t = 0; t < nthreads; ++t) { total += w[t].n_out; oom |= w[t].oom; }
        cand_t* all = (cand_t*)malloc((total ? total : 1) * sizeof(cand_t));
        if (!all) oom = 1;
        if (oom) { for (int t = 0; t < nthreads; ++t) free(w[t].out); free(all); return -1; }
        size_t p = 0;
        for (int t = 0; t < nthreads; ++t) {
            if (w[t].n_out) memcpy(all + p, w[t].out, w[t].n_out * sizeof(cand_t));
            p += w[t].n_out; free(w[t].out);
        }
        qsort(all, total, sizeof(cand_t), cand_cmp);      /* full sort of every feasible item */
        uint32_t cnt = total < (size_t)k ? (uint32_t)total : k;
        out_counts[b] = cnt;
        float qs = (dtype == ORACLE_I8 && q_scale) ? q_scale[b] : 1.0f;
        for (uint32_t j = 0; j < k; ++j) {
            size_t o = (size_t)b * k + j;
            if (j < cnt) {
                out_ids[o] = (uint32_t)(all[j].id + id_base);
                float rf = (float)all[j].rank;            /* exact: rank holds an fp32 or int32 value */
                out_scores[o] = (dtype == ORACLE_I8) ? rf * qs : rf;
                if (out_raw) out_raw[o] = (dtype == ORACLE_I8) ? all[j].raw : 0;
            } else {
                out_ids[o] = ORACLE_NO_ID;
                out_scores[o] = -INFINITY;
                if (out_raw) out_raw[o] = INT32_MIN;
            }
        }
        free(all);
    }
    return 0;
}

/*
 * Scores of listed (query, item) pairs, for spot checks at sizes where a full
 * scan is too slow.  pairs_b[p], pairs_i[p] -> rank[p] (the ranking value as a
 * double: fp32 or int32 exactly), raw[p] (int8), feasible[p] (0/1).
 */
int linr_oracle_pairs(int dtype, const void* emb, const float* row_scale, const uint32_t* mask,
                      const uint32_t* ts, uint32_t d, const void* Q, uint32_t m,
                      const oracle_filter* filters, uint64_t npairs, const uint32_t* pairs_b,
                      const uint64_t* pairs_i, double* rank, int32_t* raw, uint8_t* feasible)
{
    for (uint64_t p = 0; p < npairs; ++p) {
        uint64_t i = pairs_i[p]; uint32_t b = pairs_b[p];
        int32_t r = 0;
        rank[p] = pair_rank(dtype, emb, row_scale, d, Q, m, b, i, &r);
        if (raw) raw[p] = r;
        if (feasible) feasible[p] = (uint8_t)linr_oracle_pass(&filters[b], mask[i], ts != NULL, ts ? ts[i] : 0);
    }
    return 0;
}

/*
 * The same ranking value accumulated in fp64 (fp32 / bf16 only): used by tests to
 * show that the fp32 accumulation order of this oracle is far inside the 1e-3
 * tolerance the GPU path is held to.
 */
double linr_oracle_dot_f64(int dtype, const void* q, const void* x, uint32_t d)
{
    double s = 0.0;
    for (uint32_t j = 0; j < d; ++j) {
        double a, b;
        if (dtype == ORACLE_F32) { a = ((const float*)q)[j]; b = ((const float*)x)[j]; }
        else if (dtype == ORACLE_BF16) { a = bf16_to_f32(((const uint16_t*)q)[j]); b = bf16_to_f32(((const uint16_t*)x)[j]); }
        else { a = ((const int8_t*)q)[j]; b = ((const int8_t*)x)[j]; }
        s += a * b;
    }
    return s;
}
