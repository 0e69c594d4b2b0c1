/*
 * linr_oracle_bits.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * Plain CPU statement of the quantised search of LiNR (arXiv 2407.13218, Sec. 3.2
 * "Quantized KNN" and its figure "KNN with Quantized Filtering"):
 *
 *   1. Sign-OPORP: an embedding is compressed to k_bits one-bit values.  The paper names
 *      the construction (one permutation, one random projection, fixed-length bins, then
 *      the sign) and cites the OPORP paper for it; written out here as
 *          sketch[j] = sum_{t=0}^{L-1} signs[j*L+t] * x[perm[j*L+t]],   L = D / k_bits,
 *          bit[j]    = 1 if sketch[j] > 0 else 0,
 *      with `perm` a permutation of 0..D-1 and `signs` in {-1,+1}, both drawn once by the
 *      caller and shared by items and queries.  The sum runs in double precision, t
 *      ascending (the inputs are fp32 or bf16 values, exactly representable).  Bit j
 *      lives at position j%64 (least significant first) of 64-bit word j/64.
 *      More bits than coordinates (Sec. 5.3.1 reports 512-bit codes of 128-dimensional
 *      embeddings): the construction is repeated with R independent draws of (perm, signs),
 *      each giving k_bits / R bits from bins of L = D * R / k_bits coordinates; the code is the
 *      draws' codes one after the other, bit r * (k_bits / R) + j = bit j of draw r.
 *   2. Bit-wise matching: similarity of two codes = number of equal bits
 *      = k_bits - popcount(a XOR b).
 *   3. Quantised KNN with pre-filtering: among the items that satisfy the query's clauses
 *      (the rule of Sec. 3.1.1, shared with the exact search), the T items with the most
 *      matching bits; ties go to the lower id.
 *   The second stage of the figure (full-precision scores of those T items, then top-K)
 *   is composed in oracle/linr_oracle.py from this file and the exact oracle's pair scorer.
 *
 * Readings (the paper is silent): bit = 1 for a strictly positive bin sum (a zero sum gives
 * 0); D must be a multiple of the bits per draw; ties by ascending id; codes longer than D bits
 * come from repeating the construction with independent draws (the OPORP paper's repetition),
 * concatenated in draw order.
 *
 * This file shares no code with the HIP library.  Every function is pinned by
 * tests/test_oracle_bits_pins.py (hand-worked example, projection-matrix form in numpy,
 * closed forms, the angle law of sign projections, brute force), so the header has no
 * "parity unpinned" entry.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    uint32_t all_bits, none_bits, any_bits[4], n_any, ts_min, ts_max, pad_;
} bits_filter;

/* the exact oracle's feasibility rule (linr_oracle.c), linked from the same shared object */
int linr_oracle_pass(const void* f, uint32_t mask, int has_ts, uint32_t ts);

/* x: [n][D] doubles; out: [n][k_bits/64 rounded up] words.  Returns 0, or -1 on a bad shape. */
int linr_oracle_sign_oporp(const double* x, uint64_t n, uint32_t D, const uint32_t* perm, const int8_t* signs,
                           uint32_t k_bits, uint64_t* out)
{
    if (k_bits == 0 || D % k_bits != 0) return -1;
    const uint32_t L = D / k_bits, W = (k_bits + 63) / 64;
    for (uint64_t i = 0; i < n; ++i) {
        const double* row = x + (size_t)i * D;
        uint64_t* o = out + (size_t)i * W;
        for (uint32_t w = 0; w < W; ++w) o[w] = 0;
        for (uint32_t j = 0; j < k_bits; ++j) {
            double s = 0.0;
            for (uint32_t t = 0; t < L; ++t) {
                double v = row[perm[j * L + t]];
                s = s + (signs[j * L + t] > 0 ? v : -v);
            }
            if (s > 0.0) o[j / 64] |= (uint64_t)1 << (j % 64);
        }
    }
    return 0;
}

/* The same with `reps` independent draws: perm and signs are [reps][D]; k_bits = reps * k1 with D a multiple of k1.
   Returns 0, or -1 on a bad shape. */
int linr_oracle_sign_oporp_rep(const double* x, uint64_t n, uint32_t D, const uint32_t* perm, const int8_t* signs,
                               uint32_t k_bits, uint32_t reps, uint64_t* out)
{
    if (reps == 0 || k_bits == 0 || k_bits % reps != 0) return -1;
    const uint32_t k1 = k_bits / reps;
    if (D % k1 != 0) return -1;
    const uint32_t L = D / k1, W = (k_bits + 63) / 64;
    for (uint64_t i = 0; i < n; ++i) {
        const double* row = x + (size_t)i * D;
        uint64_t* o = out + (size_t)i * W;
        for (uint32_t w = 0; w < W; ++w) o[w] = 0;
        for (uint32_t r = 0; r < reps; ++r) {
            const uint32_t* pr = perm + (size_t)r * D;
            const int8_t* sr = signs + (size_t)r * D;
            for (uint32_t j = 0; j < k1; ++j) {
                double s = 0.0;
                for (uint32_t t = 0; t < L; ++t) {
                    double v = row[pr[j * L + t]];
                    s = s + (sr[j * L + t] > 0 ? v : -v);
                }
                const uint32_t bit = r * k1 + j;
                if (s > 0.0) o[bit / 64] |= (uint64_t)1 << (bit % 64);
            }
        }
    }
    return 0;
}

static uint32_t popcount64(uint64_t v)
{
    uint32_t c = 0;
    while (v) { v &= v - 1; ++c; }
    return c;
}

/* number of equal bits of two codes of W words holding k_bits bits (unused high bits are zero in both) */
uint32_t linr_oracle_bit_matches(const uint64_t* a, const uint64_t* b, uint32_t W, uint32_t k_bits)
{
    uint32_t diff = 0;
    for (uint32_t w = 0; w < W; ++w) diff += popcount64(a[w] ^ b[w]);
    return k_bits - diff;
}

typedef struct { int32_t matches; uint64_t id; } bcand_t;

static int bcand_cmp(const void* pa, const void* pb)
{
    const bcand_t* a = (const bcand_t*)pa;
    const bcand_t* b = (const bcand_t*)pb;
    if (a->matches != b->matches) return a->matches > b->matches ? -1 : 1;
    if (a->id != b->id) return a->id < b->id ? -1 : 1;
    return 0;
}

/*
 * bits [n][W], qbits [B][W]; out_ids / out_matches [B][T] (padding 0xFFFFFFFF / INT32_MIN), out_counts [B].
 * Item i is reported as id_base + i.
 */
int linr_oracle_bits_search(const uint64_t* bits, uint32_t W, uint32_t k_bits, const uint32_t* mask, const uint32_t* ts,
                            uint64_t n, uint64_t id_base, const uint64_t* qbits, uint32_t B, const bits_filter* filters,
                            uint32_t T, uint32_t* out_ids, int32_t* out_matches, uint32_t* out_counts)
{
    bcand_t* c = (bcand_t*)malloc((size_t)(n ? n : 1) * sizeof(bcand_t));
    if (!c) return -1;
    for (uint32_t b = 0; b < B; ++b) {
        uint64_t m = 0;
        for (uint64_t i = 0; i < n; ++i) {
            if (!linr_oracle_pass(&filters[b], mask[i], ts != NULL, ts ? ts[i] : 0)) continue;
            c[m].matches = (int32_t)linr_oracle_bit_matches(bits + (size_t)i * W, qbits + (size_t)b * W, W, k_bits);
            c[m].id = id_base + i;
            ++m;
        }
        qsort(c, (size_t)m, sizeof(bcand_t), bcand_cmp);
        uint32_t cnt = m < T ? (uint32_t)m : T;
        out_counts[b] = cnt;
        for (uint32_t j = 0; j < T; ++j) {
            out_ids[(size_t)b * T + j] = j < cnt ? (uint32_t)c[j].id : 0xFFFFFFFFu;
            out_matches[(size_t)b * T + j] = j < cnt ? c[j].matches : INT32_MIN;
        }
    }
    free(c);
    return 0;
}
