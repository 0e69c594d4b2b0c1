/*
 * linr_oracle_clauses.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * Plain CPU statement of attribute-based matching over clause lists as LiNR describes it
 * (arXiv 2407.13218, Sec. 3.1.1 "KNN with Similarity Masking" and its figure; the benchmark
 * datasets of Sec. 5.3 use it with one 64-bit attribute per clause):
 *
 *   - there are C clauses (e.g. geo-location, company name, job title);
 *   - item i carries, for clause c, a list of attributes (64-bit ids) of length
 *     counts[i][c]; all lists of an item sit back to back, clause 0 first, in row i of one
 *     values matrix [n][row_width] (the "single matrix" plus "counting matrix" of the paper:
 *     no index vector is needed because a row has a fixed width; unused tail entries are
 *     ignored);
 *   - a query carries a list per clause in the same layout, [B][q_width] + q_counts[B][C];
 *   - a clause is satisfied when at least one attribute of the item's list equals one of the
 *     query's list; a REVERSE clause (bit c of `reverse`) is satisfied when none does;
 *   - an item is feasible when every clause is satisfied.
 *   Reading (the paper is silent): a clause for which the query lists no attribute places no
 *   constraint, whether reverse or not.  Lists are sorted in the paper's storage so that a
 *   kernel may stop early; the rule itself does not depend on the order and this file does
 *   not assume it.
 *
 * The search itself is the exhaustive oracle of linr_oracle.c run over the feasible items
 * (composed in oracle/linr_oracle.py).  Pinned by tests/test_oracle_clauses_pins.py.
 */
#include <stdint.h>
#include <stddef.h>

/* feasible[i] = 1 / 0 for the n items against ONE query (qv: its values row, qc: its C counts) */
int linr_oracle_clause_feasible(const uint64_t* values, uint32_t row_width, const uint8_t* counts, uint32_t C, uint64_t n,
                                const uint64_t* qv, const uint8_t* qc, uint32_t reverse, uint8_t* feasible)
{
    for (uint64_t i = 0; i < n; ++i) {
        const uint64_t* row = values + (size_t)i * row_width;
        const uint8_t* cnt = counts + (size_t)i * C;
        uint32_t io = 0, qo = 0;
        int ok = 1;
        for (uint32_t c = 0; c < C; ++c) {
            int match = 0;
            for (uint32_t a = 0; a < cnt[c]; ++a)
                for (uint32_t b = 0; b < qc[c]; ++b)
                    if (row[io + a] == qv[qo + b]) match = 1;
            if (qc[c] != 0) {
                const int want_match = ((reverse >> c) & 1u) == 0;
                if (match != want_match) ok = 0;
            }
            io += cnt[c];
            qo += qc[c];
        }
        if (io > row_width) return -1;          /* counts of an item exceed its row */
        feasible[i] = (uint8_t)ok;
    }
    return 0;
}
