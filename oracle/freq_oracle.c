/*
 * CPU oracle for the step before the draft LM head: corpus-level token statistics
 * (Section 3.2, "Corpus-Level Token Statistics": token frequencies are counted over a
 * tokenised corpus, and the high-frequency subset V_high is taken from the ranking).
 *
 * TEST INFRASTRUCTURE ONLY: plain loops and qsort; shares nothing with the HIP path.
 *
 *   oracle_count_tokens  counts[t] += number of occurrences of t in the stream; ids outside
 *                        [0, V) are skipped and reported through *n_bad
 *   oracle_rank_tokens   the V ids ordered by count descending; equal counts by lower id
 *                        (the paper does not say how ties are ordered; this is the reading
 *                        the synthetic rankings of this build already use)
 */

#include <stdint.h>
#include <stdlib.h>

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_NOMEM (-2)

int oracle_count_tokens(const int32_t *tokens, int64_t n, int64_t V, int64_t *counts, int64_t *n_bad) {
    if ((!tokens && n > 0) || !counts || n < 0 || V < 1) return ORACLE_ERR_ARG;
    int64_t bad = 0;
    for (int64_t i = 0; i < n; ++i) {
        const int32_t t = tokens[i];
        if (t < 0 || t >= V) ++bad;
        else ++counts[t];
    }
    if (n_bad) *n_bad = bad;
    return ORACLE_OK;
}

typedef struct {
    int64_t count;
    int32_t id;
} counted_t;

static int more_frequent_first(const void *pa, const void *pb) {
    const counted_t *a = (const counted_t *)pa, *b = (const counted_t *)pb;
    if (a->count > b->count) return -1;
    if (a->count < b->count) return 1;
    return a->id < b->id ? -1 : (a->id > b->id ? 1 : 0);
}

int oracle_rank_tokens(const int64_t *counts, int64_t V, int32_t *freq_ranked_ids) {
    if (!counts || !freq_ranked_ids || V < 1 || V > INT32_MAX) return ORACLE_ERR_ARG;
    counted_t *c = (counted_t *)malloc((size_t)V * sizeof *c);
    if (!c) return ORACLE_ERR_NOMEM;
    for (int64_t t = 0; t < V; ++t) {
        c[t].count = counts[t];
        c[t].id = (int32_t)t;
    }
    qsort(c, (size_t)V, sizeof *c, more_frequent_first);
    for (int64_t i = 0; i < V; ++i) freq_ranked_ids[i] = c[i].id;
    free(c);
    return ORACLE_OK;
}
