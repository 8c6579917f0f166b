/*
 * CPU oracle for the draft-step glue around the draft LM head: the beam-search
 * expansion of one draft step and the final selection of the draft tree
 * (Section 2, "EAGLE-2 adopts a beam-search algorithm ... select the top K
 * probability tokens from the beam search history ... tree attention mask ...
 * each token can only see tokens in its ancestral path").
 *
 * TEST INFRASTRUCTURE ONLY, like the rest of this directory: plain C, sorts by
 * qsort, walks parent chains one link at a time; shares nothing with the HIP
 * path and is called only by the tests.
 *
 * The objects, as this build reads the paper (it names the steps, not the data
 * structures):
 *   beam search history  a growing list of candidates; entry i has a cumulative
 *                        log-probability score[i] (sum of the log-probabilities on
 *                        the path from the prompt), a token[i], and parent[i] = the
 *                        history index of the candidate it extends (-1: it extends
 *                        the prompt itself).
 *   one draft step       the M current nodes (score node_score[m], history index
 *                        node_hist[m], -1 at the first step) each receive k
 *                        candidates (token_ids[m][j], logp[m][j]) from the draft LM
 *                        head.  All M*k of them join the history, in row-major
 *                        order c = m*k + j, with score node_score[m] + logp[m][j]
 *                        (one fp32 addition).  The `width` best (score descending,
 *                        equal scores by lower c) are the nodes of the next step.
 *   the draft            after `depth` steps, the K best history entries (score
 *                        descending, equal scores by lower history index), listed in
 *                        ascending history index.  A log-probability is <= 0 and a
 *                        child is appended after its parent, so every ancestor of a
 *                        selected entry is selected too and precedes it.
 *   tree mask            mask[p][q] = 1 iff q == p or the entry at position q is an
 *                        ancestor of the entry at position p (the prompt prefix,
 *                        visible to all, is not part of the mask).
 *
 * Every function returns 0 on success, a negative code on bad arguments.
 */

#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_NOMEM (-2)

typedef struct {
    float score;
    int64_t index;
} ranked_t;

/* score descending, equal scores by lower index */
static int ranked_before(const void *pa, const void *pb) {
    const ranked_t *a = (const ranked_t *)pa, *b = (const ranked_t *)pb;
    if (a->score > b->score) return -1;
    if (a->score < b->score) return 1;
    if (a->index < b->index) return -1;
    if (a->index > b->index) return 1;
    return 0;
}

static int index_ascending(const void *pa, const void *pb) {
    const int64_t a = ((const ranked_t *)pa)->index, b = ((const ranked_t *)pb)->index;
    return a < b ? -1 : (a > b ? 1 : 0);
}

int oracle_beam_expand(const float *logp, const int32_t *token_ids, int64_t M, int32_t k,
                       const float *node_score, const int32_t *node_hist, int32_t width,
                       float *hist_score, int32_t *hist_token, int32_t *hist_parent,
                       int64_t hist_offset,
                       float *next_score, int32_t *next_token, int32_t *next_hist) {
    if (!logp || !token_ids || !node_score || !node_hist || !hist_score || !hist_token ||
        !hist_parent || !next_score || !next_token || !next_hist)
        return ORACLE_ERR_ARG;
    if (M < 1 || k < 1 || width < 1 || (int64_t)width > M * k || hist_offset < 0) return ORACLE_ERR_ARG;
    const int64_t C = M * k;
    ranked_t *r = (ranked_t *)malloc((size_t)C * sizeof *r);
    if (!r) return ORACLE_ERR_NOMEM;
    for (int64_t m = 0; m < M; ++m)
        for (int32_t j = 0; j < k; ++j) {
            const int64_t c = m * k + j;
            const float s = node_score[m] + logp[c];
            hist_score[hist_offset + c] = s;
            hist_token[hist_offset + c] = token_ids[c];
            hist_parent[hist_offset + c] = node_hist[m];
            r[c].score = s;
            r[c].index = c;
        }
    qsort(r, (size_t)C, sizeof *r, ranked_before);
    for (int32_t w = 0; w < width; ++w) {
        const int64_t c = r[w].index;
        next_score[w] = r[w].score;
        next_token[w] = token_ids[c];
        next_hist[w] = (int32_t)(hist_offset + c);
    }
    free(r);
    return ORACLE_OK;
}

int oracle_tree_select(const float *hist_score, const int32_t *hist_token,
                       const int32_t *hist_parent, int64_t N, int32_t K,
                       int32_t *sel_index, int32_t *sel_token, int32_t *sel_parent,
                       int32_t *sel_depth, uint8_t *tree_mask) {
    if (!hist_score || !hist_token || !hist_parent || !sel_index || !sel_token || !sel_parent ||
        !sel_depth || !tree_mask)
        return ORACLE_ERR_ARG;
    if (N < 1 || K < 1 || (int64_t)K > N) return ORACLE_ERR_ARG;
    for (int64_t i = 0; i < N; ++i)
        if (hist_parent[i] < -1 || hist_parent[i] >= i) return ORACLE_ERR_ARG;   /* parents come first */
    ranked_t *r = (ranked_t *)malloc((size_t)N * sizeof *r);
    if (!r) return ORACLE_ERR_NOMEM;
    for (int64_t i = 0; i < N; ++i) {
        r[i].score = hist_score[i];
        r[i].index = i;
    }
    qsort(r, (size_t)N, sizeof *r, ranked_before);
    qsort(r, (size_t)K, sizeof *r, index_ascending);   /* the K best, in history order */
    memset(tree_mask, 0, (size_t)K * (size_t)K);
    for (int32_t p = 0; p < K; ++p) {
        const int64_t i = r[p].index;
        sel_index[p] = (int32_t)i;
        sel_token[p] = hist_token[i];
        /* position of the parent inside the selection: -1 = the prompt, -2 = not selected
         * (cannot happen while a child never scores above its parent) */
        sel_parent[p] = hist_parent[i] < 0 ? -1 : -2;
        for (int32_t q = 0; q < p; ++q)
            if (r[q].index == hist_parent[i]) sel_parent[p] = q;
    }
    for (int32_t p = 0; p < K; ++p) {
        int32_t depth = 0;
        tree_mask[(size_t)p * K + p] = 1;
        for (int32_t q = sel_parent[p]; q >= 0; q = sel_parent[q]) {   /* up the ancestral path */
            tree_mask[(size_t)p * K + q] = 1;
            ++depth;
        }
        sel_depth[p] = depth;
    }
    free(r);
    return ORACLE_OK;
}
