/*
 * CPU oracle for the frequency-ranked draft LM head (FR-Spec, Section 3.2).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code with the HIP path and is
 * never called by it; only the tests, the smoke check and the benchmark's
 * cpu_baseline leg link it.
 *
 * What it computes, in the paper's notation:
 *   Eq. 3   W~[i,:] = W[V_high[i],:]                       oracle_build_subset
 *   Eq. 4   D_FR(x) = Softmax(H_D(x) W~^T), over the subset only
 *   Eq. 2   D(x)    = Softmax(H_D(x) W^T), the uncompressed head
 * followed by the per-row candidate selection the beam search of Section 2
 * consumes (the k most probable tokens of each row) and by the translation of
 * subset positions back to full-vocabulary ids (Section 3.2: verification and
 * the embedding keep the full vocabulary, so ids must be full-vocabulary ids).
 *
 * Readings where the paper is silent:
 *   - inputs are bf16 bit patterns, decoded exactly to fp32;
 *   - logits accumulate in fp32 in index order j = 0..d-1 (a bf16 x bf16
 *     product has at most 16 significant bits, so it is exact in fp32 and the
 *     only rounding is the running sum); an fp64 accumulation is provided as
 *     the "exact" value to bound that rounding;
 *   - log-sum-exp is taken in fp64 around the fp32 row maximum;
 *   - candidates are ordered by logit descending, equal logits by lower
 *     full-vocabulary id; the k outputs are in that order;
 *   - 0-based indices (Eq. 3 counts from 1).
 *
 * Every function returns 0 on success, a negative code on bad arguments.
 * All pointers are host pointers owned by the caller.
 */

#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_ID_RANGE (-2)
#define ORACLE_ERR_NOMEM (-3)

static inline float bf16_decode(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* Eq. 3: row gather in frequency-rank order, plus the position -> id table. */
int oracle_build_subset(const uint16_t *W_full, int64_t V, int64_t d,
                        const int32_t *freq_ranked_ids, int64_t V_sub,
                        uint16_t *W_sub, int32_t *idx_map) {
    if (!W_full || !freq_ranked_ids || !W_sub || !idx_map) return ORACLE_ERR_ARG;
    if (V < 1 || d < 1 || V_sub < 1 || V_sub > V) return ORACLE_ERR_ARG;
    for (int64_t i = 0; i < V_sub; ++i) {
        int64_t id = freq_ranked_ids[i];
        if (id < 0 || id >= V) return ORACLE_ERR_ID_RANGE;
    }
    for (int64_t i = 0; i < V_sub; ++i) {
        int64_t id = freq_ranked_ids[i];
        for (int64_t j = 0; j < d; ++j) W_sub[i * d + j] = W_full[id * d + j];
        idx_map[i] = (int32_t)id;
    }
    return ORACLE_OK;
}

/* z[m, i] = sum_j H[m, j] * W[i, j], fp32 running sum, j ascending.
 * z is [M, rows] row-major. */
int oracle_logits_f32(const uint16_t *H, int64_t M, int64_t d,
                      const uint16_t *W, int64_t rows, float *z) {
    if (!H || !W || !z || M < 1 || d < 1 || rows < 1) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        const uint16_t *w = W + i * d;
        for (int64_t m = 0; m < M; ++m) {
            const uint16_t *h = H + m * d;
            float acc = 0.0f;
            for (int64_t j = 0; j < d; ++j) acc += bf16_decode(h[j]) * bf16_decode(w[j]);
            z[m * rows + i] = acc;
        }
    }
    return ORACLE_OK;
}

/* Same sum carried in fp64 (no rounding that matters at these sizes). */
int oracle_logits_f64(const uint16_t *H, int64_t M, int64_t d,
                      const uint16_t *W, int64_t rows, double *z) {
    if (!H || !W || !z || M < 1 || d < 1 || rows < 1) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        const uint16_t *w = W + i * d;
        for (int64_t m = 0; m < M; ++m) {
            const uint16_t *h = H + m * d;
            double acc = 0.0;
            for (int64_t j = 0; j < d; ++j)
                acc += (double)bf16_decode(h[j]) * (double)bf16_decode(w[j]);
            z[m * rows + i] = acc;
        }
    }
    return ORACLE_OK;
}

/* log of Eq. 4's Softmax, row by row over all `rows` entries:
 * logZ = mx + log(sum_i exp(z_i - mx)), logp_i = z_i - logZ.
 * logp may be NULL (only logZ wanted); logZ may be NULL. */
int oracle_log_softmax(const float *z, int64_t M, int64_t rows,
                       float *logp, double *logZ) {
    if (!z || M < 1 || rows < 1) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const float *zr = z + m * rows;
        float mx = zr[0];
        for (int64_t i = 1; i < rows; ++i)
            if (zr[i] > mx) mx = zr[i];
        double S = 0.0;
        for (int64_t i = 0; i < rows; ++i) S += exp((double)zr[i] - (double)mx);
        double lz = (double)mx + log(S);
        if (logZ) logZ[m] = lz;
        if (logp)
            for (int64_t i = 0; i < rows; ++i) logp[m * rows + i] = (float)((double)zr[i] - lz);
    }
    return ORACLE_OK;
}

typedef struct {
    float z;
    int32_t id;   /* full-vocabulary id */
    int32_t pos;  /* position in the row  */
} cand_t;

static int cand_before(const void *pa, const void *pb) {
    const cand_t *a = (const cand_t *)pa, *b = (const cand_t *)pb;
    if (a->z > b->z) return -1;
    if (a->z < b->z) return 1;
    if (a->id < b->id) return -1;
    if (a->id > b->id) return 1;
    return 0;
}

/* Order all `rows` entries of one logit row by (logit desc, id asc) and keep
 * the first k.  idx_map == NULL means position i is id i. */
static int topk_row(const float *zr, int64_t rows, const int32_t *idx_map, int32_t k,
                    int32_t *out_id, int32_t *out_pos) {
    cand_t *c = (cand_t *)malloc((size_t)rows * sizeof *c);
    if (!c) return ORACLE_ERR_NOMEM;
    for (int64_t i = 0; i < rows; ++i) {
        c[i].z = zr[i];
        c[i].id = idx_map ? idx_map[i] : (int32_t)i;
        c[i].pos = (int32_t)i;
    }
    qsort(c, (size_t)rows, sizeof *c, cand_before);
    for (int32_t j = 0; j < k; ++j) {
        out_id[j] = c[j].id;
        out_pos[j] = c[j].pos;
    }
    free(c);
    return ORACLE_OK;
}

/* Per-row top-k over precomputed logits.  sub_pos (nullable) receives the
 * position inside the row of each winner. */
int oracle_topk(const float *z, int64_t M, int64_t rows, const int32_t *idx_map,
                int32_t k, int32_t *token_ids, int32_t *sub_pos) {
    if (!z || !token_ids || M < 1 || rows < 1 || k < 1 || k > rows) return ORACLE_ERR_ARG;
    int status = ORACLE_OK;
#pragma omp parallel for schedule(dynamic)
    for (int64_t m = 0; m < M; ++m) {
        int32_t *pos = (int32_t *)malloc((size_t)k * sizeof *pos);
        if (!pos) {
#pragma omp critical
            status = ORACLE_ERR_NOMEM;
            continue;
        }
        int st = topk_row(z + m * rows, rows, idx_map, k, token_ids + m * k, pos);
        if (st != ORACLE_OK) {
#pragma omp critical
            status = st;
        } else if (sub_pos) {
            memcpy(sub_pos + m * k, pos, (size_t)k * sizeof *pos);
        }
        free(pos);
    }
    return status;
}

/* Eq. 4 + candidate selection + id translation.
 *   H        bf16 [M, d]
 *   W_sub    bf16 [V_sub, d]
 *   idx_map  int32 [V_sub] (NULL = identity)
 *   token_ids int32 [M, k] out, full-vocabulary ids, most probable first
 *   logp     fp32  [M, k] out, log-probability under the subset distribution
 *   z_out    fp32  [M, V_sub] out, nullable: all logits, for the parity tests */
int oracle_draft_topk(const uint16_t *H, int64_t M, int64_t d,
                      const uint16_t *W_sub, const int32_t *idx_map, int64_t V_sub,
                      int32_t k, int32_t *token_ids, float *logp, float *z_out) {
    if (!H || !W_sub || !token_ids || !logp) return ORACLE_ERR_ARG;
    if (M < 1 || d < 1 || V_sub < 1 || k < 1 || k > V_sub) return ORACLE_ERR_ARG;
    float *z = z_out ? z_out : (float *)malloc((size_t)M * (size_t)V_sub * sizeof(float));
    double *logZ = (double *)malloc((size_t)M * sizeof(double));
    int32_t *pos = (int32_t *)malloc((size_t)M * (size_t)k * sizeof(int32_t));
    int st = ORACLE_ERR_NOMEM;
    if (z && logZ && pos) {
        st = oracle_logits_f32(H, M, d, W_sub, V_sub, z);
        if (st == ORACLE_OK) st = oracle_log_softmax(z, M, V_sub, NULL, logZ);
        if (st == ORACLE_OK) st = oracle_topk(z, M, V_sub, idx_map, k, token_ids, pos);
        if (st == ORACLE_OK)
            for (int64_t m = 0; m < M; ++m)
                for (int32_t j = 0; j < k; ++j)
                    logp[m * k + j] = (float)((double)z[m * V_sub + pos[m * k + j]] - logZ[m]);
    }
    if (!z_out) free(z);
    free(logZ);
    free(pos);
    return st;
}

/* Eq. 2: the same operation on every row of W_full; position == id. */
int oracle_full_topk(const uint16_t *H, int64_t M, int64_t d,
                     const uint16_t *W_full, int64_t V, int32_t k,
                     int32_t *token_ids, float *logp, float *z_out) {
    return oracle_draft_topk(H, M, d, W_full, NULL, V, k, token_ids, logp, z_out);
}

int oracle_num_threads(void) {
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
