/*
 * frspec_dev.h - measurement and test surface of libfrspec, apart from the product calls of
 * frspec.h: knobs that force one kernel build or one merge path, an in-kernel phase trace,
 * and plain streaming kernels that calibrate hardware counters.  Nothing here is needed to
 * use the draft LM head; none of it follows from the paper.
 */
#ifndef FRSPEC_DEV_H
#define FRSPEC_DEV_H

#include "frspec.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Kernel-selection knobs for measurements and for tests that force one code path.
 * A zero in any field means "library default".
 */
typedef struct fr_tuning {
    int32_t path;        /* 3 = skinny kernel (M <= 16), products on the matrix cores (default),
                            1 = skinny kernel, products on the vector ALUs (bf16 dot2),
                            2 = matrix-core kernels for any M: the chunked kernel up to 64 rows of H,
                            the block kernel beyond (where it serves the shape) */
    int32_t two_launch;  /* 1 = merge the per-workgroup partials in a second launch instead
                            of inside the same launch */
    int32_t variant;     /* skinny kernel build variant, 1-based (waves x pipeline depth x unit) */
    int32_t ksplit;      /* waves that share one 16-row tile along d (1, 2, 4, 8) */
    int32_t grid;        /* number of workgroups (<= 512) */
    int32_t stream_only; /* 1 = measurement only: run the contraction and drop the logits
                            (no softmax, no top-k; token_ids / logp are left untouched) */
    int32_t skew;        /* > 0: rows that every odd workgroup hands to its even neighbour when each
                            workgroup has exactly one pass (experimental die balancing; off by default) */
    int32_t no_mailbox;  /* 1 = the chunked kernel merges through the plain partial arrays and the
                            arrival counter even where the result mailbox applies */
    int32_t spin_limit;  /* > 0: polls after which a wait for other workgroups' results is given up
                            (default: about a second).  Tests set 1 to see the time-out handling
                            with every kernel still ending normally */
    int32_t chunked_only; /* 1 = more than 64 rows of H also go to the chunked kernel, in slabs of up to
                            128 rows with one pass over W per slab (the path before the block kernel) */
    void *trace;         /* optional device buffer of 8 * 512 int64: every workgroup of a
                            contraction kernel records 100 MHz timestamps of its phases there */
} fr_tuning;

/* fr_draft_topk with explicit knobs (tuning == NULL behaves exactly like fr_draft_topk). */
fr_status fr_draft_topk_tuned(const void *H, int64_t M, int64_t d,
                              const void *W_sub, const int32_t *idx_map, int64_t V_sub,
                              int32_t k, int32_t *token_ids, float *logp,
                              void *workspace, size_t workspace_bytes, fr_stream stream,
                              const fr_tuning *tuning);

/* fr_draft_topk_tiled with explicit knobs (tuning == NULL behaves exactly like it). */
fr_status fr_draft_topk_tiled_tuned(const void *H, int64_t M, int64_t d, const void *W_tiled,
                                    const int32_t *idx_map, int64_t V_sub, int32_t k,
                                    int32_t *token_ids, float *logp, void *workspace,
                                    size_t workspace_bytes, fr_stream stream,
                                    const fr_tuning *tuning);

/*
 * Bandwidth calibration kernels: a plain copy and a plain read of `bytes` bytes
 * (multiple of 16), used to scale hardware counters and to report what a trivial
 * streaming kernel achieves on the same machine.  `sink` receives one 16-byte value
 * (only so that the read cannot be optimised away).
 */
fr_status fr_calib_copy(void *dst, const void *src, size_t bytes, fr_stream stream);
fr_status fr_calib_read(const void *src, size_t bytes, void *sink, fr_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* FRSPEC_DEV_H */
