/*
 * frspec.h - C ABI of the frequency-ranked draft LM head for AMD MI355X (gfx950).
 *
 * The operations are those of FR-Spec, Section 3.2:
 *   Eq. 3  build the sub-matrix W~ whose i-th row is row V_high[i] of W_LM;
 *   Eq. 4  draft distribution Softmax(H_D W~^T), normalised over the subset;
 *   Eq. 2  the uncompressed draft distribution Softmax(H_D W_LM^T);
 * followed by the per-row selection of the k most probable tokens that the
 * EAGLE-2 beam search of Section 2 consumes, reported as full-vocabulary ids
 * (Section 3.2: only drafting is restricted, verification keeps the full
 * vocabulary, so every id that leaves the draft head is a full-vocabulary id).
 *
 * Conventions common to every call
 *   - All data pointers are DEVICE pointers into memory owned by the caller.
 *     The library allocates nothing and frees nothing (one exception, a model-load step:
 *     fr_rank_tokens, see there).  Per-call state lives in the
 *     caller's workspace; what the library itself keeps, per device and for the life of
 *     the process, is the result of a one-time set-up (number of compute units, raised
 *     LDS limits of its kernels): see fr_init.
 *   - bf16 tensors are row-major arrays of 16-bit patterns, 16-byte aligned.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream) and the call returns without synchronising.  Outputs
 *     are valid once the stream has been synchronised.
 *   - Argument errors are detected on the host before anything is launched and
 *     reported through the return value; nothing is thrown, nothing aborts.
 *   - Indices are 0-based.
 */
#ifndef FRSPEC_H
#define FRSPEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int fr_status;
typedef void *fr_stream;

#define FR_OK 0
#define FR_ERR_INVALID_ARG (-1) /* null pointer, size < 1, k > rows, k > FR_K_MAX, V_sub > V, d % 8 != 0 */
#define FR_ERR_ALIGNMENT (-2)   /* a bf16 tensor or the workspace is not 16-byte aligned */
#define FR_ERR_WORKSPACE (-3)   /* workspace smaller than fr_workspace_bytes() */
#define FR_ERR_HIP (-4)         /* the HIP runtime refused a launch or a query */
#define FR_ERR_UNSUPPORTED (-5) /* a shape outside what the kernels cover (see fr_draft_topk) */
#define FR_ERR_SCRATCH (-6)     /* fr_draft_topk_static: more rows of H or a larger k than its scratch holds */

#define FR_K_MAX 64 /* largest k accepted by the top-k calls */

/* Human-readable text for a status code; never NULL; static storage. */
const char *fr_strerror(fr_status status);

/*
 * One-time set-up of the CURRENT device: queries it and raises the LDS limit of every kernel
 * build, so that afterwards a call only ever launches kernels.  Thread-safe and idempotent.
 * Every entry point that launches performs the same set-up by itself the first time it runs
 * on a device; that first call must not happen while the stream is being captured into a
 * graph.  The set-up also prepares the device's static scratch (see fr_draft_topk_static),
 * synchronously on the null stream; a repeated fr_init() prepares that scratch again and
 * must not run while a fr_draft_topk_static call is in flight on the device.  A program that captures calls fr_init() once per device beforehand (Section 3.1 of
 * the paper: everything the drafting loop needs is prepared in advance).
 * Returns FR_ERR_HIP if the runtime refuses a query.
 */
fr_status fr_init(void);

/*
 * Eq. 3:  W_sub[i, :] = W_full[freq_ranked_ids[i], :]  and  idx_map[i] = freq_ranked_ids[i]
 * for i in [0, V_sub).  A bit copy: W_sub holds exactly the bytes of the chosen rows.
 *
 *   W_full           in   bf16 [V, d] row-major
 *   freq_ranked_ids  in   int32 [>= V_sub], ids ordered by corpus frequency, most frequent
 *                         first (Section 3.2, "Corpus-Level Token Statistics").  The list
 *                         is a set: duplicates are the caller's responsibility.
 *   W_sub            out  bf16 [V_sub, d] row-major (this layout is part of the contract)
 *   idx_map          out  int32 [V_sub]
 *   dev_error_flag   out  optional int32 on the device.  The host cannot see the ids
 *                         without a synchronisation, so range checking is done by the
 *                         kernel: an id outside [0, V) leaves that row of W_sub
 *                         untouched, stores -1 in idx_map[i] and sets *dev_error_flag
 *                         to 1.  The flag is never cleared by the library.
 * Requires d % 8 == 0 (rows are whole 16-byte chunks), 1 <= V_sub <= V.
 * W_sub must not overlap W_full.
 */
fr_status fr_build_subset(const void *W_full, int64_t V, int64_t d,
                          const int32_t *freq_ranked_ids, int64_t V_sub,
                          void *W_sub, int32_t *idx_map, int32_t *dev_error_flag,
                          fr_stream stream);

/*
 * Scratch needed by fr_draft_topk / fr_full_topk for a problem of this size (bytes; 0 if
 * the arguments are invalid).  Pure host arithmetic: usable without a GPU.
 * The same workspace may serve any call whose requirement is not larger.
 */
size_t fr_workspace_bytes(int64_t M, int64_t d, int64_t V_rows, int32_t k);

/*
 * Prepares a freshly allocated workspace: clears the arrival counters of the single-launch
 * kernels and marks every record of the result mailboxes empty (about 17 MiB is written).
 * Call once per workspace before its first use,
 * and again if a call using it was ever abandoned mid-flight.  Every completed call
 * leaves the workspace ready for the next one.  Calls that share a workspace must be
 * ordered on one stream.
 */
fr_status fr_workspace_init(void *workspace, size_t workspace_bytes, fr_stream stream);

/*
 * Reads the workspace's sticky time-out word.  The single-launch kernels wait, inside the
 * launch, for partial results of other workgroups; every such wait is bounded, and a wait that
 * ever ran out (only possible if workgroups of one launch could not make progress for about a
 * second, or if the workspace was not prepared) sets the word; the rows of the outputs whose
 * merge gave up hold "no result" (token id INT32_MAX, logp -inf; for fr_draft_step also no
 * next nodes: score -inf, token INT32_MAX, history index -1).  *timed_out receives 0 or 1.
 * Synchronous: copies 4 bytes to the host and waits for everything queued on `stream` before
 * it.  Once the word is set the workspace may still hold partial results of the abandoned
 * call: prepare it again with fr_workspace_init (which also clears the word) before its next
 * use.
 */
fr_status fr_workspace_check(const void *workspace, size_t workspace_bytes, int32_t *timed_out,
                             fr_stream stream);

/*
 * Eq. 4, candidate selection and id translation in one pass over W_sub:
 *   z[m, i]    = sum_j H[m, j] * W_sub[i, j]          bf16 products, fp32 accumulation
 *   logp[m, i] = z[m, i] - log sum_{i' < V_sub} exp(z[m, i'])   (the subset only)
 *   for each row m: the k entries with the largest z, most probable first, equal z
 *   ordered by lower full-vocabulary id; reported as idx_map[i] (i itself if idx_map is
 *   NULL) together with their logp.
 * The logits are never written to memory; W_sub is read exactly once.
 *
 *   H          in   bf16 [M, d] row-major, one row per draft-tree node
 *   W_sub      in   bf16 [V_sub, d] row-major (from fr_build_subset)
 *   idx_map    in   int32 [V_sub] or NULL for the identity
 *   token_ids  out  int32 [M, k] full-vocabulary ids
 *   logp       out  fp32  [M, k]
 *   workspace       >= fr_workspace_bytes(M, d, V_sub, k) bytes, 16-byte aligned,
 *                   prepared by fr_workspace_init
 * Requires M >= 1, d % 8 == 0, 1 <= k <= min(V_sub, FR_K_MAX), V_sub < 2^31.  W_sub (rows
 * rounded up to a multiple of 16) must not exceed 4 GiB, else FR_ERR_UNSUPPORTED.
 * M <= 16 runs in the skinny kernel (all of H resident in LDS, W streamed once through
 * registers) while H fits beside the kernel's other LDS buffers (12 rows at d = 4096);
 * larger M, or a larger H, runs in the matrix-core kernels: up to 64 rows of H in the chunked
 * kernel, 65 to 256 rows per launch in the block kernel (one pass over W_sub for all of them;
 * d a multiple of 128, k <= 16), otherwise in slabs of up to 128 rows of H, one pass per slab.
 * k <= 16 takes the fast selection and the single-launch merge at every M (k = 11 .. 16 within
 * about 1.5 us of k = 10); larger k takes a general path that costs two to five times as much.
 * NaN or infinite inputs give unspecified outputs but never a fault or a hang.
 */
fr_status fr_draft_topk(const void *H, int64_t M, int64_t d,
                        const void *W_sub, const int32_t *idx_map, int64_t V_sub,
                        int32_t k, int32_t *token_ids, float *logp,
                        void *workspace, size_t workspace_bytes, fr_stream stream);

/*
 * fr_draft_topk for callers that cannot allocate device memory or carry a workspace around:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * same kernels, the same results bit for bit; the workspace is a static array in device
 * memory (about 2.2 MiB per device, held until the process ends) instead of an argument.
 * The call allocates nothing and frees nothing.
 *   Limits: M <= 16 and k <= 16, else FR_ERR_SCRATCH (nothing is launched).
 *   The scratch belongs to the DEVICE, not to the call: every call on one device uses the same
 *   array, so calls that overlap on one device (two streams, two threads) race; order them.
 *   A completed call leaves the scratch ready for the next one (mailbox records emptied, the
 *   arrival counters taking turns), whatever the sizes of the two calls.
 *   The scratch is prepared by the per-device set-up (fr_init, or the first call of any entry
 *   point on the device: synchronous, not under capture).  Should a call ever be abandoned or
 *   report "no result" rows (see fr_workspace_check), fr_init() prepares the scratch again.
 * Arguments and everything else as in fr_draft_topk.
 */
fr_status fr_draft_topk_static(const void *H, int64_t M, int64_t d,
                               const void *W_sub, const int32_t *idx_map, int64_t V_sub,
                               int32_t k, int32_t *token_ids, float *logp, fr_stream stream);

/*
 * Eq. 2: the same operation over every row of W_full (position == token id).  This is the
 * uncompressed EAGLE-2 draft head, kept as the baseline the subset is measured against.
 */
fr_status fr_full_topk(const void *H, int64_t M, int64_t d,
                       const void *W_full, int64_t V, int32_t k,
                       int32_t *token_ids, float *logp,
                       void *workspace, size_t workspace_bytes, fr_stream stream);

/*
 * Verification aid (not on the drafting path): runs the same contraction kernels as
 * fr_draft_topk but stores the logits of Eq. 4 instead of consuming them.
 *   z_out  out  fp32 [M, V_rows] row-major
 */
fr_status fr_draft_logits(const void *H, int64_t M, int64_t d,
                          const void *W, int64_t V_rows, float *z_out, fr_stream stream);

/*
 * One draft step of the beam search that drives the draft LM head (Section 2 of the paper:
 * EAGLE-2 drafts by beam search on the draft model's softmax output).  The M nodes of the
 * step (cumulative log-probability node_score[m]; node_hist[m] = index of the node in the
 * search history, -1 for the prompt at the first step) have just received k candidates each
 * from fr_draft_topk.  All M*k candidates are appended to the search history at
 * hist_offset + c, c = m*k + j, with
 *   hist_score  = node_score[m] + logp[m, j]      (one fp32 addition)
 *   hist_token  = token_ids[m, j]
 *   hist_parent = node_hist[m]
 * and the `width` best of them (score descending, equal scores by lower c) are returned as
 * the nodes of the next step: next_score, next_token, next_hist (= hist_offset + c).
 *
 *   logp, token_ids    in   fp32 / int32 [M, k] (the outputs of fr_draft_topk)
 *   node_score         in   fp32 [M];  node_hist  in  int32 [M]
 *   hist_*             io   fp32 / int32 / int32, at least hist_offset + M*k entries (caller's
 *                           capacity; not checked)
 *   next_*             out  [width], 1 <= width <= M*k
 * All device pointers.  M*k <= 4096, else FR_ERR_UNSUPPORTED.  NaN scores are not ordered.
 * Asynchronous on `stream`.
 */
fr_status fr_beam_expand(const float *logp, const int32_t *token_ids, int64_t M, int32_t k,
                         const float *node_score, const int32_t *node_hist, int32_t width,
                         float *hist_score, int32_t *hist_token, int32_t *hist_parent,
                         int64_t hist_offset, float *next_score, int32_t *next_token,
                         int32_t *next_hist, fr_stream stream);

/*
 * fr_draft_topk and fr_beam_expand as one call: the draft LM head on the M nodes of a draft
 * step, then the expansion of the beam search with the head's own outputs.  Arguments as in
 * those two calls; token_ids / logp [M, k] are still written.  For M <= 16, k <= 16 (and a
 * device of at most 256 compute units) the expansion runs inside the LM head's launch: the
 * workgroup that merges the first row collects every row's result and appends, ranks and
 * returns the next nodes, which saves a launch per draft step (the "short-duration tasks" of
 * Section 3.1).  Otherwise the two launches follow each other on `stream`.
 */
fr_status fr_draft_step(const void *H, int64_t M, int64_t d, const void *W_sub,
                        const int32_t *idx_map, int64_t V_sub, int32_t k, const float *node_score,
                        const int32_t *node_hist, int32_t width, float *hist_score,
                        int32_t *hist_token, int32_t *hist_parent, int64_t hist_offset,
                        int32_t *token_ids, float *logp, float *next_score, int32_t *next_token,
                        int32_t *next_hist, void *workspace, size_t workspace_bytes,
                        fr_stream stream);

/*
 * The draft tree (Section 2: "select the top K probability tokens from the beam search
 * history"; "each token can only see tokens in its ancestral path").  Of the N history
 * entries the K best (score descending, equal scores by lower index) are listed in ascending
 * history index:
 *   sel_index [K]     history index
 *   sel_token [K]     token
 *   sel_parent[K]     position (0..K-1) of the parent inside this list, -1 if the entry
 *                     extends the prompt, -2 if its parent was not selected (cannot happen
 *                     when a child never scores above its parent: log-probabilities <= 0)
 *   sel_depth [K]     number of ancestors inside the list
 *   tree_mask [K, K]  uint8, row p: 1 at p and at the positions of p's ancestors, else 0
 * hist_parent[i] must be -1 or an index below i (entries are appended after their parents);
 * a walk up the path stops at anything else.  All device pointers.  N <= 4096, K <= 1024,
 * else FR_ERR_UNSUPPORTED.  Asynchronous on `stream`.
 */
fr_status fr_tree_select(const float *hist_score, const int32_t *hist_token,
                         const int32_t *hist_parent, int64_t N, int32_t K, int32_t *sel_index,
                         int32_t *sel_token, int32_t *sel_parent, int32_t *sel_depth,
                         uint8_t *tree_mask, fr_stream stream);

/*
 * fr_draft_topk for hidden states that sit in several blocks of memory (several draft heads
 * evaluated against one W_sub, as when the method is applied to Medusa-style heads, Section
 * 4.5): block b holds rows_per_block rows, bf16 [rows_per_block, d] row-major; row
 * m of the combined problem is row m % rows_per_block of block m / rows_per_block; outputs
 * are [n_blocks * rows_per_block, k].  H_blocks is a HOST array of n_blocks (<= 16) device
 * pointers, read during the call only.  Up to 16 rows in total run as one launch; beyond,
 * one launch per block.  Everything else as fr_draft_topk.
 */
fr_status fr_draft_topk_multi(const void *const *H_blocks, int32_t n_blocks, int64_t rows_per_block,
                              int64_t d, const void *W_sub, const int32_t *idx_map, int64_t V_sub,
                              int32_t k, int32_t *token_ids, float *logp, void *workspace,
                              size_t workspace_bytes, fr_stream stream);

/*
 * The same subset and the same head with W_sub in a private tiled layout (Eq. 3 fixes the
 * matrix, not how it is stored; the gather rewrites W once anyway).  A tile is 16
 * consecutive rows of W_sub; inside a tile, the 16-byte chunk holding row i (0..15),
 * elements 32*kb + 8*g .. + 7 (g = 0..3) is chunk number kb*64 + g*16 + i, i.e. element
 * (row r, column c) of W_sub is the bf16 at
 *   (r / 16) * 16 * d  +  (c / 32) * 512  +  ((c % 32) / 8) * 128  +  (r % 16) * 8  +  c % 8.
 * Every 1 KiB block is then one matrix-core operand in lane order: the kernel reads W in
 * contiguous 4 KiB pieces and needs no reordering on chip.  Rows that pad the last tile are
 * zero.  d must be a multiple of 128.
 *   fr_tiled_bytes         size of W_tiled in bytes (0 if the arguments are invalid)
 *   fr_build_subset_tiled  as fr_build_subset, writing W_tiled; a row whose id is outside
 *                          [0, V) is zero, idx_map = -1, *dev_error_flag set
 *   fr_draft_topk_tiled    as fr_draft_topk, reading W_tiled; M <= 16 (FR_ERR_UNSUPPORTED
 *                          beyond)
 */
size_t fr_tiled_bytes(int64_t V_sub, int64_t d);
fr_status fr_build_subset_tiled(const void *W_full, int64_t V, int64_t d,
                                const int32_t *freq_ranked_ids, int64_t V_sub, void *W_tiled,
                                int32_t *idx_map, int32_t *dev_error_flag, fr_stream stream);
fr_status fr_draft_topk_tiled(const void *H, int64_t M, int64_t d, const void *W_tiled,
                              const int32_t *idx_map, int64_t V_sub, int32_t k,
                              int32_t *token_ids, float *logp, void *workspace,
                              size_t workspace_bytes, fr_stream stream);


/*
 * Corpus-level token statistics (Section 3.2): the step that produces the ranking which
 * fr_build_subset consumes.
 *   fr_count_tokens  counts[t] += occurrences of t in tokens[0..n_tokens); ids outside [0, V)
 *                    are skipped and *dev_error_flag (optional) is set.  `counts` (int64 [V])
 *                    accumulates over calls: zero it before the first one.  `tokens` must be
 *                    16-byte aligned.  V <= 2^22 and n_tokens below 2^32 per share of the stream
 *                    (one share per two compute units at V = 128256), else FR_ERR_UNSUPPORTED.
 *   fr_rank_tokens   freq_ranked_ids[0..V) = all ids by count descending, equal counts by
 *                    lower id (counts must be >= 0).  V <= 2^22, else FR_ERR_UNSUPPORTED.
 *                    Takes 20 V bytes + 25 KiB of temporary device memory from the stream-ordered
 *                    allocator and returns it in stream order (a model-load step: the one call
 *                    of this library that allocates; FR_ERR_HIP if the allocation fails).
 * All device pointers; asynchronous on `stream`.
 */
fr_status fr_count_tokens(const int32_t *tokens, int64_t n_tokens, int64_t V, int64_t *counts,
                          int32_t *dev_error_flag, fr_stream stream);
fr_status fr_rank_tokens(const int64_t *counts, int64_t V, int32_t *freq_ranked_ids,
                         fr_stream stream);

/* Library version, major*100 + minor. */
int fr_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FRSPEC_H */
