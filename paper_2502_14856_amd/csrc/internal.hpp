// Host-side declarations shared by the translation units of libfrspec.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/frspec_dev.h"

namespace frspec {

// What a contraction kernel does with the logits of a tile.
enum class Sink : int {
    kFusedTopk = 0,    // fold into partials; some of the workgroups merge them (single launch)
    kPartialsOnly = 1, // fold into partials; a merge kernel follows
    kLogits = 2,       // store the logits (verification aid)
    kStreamOnly = 3,   // drop the logits (measures the contraction alone)
};

// Device-side view of the workspace.
struct WorkspaceView {
    unsigned *ticket;
    unsigned long long *mail_rec;   // self-validating result records (single-launch merge)
    unsigned long long *mail_st;
    unsigned long long *step_rec;   // hand-over records of the fused beam-search expansion
    float *part_ms;
    float *part_val;
    int *part_id;
};

// Arguments of the beam-search expansion that can ride on the skinny kernel's launch (see
// expand_step_fused): the nodes of the step, the search history, the next nodes.
struct StepArgs {
    unsigned long long *rec;   // [16][16]; nullptr: no expansion in this launch
    const float *node_score;
    const int *node_hist;
    int width;
    long long hist_offset;
    float *hist_score;
    int *hist_token;
    int *hist_parent;
    float *next_score;
    int *next_token;
    int *next_hist;
};

struct HeadProblem {
    const StepArgs *step;   // optional: beam-search expansion fused into the launch (skinny kernel)
    const void *H;        // bf16 [M, d]; or, with scattered_rows, row m starts row_delta[m] bytes from H
    bool scattered_rows;  // (skinny kernel only, M <= 16)
    long long row_delta[16];
    const void *W;        // bf16 [V_rows, d] row-major, or the tiled layout of fr_build_subset_tiled
    bool tiled;
    const int *idx_map;   // nullable
    int M, d, V_rows, k;
    int *token_ids;       // [M, k]
    float *logp;          // [M, k]
    float *z_out;         // [M, V_rows] (Sink::kLogits only)
    int z_ld;             // leading dimension of z_out
    WorkspaceView ws;
};

constexpr size_t kWorkspaceHeaderBytes = 512;
// Result mailbox of the single-launch merge: 256 rows of H x (16 list positions + 1
// statistics record) x 512 workgroups, 8 bytes each, all ones while empty.
constexpr int kMailRows = 256, kMailK = 16;   // rows of H and list positions with records
constexpr size_t kMailRecBytes = (size_t)kMailRows * kMailK * 512u * 8u;
constexpr size_t kMailStBytes = (size_t)kMailRows * 512u * 8u;
constexpr size_t kStepRecBytes = 16u * 16u * 8u;   // one record per (row of H, list position)
constexpr int kWorkspaceGridMax = 512;   // partial slots reserved per row of H
constexpr int kMatrixPathMaxM = 256;     // rows of H per matrix-core launch
constexpr int kSkinnyMaxM = 16;          // rows of H the vector-ALU kernel covers

// What the library keeps per device, filled by the per-device set-up: fr_init(), or the first
// call of any entry point that launches on that device.  The set-up queries the device, raises
// the dynamic LDS limit of every kernel build (so that no launch ever changes a function
// attribute) and is thread-safe.
struct DeviceState {
    int cus;         // compute units
    void *scratch;   // device address of this device's copy of the static scratch (fr_draft_topk_static)
};
// State of the current device, after its set-up; nullptr if the set-up failed.
const DeviceState *device_state();
// Number of compute units of the current device; <= 0 on error.
int device_cu_count();
// The parts of the set-up that live with their kernels.
fr_status prepare_skinny_kernels();
fr_status prepare_wide_kernels();
fr_status prepare_block_kernels();
fr_status prepare_glue_kernels();
fr_status prepare_freq_kernels();

// skinny.hip: kernel for M <= 16 with all of H in LDS.  Returns FR_ERR_UNSUPPORTED if H does not fit.
fr_status launch_skinny(const HeadProblem &p, Sink sink, const fr_tuning *t, hipStream_t s);
// Whether some build of the skinny kernel can hold this problem's H in LDS ...
bool skinny_fits(int M, int d, int k);
// ... and whether its default build (eight wavefronts) can: the four-wavefront build that
// takes over otherwise streams more slowly than the chunked kernel.
bool skinny_fits_eight_waves(int M, int d, int k);

// mfma.hip: matrix-core kernel for 1 <= M <= 128 (more rows run in slabs).
fr_status launch_mfma(const HeadProblem &p, Sink sink, const fr_tuning *t, hipStream_t s,
                      int *grid_used);
// Largest slab of H rows (multiple of 16, <= 128) whose per-row state fits LDS for this k.
int mfma_max_rows(int k);

// gemm.hip: register-blocked matrix-core kernel for kBlockMinM <= M <= kBlockMaxM rows of H per
// launch (d a multiple of 128, k <= 16); W is read once for all of them.
constexpr int kBlockMinM = 65, kBlockMaxM = 256;
bool block_kernel_serves(int M, int d, int k);
fr_status launch_block(const HeadProblem &p, Sink sink, const fr_tuning *t, hipStream_t s);

// merge.hip: merges G partial slots per row of H into the outputs.
fr_status launch_merge(const HeadProblem &p, int G, hipStream_t s);

// gather.hip
fr_status launch_gather_tiled(const void *W_full, int64_t V, int64_t d, const int32_t *ids,
                              int64_t V_sub, void *W_tiled, int32_t *idx_map, int32_t *flag,
                              hipStream_t s);
fr_status launch_gather(const void *W_full, int64_t V, int64_t d, const int32_t *ids,
                        int64_t V_sub, void *W_sub, int32_t *idx_map, int32_t *flag,
                        hipStream_t s);

// glue.hip: beam-search expansion of one draft step and selection of the draft tree.
constexpr int kGlueMaxCandidates = 4096;   // M * k of one step, and entries of a history
constexpr int kGlueMaxTree = 1024;         // K
fr_status launch_beam_expand(const float *logp, const int *token_ids, int C, int k, const float *node_score,
                             const int *node_hist, int width, float *hist_score, int *hist_token,
                             int *hist_parent, long long hist_offset, float *next_score, int *next_token,
                             int *next_hist, hipStream_t s);
fr_status launch_tree_select(const float *hist_score, const int *hist_token, const int *hist_parent, int N, int K,
                             int *sel_index, int *sel_token, int *sel_parent, int *sel_depth,
                             unsigned char *tree_mask, hipStream_t s);

// freq.hip: token counting and frequency ranking.
fr_status launch_count_tokens(const int *tokens, long long n, int V, unsigned long long *counts, int *flag,
                              hipStream_t s);
fr_status launch_rank_tokens(const long long *counts, int V, int *ranked, hipStream_t s);

// calib.hip
fr_status launch_copy(void *dst, const void *src, size_t bytes, hipStream_t s);
fr_status launch_read(const void *src, size_t bytes, void *sink, hipStream_t s);
fr_status launch_fill_u32(unsigned *dst, size_t n, unsigned value, hipStream_t s);

inline fr_status hip_status(hipError_t e) { return e == hipSuccess ? FR_OK : FR_ERR_HIP; }

}  // namespace frspec
