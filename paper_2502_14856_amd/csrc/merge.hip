// Stand-alone merge of the per-workgroup partials: one wavefront per row of H.
// Used when the contraction kernel is launched with Sink::kPartialsOnly (matrix-core
// path, where M is large enough that one workgroup should not merge every row).
#include "epilogue.hpp"
#include "internal.hpp"

namespace frspec {
namespace {

constexpr int kMergeWaves = 4;

__global__ __launch_bounds__(kMergeWaves * kWave) void merge_kernel(Partials P, int G, int M, int k,
                                                                   int *token_ids, float *logp) {
    __shared__ SelectScratch s_select[kMergeWaves];
    const int wave = (int)(threadIdx.x / kWave);
    const int m = blockIdx.x * kMergeWaves + wave;
    final_merge_all(P, G, m, M, M, k, token_ids, logp, &s_select[wave]);   // one row per wavefront
}

}  // namespace

fr_status launch_merge(const HeadProblem &p, int G, hipStream_t s) {
    if (G < 1 || G > kGridMax) return FR_ERR_INVALID_ARG;
    Partials P{p.ws.part_ms, p.ws.part_val, p.ws.part_id};
    const int blocks = (p.M + kMergeWaves - 1) / kMergeWaves;
    hipLaunchKernelGGL(merge_kernel, dim3(blocks), dim3(kMergeWaves * kWave), 0, s, P, G, p.M, p.k,
                       p.token_ids, p.logp);
    return hip_status(hipGetLastError());
}

}  // namespace frspec
