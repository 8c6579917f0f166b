// Draft-step glue around the draft LM head (Section 2 of the paper: drafting by beam search,
// "select the top K probability tokens from the beam search history", ancestral-path mask):
//   expand_kernel       one draft step: the M*k candidates of the step join the history with
//                       their cumulative scores; the `width` best become the next nodes
//   tree_select_kernel  the draft: the K best history entries in history order, the position
//                       of each one's parent, its depth and the ancestor mask
// Both are tiny, single-workgroup, latency-bound kernels: a few hundred to a few thousand
// candidates, ordered with the same 64-bit keys as the LM head's candidates (score descending,
// equal scores by lower index) and ranked by counting.
#include "internal.hpp"
#include "wave_ops.hpp"

namespace frspec {
namespace {

constexpr int kGlueThreads = 1024;

typedef unsigned long long u64x2_t __attribute__((ext_vector_type(2)));

// Number of keys in keys[0..n) that are larger than `mine` (n even or keys[n] readable: the
// caller pads with one zero key).
__device__ __forceinline__ int count_greater(const unsigned long long *keys, int n, unsigned long long mine) {
    const u64x2_t *kp = reinterpret_cast<const u64x2_t *>(keys);
    int rank = 0;
#pragma unroll 4
    for (int j = 0; j < n; j += 2) {
        const u64x2_t two = kp[j >> 1];
        rank += two.x > mine;
        rank += two.y > mine;
    }
    return rank;
}

__global__ __launch_bounds__(kGlueThreads) void expand_kernel(
    const float *__restrict__ logp, const int *__restrict__ token_ids, int C, int k,
    const float *__restrict__ node_score, const int *__restrict__ node_hist, int width,
    float *__restrict__ hist_score, int *__restrict__ hist_token, int *__restrict__ hist_parent,
    long long hist_offset, float *__restrict__ next_score, int *__restrict__ next_token,
    int *__restrict__ next_hist) {
    extern __shared__ u32x4 smem[];
    unsigned long long *keys = reinterpret_cast<unsigned long long *>(smem);   // [C + 1]
    const int tid = threadIdx.x;
    for (int c = tid; c < C; c += kGlueThreads) {
        const int m = c / k;
        const float s = node_score[m] + logp[c];   // the one rounding of the cumulative score
        hist_score[hist_offset + c] = s;
        hist_token[hist_offset + c] = token_ids[c];
        hist_parent[hist_offset + c] = node_hist[m];
        keys[c] = make_key(key_hi_of(s), ~(unsigned)c);
    }
    if (tid == 0) keys[C] = 0ull;
    __syncthreads();
    for (int c = tid; c < C; c += kGlueThreads) {
        const unsigned long long mine = keys[c];
        const int rank = count_greater(keys, C, mine);
        if (rank < width) {
            next_score[rank] = node_score[c / k] + logp[c];
            next_token[rank] = token_ids[c];
            next_hist[rank] = (int)(hist_offset + c);
        }
    }
}

__global__ __launch_bounds__(kGlueThreads) void tree_select_kernel(
    const float *__restrict__ hist_score, const int *__restrict__ hist_token,
    const int *__restrict__ hist_parent, int N, int K, int *__restrict__ sel_index,
    int *__restrict__ sel_token, int *__restrict__ sel_parent, int *__restrict__ sel_depth,
    unsigned char *__restrict__ tree_mask) {
    extern __shared__ u32x4 smem[];
    unsigned long long *keys = reinterpret_cast<unsigned long long *>(smem);   // [N + 2]
    int *posmap = reinterpret_cast<int *>(keys + ((N + 2) & ~1));              // [N]: position or -1
    const int tid = threadIdx.x;
    for (int i = tid; i < N; i += kGlueThreads) keys[i] = make_key(key_hi_of(hist_score[i]), ~(unsigned)i);
    if (tid == 0) keys[N] = 0ull;
    for (int i = tid; i < K * K; i += kGlueThreads) tree_mask[i] = 0;
    __syncthreads();
    // selected = fewer than K better entries
    for (int i = tid; i < N; i += kGlueThreads) posmap[i] = count_greater(keys, N, keys[i]) < K ? 0 : -1;
    __syncthreads();
    // position in history order = number of selected entries before this one
    int my_pos[(4096 + kGlueThreads - 1) / kGlueThreads];
    for (int i = tid, u = 0; i < N; i += kGlueThreads, ++u) {
        int pos = -1;
        if (posmap[i] == 0) {
            pos = 0;
            for (int j = 0; j < i; ++j) pos += posmap[j] == 0;
        }
        my_pos[u] = pos;
    }
    __syncthreads();
    for (int i = tid, u = 0; i < N; i += kGlueThreads, ++u) posmap[i] = my_pos[u];
    __syncthreads();
    for (int i = tid; i < N; i += kGlueThreads) {
        const int p = posmap[i];
        if (p < 0) continue;
        sel_index[p] = i;
        sel_token[p] = hist_token[i];
        const int h = hist_parent[i];
        // -1: extends the prompt; -2: parent not selected (impossible while no child scores
        // above its parent)
        sel_parent[p] = h < 0 ? -1 : (h < i && posmap[h] >= 0 ? posmap[h] : -2);
        tree_mask[(size_t)p * K + p] = 1;
        int depth = 0;
        // up the ancestral path; parents precede children, which also bounds the walk
        for (int q = h, below = i; q >= 0 && q < below && posmap[q] >= 0; below = q, q = hist_parent[q]) {
            tree_mask[(size_t)p * K + posmap[q]] = 1;
            ++depth;
        }
        sel_depth[p] = depth;
    }
}

}  // namespace

fr_status launch_beam_expand(const float *logp, const int *token_ids, int C, int k, const float *node_score,
                             const int *node_hist, int width, float *hist_score, int *hist_token,
                             int *hist_parent, long long hist_offset, float *next_score, int *next_token,
                             int *next_hist, hipStream_t s) {
    const size_t lds = ((size_t)C + 2) * sizeof(unsigned long long);
    hipLaunchKernelGGL(expand_kernel, dim3(1), dim3(kGlueThreads), lds, s, logp, token_ids, C, k, node_score,
                       node_hist, width, hist_score, hist_token, hist_parent, hist_offset, next_score, next_token,
                       next_hist);
    return hip_status(hipGetLastError());
}

fr_status launch_tree_select(const float *hist_score, const int *hist_token, const int *hist_parent, int N, int K,
                             int *sel_index, int *sel_token, int *sel_parent, int *sel_depth,
                             unsigned char *tree_mask, hipStream_t s) {
    const size_t lds = ((size_t)((N + 2) & ~1)) * sizeof(unsigned long long) + (size_t)N * sizeof(int);
    hipLaunchKernelGGL(tree_select_kernel, dim3(1), dim3(kGlueThreads), lds, s, hist_score, hist_token,
                       hist_parent, N, K, sel_index, sel_token, sel_parent, sel_depth, tree_mask);
    return hip_status(hipGetLastError());
}

}  // namespace frspec
