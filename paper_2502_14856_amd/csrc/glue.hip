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

constexpr int kGlueMaxN = kGlueMaxCandidates;
static_assert(kGlueMaxN % kGlueThreads == 0 && kGlueMaxN / kWave == kWave, "one wavefront scans the chunk counts");
constexpr int kGlueChunks = kGlueMaxN / kWave;                       // 64-entry chunks of a history
constexpr int kGluePerThread = kGlueMaxN / kGlueThreads;

__global__ __launch_bounds__(kGlueThreads) void tree_select_kernel(
    const float *__restrict__ hist_score, const int *__restrict__ hist_token,
    const int *__restrict__ hist_parent, int N, int K, int *__restrict__ sel_index,
    int *__restrict__ sel_token, int *__restrict__ sel_parent, int *__restrict__ sel_depth,
    unsigned char *__restrict__ tree_mask, int groups) {
    extern __shared__ u32x4 smem[];
    unsigned long long *keys = reinterpret_cast<unsigned long long *>(smem);   // [N + 2]
    int *posmap = reinterpret_cast<int *>(keys + ((N + 2) & ~1));              // [N]: position or -1
    int *par = posmap + N;                                                     // [N]: hist_parent
    __shared__ int chunk_before[kGlueChunks];   // selected entries before each 64-entry chunk
    __shared__ unsigned long long s_bound;
    __shared__ int s_survivors;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    for (int i = tid; i < N; i += kGlueThreads) {
        keys[i] = make_key(key_hi_of(hist_score[i]), ~(unsigned)i);
        par[i] = hist_parent[i];
    }
    if (tid == 0) keys[N] = 0ull;
    if (tid < kGlueChunks) chunk_before[tid] = 0;
    for (int i = tid; i < K * K; i += kGlueThreads) tree_mask[i] = 0;
    __syncthreads();

    // rank[i] = number of better entries.  A short history is scanned by several threads per
    // entry (P of them share the keys between them), a long one by one thread per entry.
    int *rank = par + N;   // [N]
    if (groups > 0) {
        // Only "is it among the K best" is needed, not every entry's rank.  The entries fall into
        // `groups` >= 2K groups (entry i in group i % groups); the K-th largest group maximum B is a
        // lower bound of the K-th best key (K different groups hold a key that large), so only the
        // entries at or above B (K plus some) are ranked, among themselves: groups^2 + (K + some)^2
        // comparisons instead of N^2.
        // (16-byte aligned: the three int arrays padded to a multiple of four ints)
        unsigned long long *gmax = reinterpret_cast<unsigned long long *>(rank + N + ((4 - (3 * N) % 4) % 4));   // [groups + 2]
        unsigned long long *surv = gmax + groups + 2;                                               // [N + 2]
        int *grank = reinterpret_cast<int *>(surv + ((N + 2) & ~1));                                // [groups]
        for (int g = tid; g < groups; g += kGlueThreads) {
            unsigned long long best = 0ull;
            for (int i = g; i < N; i += groups) best = max(best, keys[i]);
            gmax[g] = best;
            grank[g] = 0;
        }
        if (tid == 0) {
            gmax[groups] = 0ull;
            s_survivors = 0;
        }
        __syncthreads();
        {
            const int P = kGlueThreads / groups;   // threads per group maximum (groups divides 1024)
            const int g = tid / P, part = tid - g * P;
            const int per = groups / P;            // even: groups >= 2 P whenever P > 1, both powers of two
            if (P == 1)
                grank[g] = count_greater(gmax, groups, gmax[g]);
            else
                atomicAdd(&grank[g], count_greater(gmax + part * per, per, gmax[g]));
        }
        __syncthreads();
        for (int g = tid; g < groups; g += kGlueThreads)
            if (grank[g] == K - 1) s_bound = gmax[g];   // (the keys are all different: exactly one)
        __syncthreads();
        const unsigned long long B = s_bound;
        for (int i = tid; i < N; i += kGlueThreads) {
            const bool sv = keys[i] >= B;
            rank[i] = sv ? 0 : K;
            if (sv) surv[atomicAdd(&s_survivors, 1)] = keys[i];
        }
        __syncthreads();
        const int ns = s_survivors;
        if (tid < 2) surv[ns + tid] = 0ull;
        __syncthreads();
        int P = 1;
        while (P < 16 && 2 * P * ns <= kGlueThreads) P *= 2;
        for (int e = tid / P; e < ns; e += kGlueThreads / P) {
            const int part = tid % P;
            const int per = ((ns + P - 1) / P + 1) & ~1;
            const int lo = part * per, hi = lo + per < ns ? lo + per : ns;
            const unsigned long long mine = surv[e];
            if (lo < hi) atomicAdd(&rank[(int)~(unsigned)mine], count_greater(surv + lo, hi - lo, mine));
        }
        __syncthreads();
    } else {
    for (int i = tid; i < N; i += kGlueThreads) rank[i] = 0;
    __syncthreads();
    int P = 1;
    while (P < 16 && 2 * P * N <= kGlueThreads) P *= 2;
    if (P > 1) {
        const int i = tid / P, part = tid - i * P;
        if (i < N) {
            const int per = ((N + P - 1) / P + 1) & ~1;   // even, so that reads stay 16-byte aligned
            const int lo = part * per, hi = lo + per < N ? lo + per : N;
            if (lo < hi) atomicAdd(&rank[i], count_greater(keys + lo, hi - lo, keys[i]));
        }
    } else {
        for (int i = tid; i < N; i += kGlueThreads) rank[i] = count_greater(keys, N, keys[i]);
    }
    __syncthreads();
    }
    // selected = fewer than K better entries.  Entry i = tid + u * 1024 lies in chunk i / 64,
    // which one wavefront covers with one ballot.
    int before_in_chunk[kGluePerThread];
    bool selected[kGluePerThread];
#pragma unroll
    for (int u = 0; u < kGluePerThread; ++u) {
        const int i = tid + u * kGlueThreads;
        selected[u] = i < N && rank[i < N ? i : 0] < K;
        const unsigned long long mask = __ballot(selected[u]);
        before_in_chunk[u] = (int)__builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32),
                                                             __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u));
        if (lane == 0) chunk_before[i / kWave] = (int)__popcll(mask);
    }
    __syncthreads();
    if (tid < kWave) {   // exclusive prefix sum over the 64 chunk counts, in one wavefront
        const int own = chunk_before[tid];
        int incl = own;
#pragma unroll
        for (int sh = 1; sh < kWave; sh <<= 1) {
            const int other = __shfl_up(incl, sh);
            if (lane >= sh) incl += other;
        }
        chunk_before[tid] = incl - own;
    }
    __syncthreads();
    // position in history order = number of selected entries before this one
#pragma unroll
    for (int u = 0; u < kGluePerThread; ++u) {
        const int i = tid + u * kGlueThreads;
        if (i < N) posmap[i] = selected[u] ? chunk_before[i / kWave] + before_in_chunk[u] : -1;
    }
    __syncthreads();
    for (int i = tid; i < N; i += kGlueThreads) {
        const int p = posmap[i];
        if (p < 0) continue;
        sel_index[p] = i;
        sel_token[p] = hist_token[i];
        const int h = par[i];
        // -1: extends the prompt; -2: parent not selected (impossible while no child scores
        // above its parent)
        sel_parent[p] = h < 0 ? -1 : (h < i && posmap[h] >= 0 ? posmap[h] : -2);
        tree_mask[(size_t)p * K + p] = 1;
        int depth = 0;
        // up the ancestral path; parents precede children, which also bounds the walk
        for (int q = h, below = i; q >= 0 && q < below && posmap[q] >= 0; below = q, q = par[q]) {
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

// up to ~125 KiB of dynamic LDS (4096 entries, with the bound's groups and survivor list): above the default limit
fr_status prepare_glue_kernels() {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(tree_select_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 144 * 1024) != hipSuccess) {
        (void)hipGetLastError();
        return FR_ERR_HIP;
    }
    return FR_OK;
}

fr_status launch_tree_select(const float *hist_score, const int *hist_token, const int *hist_parent, int N, int K,
                             int *sel_index, int *sel_token, int *sel_parent, int *sel_depth,
                             unsigned char *tree_mask, hipStream_t s) {
    size_t lds = ((size_t)((N + 2) & ~1)) * sizeof(unsigned long long) + ((3 * (size_t)N + 3) & ~(size_t)3) * sizeof(int);
    // groups of the bound: a power of two, at least 2K; where that leaves fewer than two entries
    // per group on average the plain all-pairs ranking is as cheap
    int groups = 64;
    while (groups < 2 * K) groups *= 2;
    if (groups > kGlueThreads || 2 * groups > N) groups = 0;
    if (groups > 0)
        lds += ((size_t)groups + 2 + (size_t)((N + 2) & ~1)) * sizeof(unsigned long long) + (size_t)groups * sizeof(int);
    if (!device_state()) return FR_ERR_HIP;   // (the per-device set-up raised this kernel's LDS limit)
    hipLaunchKernelGGL(tree_select_kernel, dim3(1), dim3(kGlueThreads), lds, s, hist_score, hist_token,
                       hist_parent, N, K, sel_index, sel_token, sel_parent, sel_depth, tree_mask, groups);
    return hip_status(hipGetLastError());
}

}  // namespace frspec
