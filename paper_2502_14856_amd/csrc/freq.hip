// The step before the draft LM head: corpus-level token statistics (Section 3.2 of the
// paper).  Token frequencies are counted over a stream of token ids, and the ids are ranked
// by frequency; the first V_sub ids of the ranking are the subset that fr_build_subset
// gathers.
//   count_kernel  bound: HBM (the stream is read once per 32768-id slice of the vocabulary).
//                 A workgroup counts its share of the stream into 32-bit LDS counters, one
//                 slice of the vocabulary at a time, and adds the non-zero counters to the
//                 64-bit totals in memory.  Counting straight into memory would serialise
//                 on the few most frequent ids (the top id of a Zipf stream is ~7% of it).
//   rank_kernel   bound: vector ALU, O(V^2): the position of id t in the ranking is the
//                 number of ids that come before it (higher count, or equal count and lower
//                 id).  Counts are staged through LDS in tiles; exact, no sorting passes.
#include "internal.hpp"
#include "wave_ops.hpp"

namespace frspec {
namespace {

constexpr int kCountThreads = 1024;
constexpr int kSlice = 32768;            // ids per pass: 128 KiB of LDS counters
typedef int i32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kCountThreads) void count_kernel(const int *__restrict__ tokens, long long n, int V,
                                                              unsigned long long *__restrict__ counts,
                                                              int *__restrict__ flag) {
    extern __shared__ u32x4 smem[];
    unsigned *cnt = reinterpret_cast<unsigned *>(smem);   // [kSlice]
    const int tid = threadIdx.x;
    // this workgroup's share of the stream: whole groups of 4 tokens (16-byte loads); the
    // last workgroup also takes the odd tokens at the end
    const long long groups = n / 4;
    const long long per = (groups + gridDim.x - 1) / gridDim.x;
    const long long g0 = (long long)blockIdx.x * per;
    const long long g1 = g0 + per < groups ? g0 + per : groups;
    const bool takes_tail = blockIdx.x == gridDim.x - 1;
    bool bad = false;
    for (int base = 0; base < V; base += kSlice) {
        for (int c = tid; c < kSlice; c += kCountThreads) cnt[c] = 0u;
        __syncthreads();
        auto take = [&](int t) {
            const unsigned rel = (unsigned)(t - base);
            if (rel < (unsigned)kSlice && t < V) atomicAdd(&cnt[rel], 1u);
            if (base == 0 && (t < 0 || t >= V)) bad = true;
        };
        const i32x4 *t4 = reinterpret_cast<const i32x4 *>(tokens);
        for (long long g = g0 + tid; g < g1; g += kCountThreads) {
            const i32x4 v = __builtin_nontemporal_load(t4 + g);
            take(v.x);
            take(v.y);
            take(v.z);
            take(v.w);
        }
        if (takes_tail)
            for (long long i = groups * 4 + tid; i < n; i += kCountThreads) take(tokens[i]);
        __syncthreads();
        for (int c = tid; c < kSlice; c += kCountThreads) {
            const unsigned v = cnt[c];
            if (v != 0u) atomicAdd(&counts[base + c], (unsigned long long)v);
        }
        __syncthreads();
    }
    if (bad && flag) *flag = 1;
}

constexpr int kRankThreads = 256;
constexpr int kRankTile = 2048;

__global__ __launch_bounds__(kRankThreads) void rank_kernel(const long long *__restrict__ counts, int V,
                                                            int *__restrict__ ranked) {
    __shared__ long long tile[kRankTile];
    const int t = blockIdx.x * kRankThreads + threadIdx.x;
    const long long mine = t < V ? counts[t] : 0;
    int before = 0;   // ids that precede t in the ranking
    for (int base = 0; base < V; base += kRankTile) {
        __syncthreads();
        for (int j = threadIdx.x; j < kRankTile; j += kRankThreads)
            tile[j] = base + j < V ? counts[base + j] : -1;   // a count is never negative
        __syncthreads();
        const int n = min(kRankTile, V - base);
        if (base + n <= t) {            // the whole tile has lower ids: equal counts precede too
            for (int j = 0; j < n; ++j) before += tile[j] >= mine;
        } else if (base > t) {          // the whole tile has higher ids
            for (int j = 0; j < n; ++j) before += tile[j] > mine;
        } else {
            for (int j = 0; j < n; ++j) before += tile[j] > mine || (tile[j] == mine && base + j < t);
        }
    }
    if (t < V) ranked[before] = t;
}

}  // namespace

fr_status prepare_freq_kernels() {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(count_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            kSlice * 4) != hipSuccess) {
        (void)hipGetLastError();
        return FR_ERR_HIP;
    }
    return FR_OK;
}

fr_status launch_count_tokens(const int *tokens, long long n, int V, unsigned long long *counts, int *flag,
                              hipStream_t s) {
    const int cus = device_cu_count();
    if (cus <= 0) return FR_ERR_HIP;
    long long blocks = (n / 4 + kCountThreads - 1) / kCountThreads;
    if (blocks > cus) blocks = cus;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(count_kernel, dim3((unsigned)blocks), dim3(kCountThreads), kSlice * 4, s, tokens, n, V, counts,
                       flag);
    return hip_status(hipGetLastError());
}

fr_status launch_rank_tokens(const long long *counts, int V, int *ranked, hipStream_t s) {
    hipLaunchKernelGGL(rank_kernel, dim3((V + kRankThreads - 1) / kRankThreads), dim3(kRankThreads), 0, s, counts, V,
                       ranked);
    return hip_status(hipGetLastError());
}

}  // namespace frspec
