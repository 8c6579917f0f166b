// The step before the draft LM head: corpus-level token statistics (Section 3.2 of the
// paper).  Token frequencies are counted over a stream of token ids, and the ids are ranked
// by frequency; the first V_sub ids of the ranking are the subset that fr_build_subset
// gathers.
//   count_kernel  bound: HBM (the stream is read from memory once).  A workgroup owns one
//                 32768-id slice of the vocabulary (128 KiB of 32-bit LDS counters) and one
//                 share of the stream, counts the tokens of its slice and adds the non-zero
//                 counters to the 64-bit totals in memory.  The workgroups that own the
//                 different slices of one share sit on the same compute die and read it at the
//                 same pace, so that all but the first of them find it in that die's L2.
//                 Counting straight into memory would serialise on the few most frequent ids
//                 (the top id of a Zipf stream is ~7% of it).
//   rank_kernel   bound: vector ALU, O(V^2): the position of id t in the ranking is the
//                 number of ids that come before it (higher count, or equal count and lower
//                 id).  Counts are staged through LDS in tiles; exact, no sorting passes.
#include "internal.hpp"
#include "wave_ops.hpp"

namespace frspec {
namespace {

constexpr int kCountThreads = 1024;
constexpr int kSlice = 32768;            // ids per workgroup: 128 KiB of LDS counters
constexpr int kCountMaxV = 1 << 22;      // as in the ranking (128 slices)
typedef int i32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kCountThreads) void count_kernel(const int *__restrict__ tokens, long long n, int V,
                                                              int slices, int shares, int by_die,
                                                              unsigned long long *__restrict__ counts,
                                                              int *__restrict__ flag) {
    extern __shared__ u32x4 smem[];
    unsigned *cnt = reinterpret_cast<unsigned *>(smem);   // [kSlice]
    const int tid = threadIdx.x;
    // Which slice and which share: workgroup b runs on compute die b % 8.  With by_die, b = x + 8 y
    // takes slice y % slices of share x + 8 (y / slices): the owners of one share are on one die.
    int slice, share;
    if (by_die) {
        const int x = blockIdx.x & 7, y = blockIdx.x >> 3;
        slice = y % slices;
        share = x + 8 * (y / slices);
    } else {
        slice = blockIdx.x % slices;
        share = blockIdx.x / slices;
    }
    const int base = slice * kSlice;
    // a share: whole groups of 4 tokens (16-byte loads); the last share also takes the odd
    // tokens at the end
    const long long groups = n / 4;
    const long long per = (groups + shares - 1) / shares;
    const long long g0 = (long long)share * per;
    const long long g1 = g0 + per < groups ? g0 + per : groups;
    const bool takes_tail = share == shares - 1;
    bool bad = false;
    for (int c = tid; c < kSlice; c += kCountThreads) cnt[c] = 0u;
    __syncthreads();
    auto take = [&](int t) {
        const unsigned rel = (unsigned)(t - base);
        if (rel < (unsigned)kSlice && t < V) atomicAdd(&cnt[rel], 1u);
        if (slice == 0 && (t < 0 || t >= V)) bad = true;
    };
    const i32x4 *t4 = reinterpret_cast<const i32x4 *>(tokens);
    // eight loads in flight per thread (one load at a time would make the loop a chain of L2 round
    // trips); past the end of the share the loads are clamped and their tokens dropped
    constexpr int kInFlight = 8;
    for (long long g = g0 + tid; g < g1; g += (long long)kInFlight * kCountThreads) {
        i32x4 v[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            const long long gu = g + (long long)u * kCountThreads;
            v[u] = t4[gu < g1 ? gu : g1 - 1];
        }
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            if (g + (long long)u * kCountThreads < g1) {
                take(v[u].x);
                take(v[u].y);
                take(v[u].z);
                take(v[u].w);
            }
        }
    }
    if (takes_tail)
        for (long long i = groups * 4 + tid; i < n; i += kCountThreads) take(tokens[i]);
    __syncthreads();
    for (int c = tid; c < kSlice && base + c < V; c += kCountThreads) {
        const unsigned v = cnt[c];
        if (v != 0u) atomicAdd(&counts[base + c], (unsigned long long)v);
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
    // one workgroup per (slice of the vocabulary, share of the stream); a workgroup's 32-bit LDS
    // counters hold its share (a share of 2^32 tokens or more is refused)
    if (V < 1 || V > kCountMaxV || n < 0) return FR_ERR_UNSUPPORTED;
    const int slices = (V + kSlice - 1) / kSlice;
    int shares, by_die = 0;
    if (cus % 8 == 0 && cus / 8 >= slices) {
        shares = 8 * (cus / 8 / slices);   // the owners of a share on one compute die
        by_die = 1;
    } else {
        shares = cus / slices > 0 ? cus / slices : 1;
    }
    const long long groups = n / 4;
    if (shares > groups / kCountThreads + 1) {   // a short stream: fewer, fuller shares
        shares = (int)(groups / kCountThreads + 1);
        by_die = 0;
    }
    if ((n + shares - 1) / shares >= (1ll << 32)) return FR_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(count_kernel, dim3((unsigned)(shares * slices)), dim3(kCountThreads), kSlice * 4, s, tokens, n, V,
                       slices, shares, by_die, counts, flag);
    return hip_status(hipGetLastError());
}

fr_status launch_rank_tokens(const long long *counts, int V, int *ranked, hipStream_t s) {
    hipLaunchKernelGGL(rank_kernel, dim3((V + kRankThreads - 1) / kRankThreads), dim3(kRankThreads), 0, s, counts, V,
                       ranked);
    return hip_status(hipGetLastError());
}

}  // namespace frspec
