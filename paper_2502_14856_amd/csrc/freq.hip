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
//   bucket_*      the ranking: ids dealt into buckets by the magnitude of their count, then each id
//                 ranked against its own bucket only (see below); exact, no sorting passes.
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

/*
 * Ranking: ids by count descending, equal counts by lower id.  The position of an id is the number
 * of ids that come before it; counting that against ALL ids is O(V^2).  So the ids are first dealt
 * into 2017 buckets by the magnitude of their count (exponent and five mantissa bits: a bucket
 * spans 3% of a count, and every count below 64 has a bucket of its own), buckets of larger counts
 * first; an id is then compared only with the ids of its own bucket:
 *   bucket_count_kernel    bucket sizes (per-workgroup LDS histogram, then global atomics)
 *   bucket_scan_kernel     start[b] = sizes of all buckets of larger counts (one workgroup)
 *   bucket_scatter_kernel  (count, id) of every id into its bucket's segment, in any order
 *   bucket_rank_kernel     position inside the segment = number of its entries that come first
 *                          (64-bit keys through LDS tiles, one comparison per pair)
 * For a Zipf-like ranking that is ~10^8 comparisons instead of 1.6 * 10^10 at V = 128256; if all
 * counts are equal it is the all-pairs ranking again.  Exact for any int64 counts >= 0.
 */
constexpr int kBuckets = 2048;          // 1 + 63 * 32 = 2017 used
constexpr int kBucketThreads = 1024;
constexpr int kScatterItems = 4;        // ids per thread and tile of the scatter
constexpr int kRankThreads = 256;

__device__ __forceinline__ int bucket_of(long long c) {
    if (c <= 0) return 0;
    const int e = 63 - __clzll(c);   // 0 .. 62
    const int mant = e >= 5 ? (int)((c >> (e - 5)) & 31) : (int)((c << (5 - e)) & 31);
    return 1 + e * 32 + mant;
}

// Inside a bucket all counts agree in their exponent and five mantissa bits; what is left of the
// count (up to 41 bits while the count is below 2^47) and the id (below 2^22) fit one 64-bit key that
// orders like (count descending, id ascending) when compared as unsigned, larger = earlier.  Counts
// of 2^47 and more get key 0 and are compared field by field.
constexpr int kKeyIdBits = 22;
constexpr int kKeyMaxExponent = 46;
__device__ __forceinline__ unsigned long long key_in_bucket(long long c, int id) {
    if (c <= 0) return (unsigned long long)(((1u << kKeyIdBits) - 1u) ^ (unsigned)id) + 1ull;
    const int e = 63 - __clzll(c);
    if (e > kKeyMaxExponent) return 0ull;
    const unsigned long long rest = e > 5 ? (unsigned long long)c & ((1ull << (e - 5)) - 1ull) : 0ull;
    return ((rest << kKeyIdBits) | (unsigned long long)(((1u << kKeyIdBits) - 1u) ^ (unsigned)id)) + 1ull;
}

// table: [0, kBuckets) sizes, [kBuckets, 2 kBuckets) starts, [2 kBuckets, 3 kBuckets) fill counters
__global__ __launch_bounds__(kBucketThreads) void bucket_count_kernel(const long long *__restrict__ counts, int V,
                                                                      unsigned *__restrict__ table) {
    __shared__ unsigned hist[kBuckets];
    for (int b = threadIdx.x; b < kBuckets; b += kBucketThreads) hist[b] = 0u;
    __syncthreads();
    for (int t = blockIdx.x * kBucketThreads + threadIdx.x; t < V; t += gridDim.x * kBucketThreads)
        atomicAdd(&hist[bucket_of(counts[t])], 1u);
    __syncthreads();
    for (int b = threadIdx.x; b < kBuckets; b += kBucketThreads)
        if (hist[b] != 0u) atomicAdd(&table[b], hist[b]);
}

__global__ __launch_bounds__(kBucketThreads) void bucket_scan_kernel(unsigned *__restrict__ table) {
    // suffix sums over the bucket sizes: an inclusive scan of the reversed array, two entries per thread
    __shared__ unsigned sum[2][kBuckets];
    const int tid = threadIdx.x;
    for (int r = tid; r < kBuckets; r += kBucketThreads) sum[0][r] = table[kBuckets - 1 - r];
    __syncthreads();
    int cur = 0;
    for (int step = 1; step < kBuckets; step <<= 1) {
        for (int r = tid; r < kBuckets; r += kBucketThreads)
            sum[cur ^ 1][r] = sum[cur][r] + (r >= step ? sum[cur][r - step] : 0u);
        __syncthreads();
        cur ^= 1;
    }
    for (int r = tid; r < kBuckets; r += kBucketThreads) {
        const int b = kBuckets - 1 - r;
        table[kBuckets + b] = sum[cur][r] - table[b];   // exclusive: the buckets of larger counts only
        table[2 * kBuckets + b] = 0u;
    }
}

__global__ __launch_bounds__(kBucketThreads) void bucket_scatter_kernel(const long long *__restrict__ counts, int V,
                                                                        unsigned *__restrict__ table,
                                                                        long long *__restrict__ seg_count,
                                                                        int *__restrict__ seg_id,
                                                                        unsigned long long *__restrict__ seg_key) {
    __shared__ unsigned local[kBuckets];   // entries of this tile per bucket, then their base in the segment
    constexpr int kTile = kBucketThreads * kScatterItems;
    for (int tile0 = blockIdx.x * kTile; tile0 < V; tile0 += gridDim.x * kTile) {
        for (int b = threadIdx.x; b < kBuckets; b += kBucketThreads) local[b] = 0u;
        __syncthreads();
        long long c[kScatterItems];
        int bucket[kScatterItems];
        unsigned at[kScatterItems];
#pragma unroll
        for (int u = 0; u < kScatterItems; ++u) {
            const int t = tile0 + u * kBucketThreads + threadIdx.x;
            c[u] = t < V ? counts[t] : 0;
            bucket[u] = bucket_of(c[u]);
            at[u] = t < V ? atomicAdd(&local[bucket[u]], 1u) : 0u;
        }
        __syncthreads();
        for (int b = threadIdx.x; b < kBuckets; b += kBucketThreads)
            if (local[b] != 0u) local[b] = table[kBuckets + b] + atomicAdd(&table[2 * kBuckets + b], local[b]);
        __syncthreads();
#pragma unroll
        for (int u = 0; u < kScatterItems; ++u) {
            const int t = tile0 + u * kBucketThreads + threadIdx.x;
            if (t < V) {
                const unsigned pos = local[bucket[u]] + at[u];
                seg_count[pos] = c[u];
                seg_id[pos] = t;
                seg_key[pos] = key_in_bucket(c[u], t);
            }
        }
        __syncthreads();
    }
}

constexpr int kRankTile = 2048;

__global__ __launch_bounds__(kRankThreads) void bucket_rank_kernel(const unsigned *__restrict__ table,
                                                                   const long long *__restrict__ seg_count,
                                                                   const int *__restrict__ seg_id,
                                                                   const unsigned long long *__restrict__ seg_key,
                                                                   int V, int *__restrict__ ranked) {
    // A workgroup takes 256 consecutive entries of the segments; the buckets they belong to form one
    // contiguous range of entries, which goes through LDS in tiles; a thread counts, among the entries
    // of its own bucket, those that come first.
    __shared__ unsigned long long tile[kRankTile];
    __shared__ int s_range[2];
    const int e0 = blockIdx.x * kRankThreads, e = e0 + threadIdx.x;
    const bool real = e < V;
    const long long mine = real ? seg_count[e] : 0;
    const int id = real ? seg_id[e] : 0;
    const unsigned long long mine_key = real ? seg_key[e] : 0ull;
    const int b = bucket_of(mine);
    const int first = real ? (int)table[kBuckets + b] : 0, n = real ? (int)table[b] : 0;
    if (threadIdx.x == 0) s_range[0] = first;
    if (e == min(e0 + kRankThreads, V) - 1) s_range[1] = first + n;
    __syncthreads();
    const int range_lo = s_range[0], range_hi = s_range[1];
    int before = 0;   // entries of the bucket that precede this one in the ranking
    for (int base = range_lo; base < range_hi; base += kRankTile) {
        __syncthreads();
        for (int j = threadIdx.x; j < kRankTile; j += kRankThreads) tile[j] = base + j < range_hi ? seg_key[base + j] : 0ull;
        __syncthreads();
        const int lo = max(base, first), hi = min(base + kRankTile, first + n);
        if (mine_key != 0ull) {
#pragma unroll 4
            for (int j = lo; j < hi; ++j) before += tile[j - base] > mine_key;
        } else {   // counts of 2^47 and more: field by field, from memory
            for (int j = lo; j < hi; ++j) {
                const long long cj = seg_count[j];
                before += cj > mine || (cj == mine && seg_id[j] < id);
            }
        }
    }
    if (real) ranked[first + before] = id;
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
    // temporary device memory, allocated and freed in stream order: the bucket table and the
    // (count, id) segments
    const size_t table_bytes = 3 * kBuckets * sizeof(unsigned);
    const size_t seg_count_off = (table_bytes + 255) & ~static_cast<size_t>(255);
    const size_t seg_id_off = seg_count_off + static_cast<size_t>(V) * sizeof(long long);
    const size_t seg_key_off = (seg_id_off + static_cast<size_t>(V) * sizeof(int) + 255) & ~static_cast<size_t>(255);
    const size_t bytes = seg_key_off + static_cast<size_t>(V) * sizeof(unsigned long long);
    void *tmp = nullptr;
    if (hipMallocAsync(&tmp, bytes, s) != hipSuccess || !tmp) {
        (void)hipGetLastError();
        return FR_ERR_HIP;
    }
    unsigned *table = static_cast<unsigned *>(tmp);
    long long *seg_count = reinterpret_cast<long long *>(static_cast<char *>(tmp) + seg_count_off);
    int *seg_id = reinterpret_cast<int *>(static_cast<char *>(tmp) + seg_id_off);
    unsigned long long *seg_key = reinterpret_cast<unsigned long long *>(static_cast<char *>(tmp) + seg_key_off);
    fr_status st = launch_fill_u32(table, 3 * kBuckets, 0u, s);
    if (st == FR_OK) {
        const int cus = device_cu_count();
        int grid = (V + kBucketThreads * kScatterItems - 1) / (kBucketThreads * kScatterItems);
        if (cus > 0 && grid > cus) grid = cus;
        hipLaunchKernelGGL(bucket_count_kernel, dim3(grid), dim3(kBucketThreads), 0, s, counts, V, table);
        hipLaunchKernelGGL(bucket_scan_kernel, dim3(1), dim3(kBucketThreads), 0, s, table);
        hipLaunchKernelGGL(bucket_scatter_kernel, dim3(grid), dim3(kBucketThreads), 0, s, counts, V, table, seg_count,
                           seg_id, seg_key);
        hipLaunchKernelGGL(bucket_rank_kernel, dim3((V + kRankThreads - 1) / kRankThreads), dim3(kRankThreads), 0, s,
                           table, seg_count, seg_id, seg_key, V, ranked);
        st = hip_status(hipGetLastError());
    }
    if (hipFreeAsync(tmp, s) != hipSuccess) {
        (void)hipGetLastError();
        return FR_ERR_HIP;
    }
    return st;
}

}  // namespace frspec
