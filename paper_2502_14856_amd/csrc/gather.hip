// Eq. 3: W_sub[i, :] = W_full[ids[i], :], idx_map[i] = ids[i].  A pure copy: one
// wavefront moves one row at a time with 16-byte loads and stores.
#include "internal.hpp"
#include "wave_ops.hpp"

namespace frspec {
namespace {

constexpr int kGatherThreads = 256;
constexpr int kGatherWaves = kGatherThreads / 64;

__global__ __launch_bounds__(kGatherThreads) void gather_kernel(const u32x4 *__restrict__ W_full,
                                                                int V, int d8,
                                                                const int *__restrict__ ids,
                                                                int V_sub, u32x4 *__restrict__ W_sub,
                                                                int *__restrict__ idx_map,
                                                                int *flag) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int stride = gridDim.x * kGatherWaves;
    for (int i = blockIdx.x * kGatherWaves + wave; i < V_sub; i += stride) {
        const int id = ids[i];
        const bool ok = (id >= 0) && (id < V);   // uniform over the wavefront
        if (lane == 0) {
            idx_map[i] = ok ? id : -1;
            if (!ok && flag) *flag = 1;
        }
        if (!ok) continue;
        const u32x4 *src = W_full + (size_t)id * d8;
        u32x4 *dst = W_sub + (size_t)i * d8;
        int c = lane;
        for (; c + 192 < d8; c += 256) {   // four independent 16-byte moves in flight
            u32x4 v0 = __builtin_nontemporal_load(src + c);
            u32x4 v1 = __builtin_nontemporal_load(src + c + 64);
            u32x4 v2 = __builtin_nontemporal_load(src + c + 128);
            u32x4 v3 = __builtin_nontemporal_load(src + c + 192);
            __builtin_nontemporal_store(v0, dst + c);
            __builtin_nontemporal_store(v1, dst + c + 64);
            __builtin_nontemporal_store(v2, dst + c + 128);
            __builtin_nontemporal_store(v3, dst + c + 192);
        }
        for (; c < d8; c += 64) __builtin_nontemporal_store(__builtin_nontemporal_load(src + c), dst + c);
    }
}

// The same gather into the tiled layout: 16 rows form a tile; inside a tile the 16-byte chunk
// (row i, elements 32*kb + 8*g .. + 7) sits at chunk index kb*64 + g*16 + i, so that every
// 1 KiB block is one matrix-core A operand in lane order.  Rows past V_sub (padding of the
// last tile) and rows with an id outside [0, V) are zero.  One workgroup per tile; thread t
// moves chunks t, t + 256, ...: 256 contiguous bytes of each of the 16 rows per round.
__global__ __launch_bounds__(kGatherThreads) void gather_tiled_kernel(const u32x4 *__restrict__ W_full, int V,
                                                                      int d8, const int *__restrict__ ids,
                                                                      int V_sub, u32x4 *__restrict__ W_tiled,
                                                                      int *__restrict__ idx_map, int *flag) {
    __shared__ int row_of[16];
    const int tiles = (V_sub + 15) / 16;
    for (int tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        __syncthreads();
        if (threadIdx.x < 16) {
            const int i = tile * 16 + threadIdx.x;
            int id = -1;
            if (i < V_sub) {
                id = ids[i];
                const bool ok = (id >= 0) && (id < V);
                idx_map[i] = ok ? id : -1;
                if (!ok) {
                    id = -1;
                    if (flag) *flag = 1;
                }
            }
            row_of[threadIdx.x] = id;
        }
        __syncthreads();
        u32x4 *dst = W_tiled + (size_t)tile * 16 * d8;
        for (int o = threadIdx.x; o < 16 * d8; o += kGatherThreads) {
            const int kb = o >> 6, g = (o >> 4) & 3, i = o & 15;
            const int id = row_of[i];
            u32x4 v = zero_u32x4();
            if (id >= 0) v = __builtin_nontemporal_load(W_full + (size_t)id * d8 + kb * 4 + g);
            __builtin_nontemporal_store(v, dst + o);
        }
    }
}

}  // namespace

fr_status launch_gather_tiled(const void *W_full, int64_t V, int64_t d, const int32_t *ids,
                              int64_t V_sub, void *W_tiled, int32_t *idx_map, int32_t *flag,
                              hipStream_t s) {
    const int cus = device_cu_count();
    if (cus <= 0) return FR_ERR_HIP;
    int64_t blocks = (V_sub + 15) / 16;
    const int64_t cap = (int64_t)cus * 8;
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(gather_tiled_kernel, dim3((unsigned)blocks), dim3(kGatherThreads), 0, s,
                       static_cast<const u32x4 *>(W_full), (int)V, (int)(d / 8), ids, (int)V_sub,
                       static_cast<u32x4 *>(W_tiled), idx_map, flag);
    return hip_status(hipGetLastError());
}

fr_status launch_gather(const void *W_full, int64_t V, int64_t d, const int32_t *ids,
                        int64_t V_sub, void *W_sub, int32_t *idx_map, int32_t *flag,
                        hipStream_t s) {
    const int cus = device_cu_count();
    if (cus <= 0) return FR_ERR_HIP;
    int64_t blocks = (V_sub + kGatherWaves - 1) / kGatherWaves;
    const int64_t cap = (int64_t)cus * 8;
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(gather_kernel, dim3((unsigned)blocks), dim3(kGatherThreads), 0, s,
                       static_cast<const u32x4 *>(W_full), (int)V, (int)(d / 8), ids, (int)V_sub,
                       static_cast<u32x4 *>(W_sub), idx_map, flag);
    return hip_status(hipGetLastError());
}

}  // namespace frspec
