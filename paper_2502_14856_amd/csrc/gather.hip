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

}  // namespace

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
