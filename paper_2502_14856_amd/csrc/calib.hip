// Plain streaming kernels of known traffic, used to calibrate hardware counters and to
// report what a trivial copy / read achieves on the same device.
#include "internal.hpp"
#include "wave_ops.hpp"

namespace frspec {
namespace {

constexpr int kThreads = 256;

__global__ __launch_bounds__(kThreads) void copy_kernel(u32x4 *__restrict__ dst,
                                                        const u32x4 *__restrict__ src, size_t n) {
    const size_t stride = (size_t)gridDim.x * kThreads;
    size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    for (; i + 3 * stride < n; i += 4 * stride) {
        u32x4 a = __builtin_nontemporal_load(src + i);
        u32x4 b = __builtin_nontemporal_load(src + i + stride);
        u32x4 c = __builtin_nontemporal_load(src + i + 2 * stride);
        u32x4 d = __builtin_nontemporal_load(src + i + 3 * stride);
        __builtin_nontemporal_store(a, dst + i);
        __builtin_nontemporal_store(b, dst + i + stride);
        __builtin_nontemporal_store(c, dst + i + 2 * stride);
        __builtin_nontemporal_store(d, dst + i + 3 * stride);
    }
    for (; i < n; i += stride) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// Each workgroup reads one contiguous slab, eight 16-byte loads per thread in flight.
__global__ __launch_bounds__(kThreads) void read_kernel(const u32x4 *__restrict__ src, size_t n,
                                                        u32x4 *sink) {
    const size_t per_block = (n + gridDim.x - 1) / gridDim.x;
    const size_t lo = (size_t)blockIdx.x * per_block;
    const size_t hi = lo + per_block < n ? lo + per_block : n;
    u32x4 acc = zero_u32x4();
    size_t i = lo + threadIdx.x;
    for (; i + 7 * kThreads < hi; i += 8 * kThreads) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * kThreads);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            acc.x ^= v[u].x;
            acc.y ^= v[u].y;
            acc.z ^= v[u].z;
            acc.w ^= v[u].w;
        }
    }
    for (; i < hi; i += kThreads) {
        u32x4 v = __builtin_nontemporal_load(src + i);
        acc.x ^= v.x;
        acc.y ^= v.y;
        acc.z ^= v.z;
        acc.w ^= v.w;
    }
    // a store that practically never happens keeps the loads alive
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u && acc.x == 0x7F4A7C15u) *sink = acc;
}

__global__ void fill_u32_kernel(unsigned *dst, size_t n, unsigned value) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = value;
}

}  // namespace

fr_status launch_copy(void *dst, const void *src, size_t bytes, hipStream_t s) {
    const int cus = device_cu_count();
    if (cus <= 0) return FR_ERR_HIP;
    const size_t n = bytes / 16;
    size_t blocks = (n + kThreads - 1) / kThreads;
    const size_t cap = (size_t)cus * 8;
    if (blocks > cap) blocks = cap;
    if (blocks == 0) return FR_OK;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, s,
                       static_cast<u32x4 *>(dst), static_cast<const u32x4 *>(src), n);
    return hip_status(hipGetLastError());
}

fr_status launch_read(const void *src, size_t bytes, void *sink, hipStream_t s) {
    const int cus = device_cu_count();
    if (cus <= 0) return FR_ERR_HIP;
    const size_t n = bytes / 16;
    if (n == 0) return FR_OK;
    size_t blocks = (size_t)cus * 8;
    if (blocks > (n + kThreads - 1) / kThreads) blocks = (n + kThreads - 1) / kThreads;
    hipLaunchKernelGGL(read_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, s,
                       static_cast<const u32x4 *>(src), n, static_cast<u32x4 *>(sink));
    return hip_status(hipGetLastError());
}

fr_status launch_fill_u32(unsigned *dst, size_t n, unsigned value, hipStream_t s) {
    if (n == 0) return FR_OK;
    const unsigned blocks = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks), dim3(256), 0, s, dst, n, value);
    return hip_status(hipGetLastError());
}

}  // namespace frspec
