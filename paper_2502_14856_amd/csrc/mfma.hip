// Matrix-core kernel for many H rows (16 < M <= 256): Eq. 4 as a dense contraction
// [V_rows x d] x [d x M] on v_mfma_f32_16x16x32_bf16, fused with the same online
// log-softmax / top-k / remap epilogue as the skinny kernel.
//
//   * W is the streamed operand: each wavefront owns RB blocks of 16 vocabulary rows and
//     loads its MFMA A fragments straight from HBM into registers (every byte of W is
//     loaded by exactly one wavefront, once), PD chunks of 64 elements ahead;
//   * H is the reused operand: the workgroup stages it through LDS in chunks of 64
//     elements (double buffered), and every wavefront reads its B fragments from there;
//   * inside a 64-element chunk lane group g (= lane / 16) takes elements
//     [16g, 16g + 16): two 16-byte loads that are adjacent in memory, so the four groups
//     cover a 128-byte line of each row.  The contraction does not care about the order
//     of d as long as W and H agree, and both use this mapping;
//   * accumulators hold z[16 rows x 16 m] per (row block, m tile): lane (j, g) owns rows
//     4g..4g+3 of column m = j.
#include "epilogue.hpp"
#include "internal.hpp"

namespace frspec {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kMfmaWaves = 4;
constexpr int kMfmaThreads = kMfmaWaves * kWave;
constexpr int kChunkElems = 64;           // elements of d per LDS stage
constexpr int kChunk16 = kChunkElems / 8; // 16-byte units per row per stage
constexpr int kHPitch16 = kChunk16 + 1;   // padded LDS pitch (144 bytes): conflict-free B reads
constexpr int kZPad = 4;

struct MfmaArgs {
    const u32x4 *H;
    const u32x4 *W;
    const int *idx_map;
    int M, d8, V_rows, k;
    int chunks;   // ceil(d8 / 8)
    int passes;
    int sink;
    Partials part;
    unsigned *ticket;
    int *token_ids;
    float *logp;
    float *z_out;
    int z_ld;
};

__host__ __device__ constexpr int mfma_round_up(int x, int m) { return (x + m - 1) / m * m; }

struct MfmaLds {
    int h_off, z_off, ids_off, ms_off, val_off, id_off, total;
    __host__ __device__ MfmaLds(int MT16, int ZR, int k) {
        const int Mp = MT16 * 16;
        int o = 0;
        h_off = o;   o += 2 * Mp * kHPitch16 * 16;
        z_off = o;   o += 16 * (ZR + kZPad) * 4;
        ids_off = o; o += ZR * 4;
        ms_off = o;  o += Mp * 2 * 4;
        val_off = o; o += Mp * k * 4;
        id_off = o;  o += Mp * k * 4;
        total = mfma_round_up(o, 16);
    }
};

template <int MT16, int RB, int PD>
__global__ __launch_bounds__(kMfmaThreads) void mfma_kernel(MfmaArgs a) {
    constexpr int Mp = MT16 * 16;
    constexpr int ZR = kMfmaWaves * RB * 16;   // vocabulary rows per pass
    constexpr int kHLoads = (Mp * kChunk16 + kMfmaThreads - 1) / kMfmaThreads;
    extern __shared__ u32x4 smem[];
    char *base = reinterpret_cast<char *>(smem);
    const MfmaLds L(MT16, ZR, a.k);
    u32x4 *H_lds = reinterpret_cast<u32x4 *>(base + L.h_off);
    float *z_stage = reinterpret_cast<float *>(base + L.z_off);
    int *ids_lds = reinterpret_cast<int *>(base + L.ids_off);
    float *run_ms = reinterpret_cast<float *>(base + L.ms_off);
    float *run_val = reinterpret_cast<float *>(base + L.val_off);
    int *run_id = reinterpret_cast<int *>(base + L.id_off);
    __shared__ int s_slot;
    __shared__ SelectScratch s_select[kMfmaWaves];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int j = lane & 15;   // A: row inside the 16-row block; B and D: column m
    const int g = lane >> 4;   // A, B: 16-element group of the chunk; D: rows 4g..4g+3

    for (int i = tid; i < Mp * a.k; i += kMfmaThreads) {
        run_val[i] = kNegInf;
        run_id[i] = INT_MAX;
    }
    for (int i = tid; i < Mp; i += kMfmaThreads) {
        run_ms[2 * i] = kNegInf;
        run_ms[2 * i + 1] = 0.0f;
    }

    // global -> register half of the H staging: element (row, c16) of a chunk
    u32x4 hreg[kHLoads];
    auto h_fetch = [&](int chunk) {
#pragma unroll
        for (int u = 0; u < kHLoads; ++u) {
            const int e = tid + u * kMfmaThreads;
            const int row = e / kChunk16, c16 = e - row * kChunk16;
            const int col = chunk * kChunk16 + c16;
            u32x4 v = zero_u32x4();
            if (e < Mp * kChunk16 && row < a.M && col < a.d8) v = a.H[(size_t)row * a.d8 + col];
            hreg[u] = v;
        }
    };
    auto h_store = [&](int buf) {
#pragma unroll
        for (int u = 0; u < kHLoads; ++u) {
            const int e = tid + u * kMfmaThreads;
            const int row = e / kChunk16, c16 = e - row * kChunk16;
            if (e < Mp * kChunk16) H_lds[(buf * Mp + row) * kHPitch16 + c16] = hreg[u];
        }
    };

    for (int p = blockIdx.x; p < a.passes; p += gridDim.x) {
        const int pass_row0 = p * ZR;
        const int n_valid = min(ZR, a.V_rows - pass_row0);
        __syncthreads();   // previous pass has finished with ids_lds, z_stage and H_lds
        if (tid < n_valid) {
            const int row = pass_row0 + tid;
            ids_lds[tid] = a.idx_map ? a.idx_map[row] : row;
        }

        const u32x4 *wrow[RB];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int row = min(pass_row0 + (wave * RB + rb) * 16 + j, a.V_rows - 1);
            wrow[rb] = a.W + (size_t)row * a.d8;
        }
        f32x4_t acc[RB][MT16];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int mt = 0; mt < MT16; ++mt) acc[rb][mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

        u32x4 wreg[PD][RB][2];
        // Past the end of a row the chunk index is clamped: the bytes are valid finite
        // weights and the matching H entries staged in LDS are zero.
        auto w_issue = [&](int slot, int chunk) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    const int c16 = min(chunk * kChunk16 + g * 2 + kk, a.d8 - 1);
                    wreg[slot][rb][kk] = __builtin_nontemporal_load(wrow[rb] + c16);
                }
        };
#pragma unroll
        for (int u = 0; u < PD; ++u)
            if (u < a.chunks) w_issue(u, u);
        h_fetch(0);
        h_store(0);
        __syncthreads();

        for (int c0 = 0; c0 < a.chunks; c0 += PD) {
#pragma unroll
            for (int u = 0; u < PD; ++u) {
                const int c = c0 + u;
                if (c < a.chunks) {
                    const int cur = c & 1;
                    if (c + 1 < a.chunks) h_fetch(c + 1);
#pragma unroll
                    for (int kk = 0; kk < 2; ++kk) {
                        bf16x8_t bfrag[MT16];
#pragma unroll
                        for (int mt = 0; mt < MT16; ++mt)
                            bfrag[mt] = __builtin_bit_cast(
                                bf16x8_t, H_lds[(cur * Mp + mt * 16 + j) * kHPitch16 + g * 2 + kk]);
#pragma unroll
                        for (int rb = 0; rb < RB; ++rb) {
                            const bf16x8_t afrag = __builtin_bit_cast(bf16x8_t, wreg[u][rb][kk]);
#pragma unroll
                            for (int mt = 0; mt < MT16; ++mt)
                                acc[rb][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                    afrag, bfrag[mt], acc[rb][mt], 0, 0, 0);
                        }
                    }
                    if (c + PD < a.chunks) w_issue(u, c + PD);
                    if (c + 1 < a.chunks) h_store(cur ^ 1);
                    __syncthreads();
                }
            }
        }

        // ---- consume the pass, one tile of 16 H rows at a time ----
#pragma unroll
        for (int mt = 0; mt < MT16; ++mt) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                float *dst = z_stage + j * (ZR + kZPad) + (wave * RB + rb) * 16 + 4 * g;
                *reinterpret_cast<f32x4_t *>(dst) = acc[rb][mt];
            }
            __syncthreads();
            if (a.sink == (int)Sink::kLogits) {
                for (int i = tid; i < 16 * ZR; i += kMfmaThreads) {
                    const int ml = i / ZR, r = i - ml * ZR;
                    const int m = mt * 16 + ml;
                    if (m < a.M && r < n_valid)
                        a.z_out[(size_t)m * a.z_ld + pass_row0 + r] = z_stage[ml * (ZR + kZPad) + r];
                }
            } else if (a.sink != (int)Sink::kStreamOnly) {
                const int m_end = min(a.M, mt * 16 + 16);
                auto row_of = [&](int m) {
                    return FoldRow{z_stage + (m - mt * 16) * (ZR + kZPad), run_ms + 2 * m,
                                   run_val + m * a.k, run_id + m * a.k};
                };
                if (p == (int)blockIdx.x)
                    block_fold_all<ZR, false>(mt * 16 + wave, kMfmaWaves, m_end, row_of, 1, 0, ids_lds,
                                              n_valid, a.k, &s_select[wave]);
                else
                    block_fold_all<ZR, true>(mt * 16 + wave, kMfmaWaves, m_end, row_of, 1, 0, ids_lds,
                                             n_valid, a.k, &s_select[wave]);
            }
            __syncthreads();
        }
    }

    if (a.sink == (int)Sink::kLogits || a.sink == (int)Sink::kStreamOnly) return;

    const int gidx = blockIdx.x, G = gridDim.x;
    const Partials part = a.part;   // a local copy keeps the argument block itself in registers
    for (int m = wave; m < a.M; m += kMfmaWaves) {
        if (lane < a.k) {
            publish(part.val + part_index(m * a.k + lane, gidx), run_val[m * a.k + lane]);
            publish(part.id + part_index(m * a.k + lane, gidx), run_id[m * a.k + lane]);
        }
        if (lane < 2) publish(part.ms + part_index(m * 2 + lane, gidx), run_ms[2 * m + lane]);
    }
    if (a.sink == (int)Sink::kPartialsOnly) return;

    const Arrival ar{a.ticket, a.ticket + 1, a.ticket + 2};
    const int R = merger_count(G, a.M);
    const int r = arrive_and_wait(ar, G, R, &s_slot);
    if (r < 0) return;
    final_merge_all(part, G, r + R * wave, R * kMfmaWaves, a.M, a.k, a.token_ids, a.logp, &s_select[wave]);
    merger_done(ar, R);
}

constexpr int kLdsBudget = 160 * 1024;
constexpr int kStaticLdsReserve = 8 * 1024;   // room for the kernel's static LDS (selection scratch)
constexpr int kRB = 2;
constexpr int kPD = 3;
constexpr int kZR = kMfmaWaves * kRB * 16;

template <int MT16>
fr_status launch_one(const MfmaArgs &a, int grid, int lds, hipStream_t s) {
    auto kern = mfma_kernel<MT16, kRB, kPD>;
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                kLdsBudget - kStaticLdsReserve) != hipSuccess) {
            (void)hipGetLastError();
            return FR_ERR_HIP;
        }
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kMfmaThreads), lds, s, a);
    return hip_status(hipGetLastError());
}

int mt16_bucket(int M) {
    const int t = (M + 15) / 16;
    for (int b : {1, 2, 4, 8, 12, 16})
        if (t <= b) return b;
    return -1;
}

}  // namespace

// Largest slab of H rows (multiple of 16, <= 256) whose state fits LDS for this k.
int mfma_max_rows(int k) {
    int best = 0;
    for (int mt : {1, 2, 4, 8, 12, 16})
        if (MfmaLds(mt, kZR, k).total <= kLdsBudget - kStaticLdsReserve) best = mt * 16;
    return best;
}

fr_status launch_mfma(const HeadProblem &p, Sink sink, const fr_tuning *t, hipStream_t s,
                      int *grid_used) {
    const int MT16 = mt16_bucket(p.M);
    if (MT16 < 0) return FR_ERR_UNSUPPORTED;
    const int lds = MfmaLds(MT16, kZR, p.k).total;
    if (lds > kLdsBudget - kStaticLdsReserve) return FR_ERR_UNSUPPORTED;
    const int cus = device_cu_count();
    if (cus <= 0) return FR_ERR_HIP;

    MfmaArgs a{};
    a.H = static_cast<const u32x4 *>(p.H);
    a.W = static_cast<const u32x4 *>(p.W);
    a.idx_map = p.idx_map;
    a.M = p.M;
    a.d8 = p.d / 8;
    a.V_rows = p.V_rows;
    a.k = p.k;
    a.chunks = (a.d8 + kChunk16 - 1) / kChunk16;
    a.passes = (p.V_rows + kZR - 1) / kZR;
    a.sink = (int)sink;
    a.part.ms = p.ws.part_ms;
    a.part.val = p.ws.part_val;
    a.part.id = p.ws.part_id;
    a.ticket = p.ws.ticket;
    a.token_ids = p.token_ids;
    a.logp = p.logp;
    a.z_out = p.z_out;
    a.z_ld = p.z_ld;

    // workgroups per compute unit that the LDS footprint allows
    int per_cu = kLdsBudget / (lds + 512);
    if (per_cu < 1) per_cu = 1;
    if (per_cu > 2) per_cu = 2;
    int grid = cus * per_cu;
    if (grid > a.passes) grid = a.passes;
    if (t && t->grid > 0) grid = t->grid < a.passes ? t->grid : a.passes;
    if (grid > kGridMax) grid = kGridMax;
    if (grid_used) *grid_used = grid;

    fr_status st = FR_ERR_UNSUPPORTED;
    switch (MT16) {
        case 1: st = launch_one<1>(a, grid, lds, s); break;
        case 2: st = launch_one<2>(a, grid, lds, s); break;
        case 4: st = launch_one<4>(a, grid, lds, s); break;
        case 8: st = launch_one<8>(a, grid, lds, s); break;
        case 12: st = launch_one<12>(a, grid, lds, s); break;
        case 16: st = launch_one<16>(a, grid, lds, s); break;
    }
    if (st != FR_OK) return st;
    if (sink == Sink::kPartialsOnly) return launch_merge(p, grid, s);
    return FR_OK;
}

}  // namespace frspec
