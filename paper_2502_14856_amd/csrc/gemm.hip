// Block kernel for many rows of H (65 to 256 per launch): Eq. 4 as a register-blocked dense
// contraction [128 vocabulary rows x d] x [d x Mp] per workgroup on v_mfma_f32_16x16x32_bf16,
// followed by the same online log-softmax / top-k / remap epilogue as the other kernels.
//
// Where the chunked kernel (mfma.hip) gives every wavefront 16 vocabulary rows and ALL rows of H
// (each wavefront then reads every H fragment from LDS, which is what bounds it beyond ~64 rows),
// this kernel tiles both operands: eight wavefronts as 2 (vocabulary) x 4 (rows of H), each
// with a 64 x 16*NT tile of the logits in 16*NT accumulator registers, so a fragment read from
// LDS feeds NT (W fragments) or 4 (H fragments) products.  W is read from memory exactly
// once per call for up to 256 rows of H.
//
//   * both operands go through LDS in K-steps of 64 elements of d: W in a ring of three
//     stages (a load instruction covers 256 contiguous bytes of a row, i.e. two K-steps),
//     H in two buffers; rows are 128 bytes with the 16-byte chunks XOR-swizzled by the row
//     number, so that the fragment reads (16 rows x one chunk per quarter wavefront) touch
//     every bank once without padding (measured: no bank conflicts);
//   * the wavefronts are specialised for the loads, because a wavefront's loads complete in
//     order: wavefronts 0-3 fetch W one slab (256 bytes per row) ahead, wavefronts 4-7
//     fetch H (resident in L2) two K-steps ahead.  One wavefront doing both would have to
//     wait for all its older W loads whenever it needs the next piece of H;
//   * one barrier per K-step: what is written after barrier s is read after barrier s+1;
//   * every workgroup visits the slabs of d cyclically from a different start, as in the
//     other kernels (all workgroups advance at the same pace).
#include <type_traits>

#include "epilogue.hpp"
#include "internal.hpp"

namespace frspec {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) char *GlobalBytes;
typedef const __attribute__((address_space(1))) u32x4 *GlobalVec;
__device__ __forceinline__ u32x4 load_stream(GlobalBytes base, unsigned byte_offset) {
    return __builtin_nontemporal_load(reinterpret_cast<GlobalVec>(base + byte_offset));
}
__device__ __forceinline__ u32x4 load_cached(GlobalBytes base, unsigned byte_offset) {
    return *reinterpret_cast<GlobalVec>(base + byte_offset);
}

constexpr int kTV = 128;           // vocabulary rows per pass
constexpr int kStepChunks = 8;     // 16-byte chunks of d per K-step
constexpr int kSlabChunks = 16;    // chunks per slab = per W load instruction and row
constexpr int kWStages = 3;        // K-steps of W in LDS
constexpr int kWDepth = 1;         // slabs of W in flight per W-loading wavefront (2 or 3 measured 2-3 us slower: the
                                   // compute unit returns loads in order, and the H loads queue behind more W)
constexpr int kStage16 = kTV * kStepChunks;   // 16-byte units per W stage
constexpr int kZPad = 4;
constexpr int kFoldRows = 128;     // rows of H whose logits are staged and folded at once
constexpr int kBlockWaves = 8;
constexpr int kBlockThreads = kBlockWaves * kWave;
constexpr int kRoleThreads = kBlockThreads / 2;   // threads per loading role (four wavefronts)

struct BlockArgs {
    const u32x4 *H;
    const u32x4 *W;
    const int *idx_map;
    int M, d8, V_rows, k;
    int nslabs;   // d8 / 16
    int passes;
    int sink;
    unsigned spin_limit;
    Partials part;
    Mailbox mail;
    int mailbox;
    unsigned *ticket;
    int *token_ids;
    float *logp;
    float *z_out;
    int z_ld;
    long long *trace;
};

__host__ __device__ constexpr int block_round_up(int x, int m) { return (x + m - 1) / m * m; }

struct BlockLds {
    int w_off, h_off, ids_off, ms_off, val_off, id_off, total;
    __host__ __device__ BlockLds(int NT, int k) {
        const int Mp = 64 * NT;
        int o = 0;
        w_off = o;   o += kWStages * kStage16 * 16;
        h_off = o;   o += 2 * Mp * kStepChunks * 16;
        const int z_bytes = kFoldRows * (kTV + kZPad) * 4;   // the logits of a round reuse the operand buffers
        if (o < z_bytes) o = z_bytes;
        ids_off = o; o += kTV * 4;
        ms_off = o;  o += Mp * 2 * 4;
        val_off = o; o += Mp * k * 4;
        id_off = o;  o += Mp * k * 4;
        total = block_round_up(o, 16);
    }
};

// position of chunk c of row `row` inside a stage (16-byte units)
__host__ __device__ constexpr int swizzled(int row, int c) { return row * kStepChunks + (c ^ ((row >> 1) & 7)); }

// LEAN: the build for the plain fused call (sink, mailbox, no trace as compile-time constants), as in
// the skinny kernel.
template <int NT, bool LEAN = false>
__global__ __launch_bounds__(kBlockThreads) void block_kernel(BlockArgs a) {
    constexpr int Mp = 64 * NT;
    constexpr int kHStage16 = Mp * kStepChunks;                 // 16-byte units per H buffer
    constexpr int kWLoads = kTV * kSlabChunks / kRoleThreads;   // per W-loading thread and slab (8)
    constexpr int kHLoads = kHStage16 / kRoleThreads;           // per H-loading thread and K-step (2 NT)
    constexpr int kRegs = kWDepth * kWLoads > 2 * kHLoads ? kWDepth * kWLoads : 2 * kHLoads;
    // slabs after which both rings repeat: three stages at two per slab, kWDepth register sets
    constexpr int U = kWDepth % 3 == 0 ? kWDepth : 3 * kWDepth;
    static_assert(kWStages == 3 && (U == 3 || U == 6), "the ring positions below assume these");

    extern __shared__ u32x4 smem[];
    char *base = reinterpret_cast<char *>(smem);
    const BlockLds L(NT, a.k);
    u32x4 *W_lds = reinterpret_cast<u32x4 *>(base + L.w_off);
    u32x4 *H_lds = reinterpret_cast<u32x4 *>(base + L.h_off);
    float *z_all = reinterpret_cast<float *>(base);
    int *ids_lds = reinterpret_cast<int *>(base + L.ids_off);
    float *run_ms = reinterpret_cast<float *>(base + L.ms_off);
    float *run_val = reinterpret_cast<float *>(base + L.val_off);
    int *run_id = reinterpret_cast<int *>(base + L.id_off);
    __shared__ int s_slot;
    __shared__ SelectScratch s_select[kBlockWaves];
    __shared__ MergeScratch s_merge;

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int j = lane & 15, g = lane >> 4;
    const int wv = wave & 1, wm = wave >> 1;   // this wavefront's tile: rows 64 wv.., columns 16 NT wm..
    const bool w_role = wave < kBlockWaves / 2;
    const int lt = tid & (kRoleThreads - 1);   // thread number inside its loading role
    const int G = gridDim.x;
    auto stamp = [&](int slot) {
        if constexpr (!LEAN)
            if (a.trace && tid == 0) a.trace[blockIdx.x * 8 + slot] = (long long)__builtin_amdgcn_s_memrealtime();
    };
    stamp(0);
    // (lean build: the plain fused call through the mailbox, no phase trace, default wait limit)
    const int sink = LEAN ? (int)Sink::kFusedTopk : a.sink;
    const bool mailbox = LEAN || a.mailbox != 0;
    const Arrival ar(a.ticket);
    const unsigned turn = (!LEAN && sink == (int)Sink::kFusedTopk) ? ar.turn() : 0u;

    for (int i = tid; i < Mp * a.k; i += kBlockThreads) {
        run_val[i] = kNegInf;
        run_id[i] = INT_MAX;
    }
    for (int i = tid; i < Mp; i += kBlockThreads) {
        run_ms[2 * i] = kNegInf;
        run_ms[2 * i + 1] = 0.0f;
    }

    const int nslabs = a.nslabs, nsteps = 2 * nslabs;
    const int q0 = (int)((blockIdx.x + (blockIdx.x >> 3)) % (unsigned)nslabs);
    auto slab_at = [&](int i) {   // i-th slab of the visiting order
        const int q = i + q0;
        return q >= nslabs ? q - nslabs : q;
    };
    auto chunk_of_step = [&](int s) {   // first chunk of the s-th K-step of the visiting order
        return slab_at(s >> 1) * kSlabChunks + (s & 1) * kStepChunks;
    };

    const GlobalBytes Wb = (GlobalBytes)a.W, Hb = (GlobalBytes)a.H;

    // W role: thread (wavefront w of 4, row slot rs, chunk lk) loads rows 32 w + 4 u + rs, u < 8
    // (an instruction covers 4 rows x 256 contiguous bytes)
    const int lk = lane & 15, rs = lane >> 4;
    const int wl_row0 = (wave & 3) * 32 + rs;
    // H role: piece e = lt + 256 u of a K-step: row e / 8, position e % 8 of the stage
    unsigned h_src[kHLoads];
#pragma unroll
    for (int u = 0; u < kHLoads; ++u) {
        const int e = lt + u * kRoleThreads, row = e >> 3, pos = e & 7;
        const int c = pos ^ ((row >> 1) & 7);
        h_src[u] = ((unsigned)min(row, a.M - 1) * (unsigned)a.d8 + (unsigned)c) * 16u;
    }

    // fragment addresses: row j of a 16-row block, chunk (4 kk + g) of the K-step
    const int sw = (j >> 1) & 7;
    const int cpos0 = g ^ sw, cpos1 = (4 + g) ^ sw;
    const u32x4 *a_frag = W_lds + (wv * 64 + j) * kStepChunks;
    const u32x4 *b_frag = H_lds + (wm * 16 * NT + j) * kStepChunks;

    u32x4 stg[kRegs];   // the loads in flight of this thread's role
    f32x4_t acc[4][NT];

    for (int p = blockIdx.x; p < a.passes; p += G) {
        const int pass_row0 = p * kTV;
        const int n_valid = min(kTV, a.V_rows - pass_row0);
        __syncthreads();   // the previous pass is done with every buffer
        // the token id of local row tid % 128: asked for ahead of the operands (unconditionally,
        // see the start-up rules of the other kernels), stored when the products are done
        const int id_row = min(pass_row0 + (tid & (kTV - 1)), a.V_rows - 1);
        const int id_mine = a.idx_map ? __builtin_nontemporal_load(a.idx_map + id_row) : id_row;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int n = 0; n < NT; ++n) acc[t][n] = f32x4_t{0.f, 0.f, 0.f, 0.f};

        unsigned w_src[kWLoads];
#pragma unroll
        for (int u = 0; u < kWLoads; ++u) {
            const int row = min(pass_row0 + wl_row0 + 4 * u, a.V_rows - 1);
            w_src[u] = ((unsigned)row * (unsigned)a.d8 + (unsigned)lk) * 16u;
        }
        // Slab number i of the visiting order into register set `set`.  Past the end of the row the
        // loads stay in the instruction stream (the count of loads in flight stays exact) but
        // read the start of H, which is in cache anyway.
        auto w_issue = [&](int set, int i) {
            const bool real = i < nslabs;
            const GlobalBytes b = real ? Wb : Hb;
            const unsigned add = real ? (unsigned)slab_at(i) * (kSlabChunks * 16u) : 0u;
#pragma unroll
            for (int u = 0; u < kWLoads; ++u)
                stg[set * kWLoads + u] = load_stream(b, real ? w_src[u] + add : (unsigned)lk * 16u);
        };
        // ... and into the two stages that follow `first_stage` in the ring
        auto w_store = [&](int set, int first_stage) {
#pragma unroll
            for (int u = 0; u < kWLoads; ++u) {
                const int row = wl_row0 + 4 * u;
                const int stage = (first_stage + (lk >> 3)) % kWStages;
                W_lds[stage * kStage16 + swizzled(row, lk & 7)] = stg[set * kWLoads + u];
            }
        };
        auto h_issue = [&](int set, int s) {
            const unsigned add = (unsigned)chunk_of_step(min(s, nsteps - 1)) * 16u;
#pragma unroll
            for (int u = 0; u < kHLoads; ++u) stg[set * kHLoads + u] = load_cached(Hb, h_src[u] + add);
        };
        auto h_store = [&](int set, int buf) {
#pragma unroll
            for (int u = 0; u < kHLoads; ++u) H_lds[buf * kHStage16 + lt + u * kRoleThreads] = stg[set * kHLoads + u];
        };

        // the products of one K-step: W stage `st`, H buffer `hb`
        auto products = [&](int st, int hb) {
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                const int cp = kk ? cpos1 : cpos0;
                bf16x8_t af[4], bf[NT];
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    af[t] = __builtin_bit_cast(bf16x8_t, a_frag[st * kStage16 + t * 16 * kStepChunks + cp]);
#pragma unroll
                for (int n = 0; n < NT; ++n)
                    bf[n] = __builtin_bit_cast(bf16x8_t, b_frag[hb * kHStage16 + n * 16 * kStepChunks + cp]);
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int n = 0; n < NT; ++n)
                        acc[t][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[t], bf[n], acc[t][n], 0, 0, 0);
            }
        };

        // Slab number i of the visiting order (K-steps 2i and 2i+1), at ring position QI = i % U.
        // W role: after the barrier of the odd step it stores slab i+1 (whose two stages were
        // last read in K-steps 2i-1 and 2i) and asks for slab i+1+kWDepth.  H role: after every
        // barrier s it stores K-step s+1 and asks for K-step s+3.
        auto slab_round = [&](auto role, auto qi_tag, int i) {
            constexpr bool kWRole = decltype(role)::value;
            constexpr int QI = decltype(qi_tag)::value;
            constexpr int st0 = (2 * QI) % kWStages, st1 = (2 * QI + 1) % kWStages, st2 = (2 * QI + 2) % kWStages;
            constexpr int next_set = (QI + 1) % kWDepth;
            __syncthreads();
            if constexpr (!kWRole) {
                h_store(1, 1);
                h_issue(1, 2 * i + 3);
            }
            // (no scheduling barrier here: the compiler spreads the stores and loads above over the
            // products below, which measured 3 to 6 us faster than keeping them ahead)
            products(st0, 0);
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
            if constexpr (kWRole) {
                w_store(next_set, st2);
                w_issue(next_set, i + 1 + kWDepth);
            } else {
                h_store(0, 0);
                h_issue(0, 2 * i + 4);
            }
            products(st1, 1);
            __builtin_amdgcn_sched_barrier(0);
        };
        auto main_loop = [&](auto role) {
            constexpr bool kWRole = decltype(role)::value;
            // start: the first kWDepth slabs of W requested, slab 0 stored (stages 0 and 1) and the next
            // slab requested; H K-steps 0 and 1 requested, K-step 0 stored (buffer 0), K-step 2 requested
            if constexpr (kWRole) {
#pragma unroll
                for (int q = 0; q < kWDepth; ++q) w_issue(q, q);
                w_store(0, 0);
                w_issue(0, kWDepth);
            } else {
                h_issue(0, 0);
                h_issue(1, 1);
                h_store(0, 0);
                h_issue(0, 2);
            }
            int i = 0;
            for (; i + U <= nslabs; i += U) {
                slab_round(role, std::integral_constant<int, 0>{}, i);
                slab_round(role, std::integral_constant<int, 1>{}, i + 1);
                slab_round(role, std::integral_constant<int, 2>{}, i + 2);
                if constexpr (U == 6) {
                    slab_round(role, std::integral_constant<int, 3>{}, i + 3);
                    slab_round(role, std::integral_constant<int, 4>{}, i + 4);
                    slab_round(role, std::integral_constant<int, 5>{}, i + 5);
                }
            }
            if (i < nslabs) slab_round(role, std::integral_constant<int, 0>{}, i);
            if (i + 1 < nslabs) slab_round(role, std::integral_constant<int, 1>{}, i + 1);
            if constexpr (U == 6) {
                if (i + 2 < nslabs) slab_round(role, std::integral_constant<int, 2>{}, i + 2);
                if (i + 3 < nslabs) slab_round(role, std::integral_constant<int, 3>{}, i + 3);
                if (i + 4 < nslabs) slab_round(role, std::integral_constant<int, 4>{}, i + 4);
            }
        };
        if (w_role)
            main_loop(std::true_type{});
        else
            main_loop(std::false_type{});

        // ---- consume the pass: rounds of 128 rows of H through the operand buffers ----
        stamp(2);
        if (tid < kTV) ids_lds[tid] = id_mine;
        const bool last = p + G >= a.passes;
        for (int m_base = 0; m_base < a.M; m_base += kFoldRows) {
            __syncthreads();   // the products (or the previous round's fold) are done with the buffers
#pragma unroll
            for (int n = 0; n < NT; ++n) {
                const int m0 = (wm * NT + n) * 16;
                if (m0 >= m_base && m0 < m_base + kFoldRows) {
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        float *dst = z_all + (m0 - m_base + j) * (kTV + kZPad) + wv * 64 + t * 16 + 4 * g;
                        *reinterpret_cast<f32x4_t *>(dst) = acc[t][n];
                    }
                }
            }
            __syncthreads();
            const int m_end = min(a.M, m_base + kFoldRows);
            if (sink == (int)Sink::kLogits) {
                for (int e = tid; e < kFoldRows * kTV; e += kBlockThreads) {
                    const int m = m_base + e / kTV, r = e % kTV;
                    if (m < m_end && r < n_valid)
                        a.z_out[(size_t)m * a.z_ld + pass_row0 + r] = z_all[(m - m_base) * (kTV + kZPad) + r];
                }
            } else if (sink != (int)Sink::kStreamOnly) {
                auto row_of = [&](int m) {
                    return FoldRow{z_all + (m - m_base) * (kTV + kZPad), run_ms + 2 * m, run_val + m * a.k,
                                   run_id + m * a.k};
                };
                const FoldSink out{!last ? FoldTo::kLds : (mailbox ? FoldTo::kMailbox : FoldTo::kPartials),
                                   a.part, a.mail, (int)blockIdx.x, run_ms, run_val, run_id};
                auto fold_with = [&](auto b32) {   // (bound from 16 groups up to k = 10, from 32 beyond)
                    constexpr bool B32 = decltype(b32)::value;
                    if (p == (int)blockIdx.x)
                        fold_pass<kTV, false, false, true, B32>(z_all, kTV + kZPad, 1, 0, ids_lds, n_valid, a.k, m_base,
                                                                m_end, wave, kBlockWaves, row_of, out, &s_select[wave]);
                    else
                        fold_pass<kTV, true, false, true, B32>(z_all, kTV + kZPad, 1, 0, ids_lds, n_valid, a.k, m_base,
                                                               m_end, wave, kBlockWaves, row_of, out, &s_select[wave]);
                };
                if (a.k >= kBound32FromK) fold_with(std::true_type{});
                else fold_with(std::false_type{});
            }
        }
    }

    if (sink == (int)Sink::kLogits || sink == (int)Sink::kStreamOnly) return;
    stamp(3);
    const int gidx = blockIdx.x;
    const Partials part = a.part;
    if (mailbox) {
        // as in the chunked kernel: the last R workgroups of the grid merge one row of H each
        const Mailbox mb = a.mail;
        const int R = G < a.M ? G : a.M;
        if (gidx < G - R) return;
        stamp(4);
        const unsigned spin = LEAN ? kMailSpinLimit : (a.spin_limit ? a.spin_limit : kMailSpinLimit);
        if (a.k >= kBound32FromK)
            merge_rows_mailbox<8, true>(mb, part, a.ticket + 1, G, gidx - (G - R), R, a.M, a.k, a.token_ids, a.logp,
                                        &s_merge, &s_select[0], nullptr, spin);
        else
            merge_rows_mailbox<8, false>(mb, part, a.ticket + 1, G, gidx - (G - R), R, a.M, a.k, a.token_ids, a.logp,
                                         &s_merge, &s_select[0], nullptr, spin);
        __syncthreads();
        stamp(5);
        return;
    }
    if (sink == (int)Sink::kPartialsOnly) return;

    const int R = merger_count(G, a.M);
    const int r = arrive_and_wait(ar, (unsigned)__builtin_amdgcn_readfirstlane((int)turn), G, R, &s_slot,
                                  a.spin_limit ? a.spin_limit : kSpinLimit);
    if (r < 0) return;
    if (r & kWaitTimedOut)
        write_no_result((r & ~kWaitTimedOut) + R * wave, R * kBlockWaves, a.M, a.k, a.token_ids, a.logp);
    else
        final_merge_all(part, G, r + R * wave, R * kBlockWaves, a.M, a.k, a.token_ids, a.logp, &s_select[wave]);
}

constexpr int kLdsBudget = 160 * 1024;
constexpr int kStaticLdsReserve = 12 * 1024;

typedef void (*BlockKernel)(BlockArgs);
BlockKernel select_kernel(int nt, bool lean = false) {
    switch (nt) {
        case 2: return lean ? block_kernel<2, true> : block_kernel<2>;
        case 3: return lean ? block_kernel<3, true> : block_kernel<3>;
        case 4: return lean ? block_kernel<4, true> : block_kernel<4>;
    }
    return nullptr;
}
int tiles_for(int M) { return M <= 128 ? 2 : M <= 192 ? 3 : 4; }

}  // namespace

fr_status prepare_block_kernels() {
    for (int b = 0; b < 6; ++b)
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(select_kernel(2 + b / 2, (b & 1) != 0)),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                kLdsBudget - kStaticLdsReserve) != hipSuccess) {
            (void)hipGetLastError();
            return FR_ERR_HIP;
        }
    return FR_OK;
}

bool block_kernel_serves(int M, int d, int k) {
    if (M <= kBlockMinM - 1 || M > kBlockMaxM || (d % 128) != 0 || k > kSmallKMax) return false;
    if ((long long)M * d * 2 > (1ll << 32)) return false;   // H is addressed with 32-bit byte offsets
    return BlockLds(tiles_for(M), k).total <= kLdsBudget - kStaticLdsReserve;
}

fr_status launch_block(const HeadProblem &p, Sink sink, const fr_tuning *t, hipStream_t s) {
    if (!block_kernel_serves(p.M, p.d, p.k)) return FR_ERR_UNSUPPORTED;
    const int nt = tiles_for(p.M);
    const int lds = BlockLds(nt, p.k).total;
    const int cus = device_cu_count();
    if (cus <= 0) return FR_ERR_HIP;

    BlockArgs a{};
    a.H = static_cast<const u32x4 *>(p.H);
    a.W = static_cast<const u32x4 *>(p.W);
    a.idx_map = p.idx_map;
    a.M = p.M;
    a.d8 = p.d / 8;
    a.V_rows = p.V_rows;
    a.k = p.k;
    a.nslabs = a.d8 / kSlabChunks;
    a.passes = (p.V_rows + kTV - 1) / kTV;
    a.sink = (int)sink;
    a.part.ms = p.ws.part_ms;
    a.part.val = p.ws.part_val;
    a.part.id = p.ws.part_id;
    a.ticket = p.ws.ticket;
    a.mail.rec = p.ws.mail_rec;
    a.mail.st = p.ws.mail_st;
    a.token_ids = p.token_ids;
    a.logp = p.logp;
    a.z_out = p.z_out;
    a.z_ld = p.z_ld;
    a.trace = t ? static_cast<long long *>(t->trace) : nullptr;
    a.spin_limit = t && t->spin_limit > 0 ? (unsigned)t->spin_limit : 0u;

    int grid = cus < a.passes ? cus : a.passes;   // one persistent workgroup per compute unit
    if (t && t->grid > 0) grid = t->grid < a.passes ? t->grid : a.passes;
    if (grid > kGridMax) grid = kGridMax;
    a.mailbox = sink == Sink::kFusedTopk && p.k <= kMailK && p.M <= kMailRows && grid <= 4 * kWave &&
                !(t && t->no_mailbox);

    const bool lean = sink == Sink::kFusedTopk && a.mailbox && !a.trace && a.spin_limit == 0u;
    hipLaunchKernelGGL(select_kernel(nt, lean), dim3(grid), dim3(kBlockThreads), lds, s, a);
    const fr_status st = hip_status(hipGetLastError());
    if (st != FR_OK) return st;
    if (sink == Sink::kPartialsOnly) return launch_merge(p, grid, s);
    return FR_OK;
}

}  // namespace frspec
