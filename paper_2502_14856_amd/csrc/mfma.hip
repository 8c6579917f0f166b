// Wide kernel for many H rows (up to 128 per launch; more rows run as several launches):
// Eq. 4 as a dense contraction
// [V_rows x d] x [d x M] on v_mfma_f32_16x16x32_bf16, fused with the same online
// log-softmax / top-k / remap epilogue as the skinny kernel.
//
//   * W is the streamed operand and is read exactly once, with the load pattern that
//     streams best (one instruction = 4 rows x 256 contiguous bytes, a register pipeline
//     of DEPTH steps, every workgroup starting at a different column).  A wavefront owns
//     RB blocks of 16 vocabulary rows; each 16 x 128 slab is transposed through a
//     per-wavefront LDS buffer into MFMA operand order;
//   * H is the reused operand and no longer fits LDS as a whole: the workgroup stages it
//     in chunks of HCH x 64 elements of d (double buffered, one barrier per chunk), and
//     every wavefront reads its B fragments from there;
//   * accumulators hold z[16 rows x 16 m] per (row block, m tile): lane (j, g) owns rows
//     4g..4g+3 of column m = j.
// Six builds, all 8 wavefronts x 16 rows: 1, 2, 3, 4, 6 or 8 tiles of 16 rows of H (M <= 16, 32,
// 48, 64, 96, 128), with H chunks of 512, 512, 512, 256, 256 and 128 elements; bound by HBM up to about 100 rows of
// H, by the matrix cores and the LDS reads of the H fragments beyond.
#include <type_traits>

#include "epilogue.hpp"
#include "internal.hpp"

namespace frspec {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) char *GlobalBytes;
typedef const __attribute__((address_space(1))) u32x4 *GlobalVec;
__device__ __forceinline__ u32x4 load_w(GlobalBytes base, unsigned byte_offset) {
    return __builtin_nontemporal_load(reinterpret_cast<GlobalVec>(base + byte_offset));
}

constexpr int kStep16 = 16;                    // 16-byte chunks of d per step (128 elements)
constexpr int kStagePitch16 = kStep16 + 1;     // 272-byte staging rows
constexpr int kZPad = 4;
constexpr int kZR = 128;                       // vocabulary rows per pass, all builds

struct WideArgs {
    const u32x4 *H;
    const u32x4 *W;
    const int *idx_map;
    int M, d8, V_rows, k;
    int steps;    // ceil(d8 / 16)
    int passes;
    int sink;
    unsigned spin_limit;  // polls after which a wait for other workgroups is given up (0: the default)
    Partials part;
    Mailbox mail;
    int mailbox;  // the results go through the mailbox records (single launch, k <= 16, M <= 128)
    unsigned *ticket;
    int *token_ids;
    float *logp;
    float *z_out;
    int z_ld;
    long long *trace;   // optional [gridDim.x][8] phase timestamps (100 MHz clock)
};

__host__ __device__ constexpr int wide_round_up(int x, int m) { return (x + m - 1) / m * m; }

struct WideLds {
    int h_off, stage_off, ids_off, ms_off, val_off, id_off, total;
    __host__ __device__ WideLds(int MT16, int HCH, int k) {
        const int Mp = MT16 * 16;
        int o = 0;
        h_off = o;     o += 2 * Mp * (HCH * 8 + 1) * 16;
        stage_off = o; o += kZR * kStagePitch16 * 16;
        ids_off = o;   o += kZR * 4;
        ms_off = o;    o += Mp * 2 * 4;
        val_off = o;   o += Mp * k * 4;
        id_off = o;    o += Mp * k * 4;
        total = wide_round_up(o, 16);
    }
};

// LEAN: the build for the plain fused call (sink, mailbox, no trace as compile-time constants), as in
// the skinny kernel.
template <int MT16, int RB, int WAVES, int DEPTH, int HCH, bool LEAN = false>
__global__ __launch_bounds__(WAVES * kWave) void wide_kernel(WideArgs a) {
    static_assert(WAVES * RB * 16 == kZR, "a pass is 128 vocabulary rows");
    static_assert((2 * DEPTH) % HCH == 0, "groups of steps start on an H chunk boundary");
    constexpr int Mp = MT16 * 16;
    constexpr int NT = WAVES * kWave;
    constexpr int HP = HCH * 8 + 1;                        // H chunk pitch in 16-byte units
    constexpr int kHLoads = (Mp * HCH * 8 + NT - 1) / NT;  // 16-byte loads per thread per chunk
    constexpr int kRowsPerLane = 4;
    constexpr unsigned kStepBytes = kStep16 * 16;
    extern __shared__ u32x4 smem[];
    char *base = reinterpret_cast<char *>(smem);
    const WideLds L(MT16, HCH, a.k);
    u32x4 *H_lds = reinterpret_cast<u32x4 *>(base + L.h_off);
    u32x4 *stage_lds = reinterpret_cast<u32x4 *>(base + L.stage_off);
    int *ids_lds = reinterpret_cast<int *>(base + L.ids_off);
    float *run_ms = reinterpret_cast<float *>(base + L.ms_off);
    float *run_val = reinterpret_cast<float *>(base + L.val_off);
    int *run_id = reinterpret_cast<int *>(base + L.id_off);
    __shared__ int s_slot;
    __shared__ SelectScratch s_select[WAVES];
    __shared__ MergeScratch s_merge;

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int lk = lane & 15, rs = lane >> 4;   // load layout: 16-byte chunk, row slot
    const int j = lk, g = rs;                   // operand layout: row / column, k group
    const int G = gridDim.x;
    auto stamp = [&](int slot) {
        if constexpr (!LEAN)
            if (a.trace && tid == 0) a.trace[blockIdx.x * 8 + slot] = (long long)__builtin_amdgcn_s_memrealtime();
    };
    stamp(0);
    // which arrival counter this call uses: asked for now, needed at the very end
    // (lean build: the plain fused call through the mailbox, no phase trace, default wait limit)
    const int sink = LEAN ? (int)Sink::kFusedTopk : a.sink;
    const bool mailbox = LEAN || a.mailbox != 0;
    const Arrival ar(a.ticket);
    const unsigned turn = (!LEAN && sink == (int)Sink::kFusedTopk) ? ar.turn() : 0u;

    for (int i = tid; i < Mp * a.k; i += NT) {
        run_val[i] = kNegInf;
        run_id[i] = INT_MAX;
    }
    for (int i = tid; i < Mp; i += NT) {
        run_ms[2 * i] = kNegInf;
        run_ms[2 * i + 1] = 0.0f;
    }

    // Order in which the steps along d are visited: whole groups of DEPTH full steps,
    // cyclically from a group that differs per workgroup (all workgroups advance at the
    // same pace; see the skinny kernel), then the leftover steps.
    const int full_steps = a.d8 / kStep16;
    const int groups = full_steps / DEPTH;
    const int np = groups * DEPTH;
    // (workgroup b runs on compute die b % 8: with an even number of groups, b % groups alone
    // would give all workgroups of a die the same columns at any moment, and the dies then
    // finish up to 7 us apart; the second term spreads every die over all the groups)
    const int g_first =
        groups > 0 ? (int)((blockIdx.x + ((groups & 1) ? 0u : blockIdx.x >> 3)) % (unsigned)groups) : 0;
    auto step_at = [&](int i) {
        if (i >= np) return i;
        int s = g_first * DEPTH + i;
        return s >= np ? s - np : s;
    };

    // H chunk c = elements [c * HCH * 64, (c + 1) * HCH * 64) of d, all Mp rows (zero padded)
    // Every load is issued unconditionally, from a clamped (always valid) address: a load
    // under a branch leaves the compiler without the number of loads outstanding behind
    // it, and it then waits for all of them (vmcnt(0)), which would drain the W pipeline at
    // every chunk.  What must read as zero is masked when the chunk is written to LDS.
    u32x4 hreg[kHLoads];
    unsigned hvalid = 0u;   // bit u: piece u of the fetched chunk is inside H
    auto h_fetch = [&](int c) {
        hvalid = 0u;
#pragma unroll
        for (int u = 0; u < kHLoads; ++u) {
            const int e = tid + u * NT;
            const int row = e / (HCH * 8), c16 = e - row * (HCH * 8);
            const int col = c * (HCH * 8) + c16;
            hreg[u] = a.H[(size_t)min(row, a.M - 1) * a.d8 + min(col, a.d8 - 1)];
            if (e < Mp * HCH * 8 && row < a.M && col < a.d8) hvalid |= 1u << u;
        }
    };
    auto h_store = [&](int buf) {
#pragma unroll
        for (int u = 0; u < kHLoads; ++u) {
            const int e = tid + u * NT;
            const int row = e / (HCH * 8), c16 = e - row * (HCH * 8);
            if (e < Mp * HCH * 8) H_lds[(buf * Mp + row) * HP + c16] = ((hvalid >> u) & 1u) ? hreg[u] : zero_u32x4();
        }
    };

    const GlobalBytes Wb = (GlobalBytes)a.W;
    auto row_offsets = [&](int pass, unsigned (&wo)[RB][kRowsPerLane]) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int r = 0; r < kRowsPerLane; ++r) {
                const int row = min(pass * kZR + (wave * RB + rb) * 16 + rs * kRowsPerLane + r, a.V_rows - 1);
                wo[rb][r] = ((unsigned)row * (unsigned)a.d8 + (unsigned)lk) * 16u;
            }
    };
    u32x4 wb[DEPTH][RB][kRowsPerLane];
    unsigned wo[RB][kRowsPerLane];
    auto w_issue = [&](int u, int s) {   // full step s, no bounds handling
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int r = 0; r < kRowsPerLane; ++r)
                wb[u][rb][r] = load_w(Wb, wo[rb][r] + (unsigned)s * kStepBytes);
    };
    // token id of local row `tid` of a pass: asked for before that pass's loads of W, so that
    // waiting for it does not mean waiting for them
    const int *idx_or_null = a.idx_map;
    auto request_id = [&](int pass) {
        const int row = min(pass * kZR + (tid < kZR ? tid : 0), a.V_rows - 1);
        return idx_or_null ? __builtin_nontemporal_load(idx_or_null + row) : row;
    };

    // Start of the stream (the host launches no more workgroups than there are passes): the
    // ids and the first H chunk are requested first, the first DEPTH steps of W right behind
    // them, all unconditionally (when the row has fewer steps than the pipeline is deep the
    // surplus loads are clamped into the matrix and never used).
    int p = blockIdx.x;
    const int first_chunk = (2 * step_at(0)) / HCH;
    int id_next = request_id(p);
    h_fetch(first_chunk);
    {
        const unsigned w_last = ((unsigned)a.V_rows * (unsigned)a.d8 - 1u) * 16u;
        row_offsets(p, wo);
#pragma unroll
        for (int u = 0; u < DEPTH; ++u)
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int r = 0; r < kRowsPerLane; ++r)
                    wb[u][rb][r] = load_w(Wb, min(wo[rb][r] + (unsigned)step_at(u) * kStepBytes, w_last));
    }

    for (; p < a.passes; p += G) {
        const int pass_row0 = p * kZR;
        const int n_valid = min(kZR, a.V_rows - pass_row0);
        __syncthreads();   // the previous pass is done with ids_lds and the H buffers (its logits)
        if (tid < n_valid) ids_lds[tid] = id_next;
        h_store(0);   // the first chunk: fetched at the start, or while the previous pass drained

        f32x4_t acc[RB][MT16];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int mt = 0; mt < MT16; ++mt) acc[rb][mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

        // Step number i of the visiting order; its 16 x 128 slab(s) of W are in `w`.  The two
        // halves of a step may lie in different H chunks.
        // `sub0` = (2 * i) % HCH: a compile-time constant in the unrolled pipelined steps.
        bool have_next = false;
        auto process_step = [&](int i, int sub0, const u32x4 (&w)[RB][kRowsPerLane]) {
            bf16x8_t af[RB][4];
#pragma unroll
            for (int hs = 0; hs < 2; ++hs) {
                const int h = 2 * i + hs;          // half-step number in visiting order
                const int sub = (sub0 + hs) % HCH; // its place inside the current H chunk
                const int buf = (h / HCH) & 1;
                if (sub == 0) {
                    __syncthreads();               // the chunk in `buf` is complete; the other buffer is free
                    const int h2 = h + HCH;
                    have_next = h2 < 2 * a.steps;
                    // always a fetch: behind the last chunk of a pass comes the first one again,
                    // which the next pass (if there is one) starts with
                    h_fetch(have_next ? (2 * step_at(h2 >> 1) + (h2 & 1)) / HCH : first_chunk);
                }
                if (hs == 0) {
                    // transpose the slab into operand order through this wavefront's staging rows
                    u32x4 *st = stage_lds + wave * (RB * 16 * kStagePitch16);
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                        for (int r = 0; r < kRowsPerLane; ++r)
                            st[(rb * 16 + rs * kRowsPerLane + r) * kStagePitch16 + lk] = w[rb][r];
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                        for (int kk = 0; kk < 4; ++kk)
                            af[rb][kk] = __builtin_bit_cast(bf16x8_t, st[(rb * 16 + j) * kStagePitch16 + kk * 4 + g]);
                }
#pragma unroll
                for (int kk2 = 0; kk2 < 2; ++kk2) {
#pragma unroll
                    for (int mt = 0; mt < MT16; ++mt) {
                        const bf16x8_t bf = __builtin_bit_cast(
                            bf16x8_t, H_lds[(buf * Mp + mt * 16 + j) * HP + sub * 8 + kk2 * 4 + g]);
#pragma unroll
                        for (int rb = 0; rb < RB; ++rb)
                            acc[rb][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[rb][2 * hs + kk2], bf,
                                                                                  acc[rb][mt], 0, 0, 0);
                    }
                }
                if (sub == HCH - 1) {
                    // (pinned behind the products: the wait for the chunk belongs here, not before them)
                    __builtin_amdgcn_sched_barrier(0);
                    if (have_next) h_store(buf ^ 1);
                }
            }
        };

        // Steady state: consume stage u, refill it with the same stage of the next group
        // (unconditionally: the drain below is a copy of its own).
        int i = 0;
        for (int grp = 0; grp + 1 < groups; ++grp) {
#pragma unroll
            for (int u = 0; u < DEPTH; ++u) {
                process_step(i, (2 * u) % HCH, wb[u]);
                __builtin_amdgcn_sched_barrier(0);
                w_issue(u, step_at(i + DEPTH));
                __builtin_amdgcn_sched_barrier(0);
                ++i;
            }
        }
        if (groups > 0) {
            if (p + G < a.passes) {   // the stages freed here start on the next pass of this workgroup
                id_next = request_id(p + G);
                row_offsets(p + G, wo);
#pragma unroll
                for (int u = 0; u < DEPTH; ++u) {
                    process_step(i, (2 * u) % HCH, wb[u]);
                    __builtin_amdgcn_sched_barrier(0);
                    w_issue(u, step_at(u));
                    __builtin_amdgcn_sched_barrier(0);
                    ++i;
                }
            } else {
#pragma unroll
                for (int u = 0; u < DEPTH; ++u) {
                    process_step(i, (2 * u) % HCH, wb[u]);
                    ++i;
                }
            }
        } else if (p + G < a.passes) {
            id_next = request_id(p + G);
        }
        if (i < a.steps) {
            // Leftover steps, not pipelined.  A chunk index past the end of the row is clamped:
            // the bytes loaded are valid finite weights and the matching H entries are zero.
            unsigned wr[RB][kRowsPerLane];
            row_offsets(p, wr);
            for (; i < a.steps; ++i) {
                const int c = min(i * kStep16 + lk, a.d8 - 1) - lk;
                u32x4 w[RB][kRowsPerLane];
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                    for (int r = 0; r < kRowsPerLane; ++r) w[rb][r] = load_w(Wb, wr[rb][r] + (unsigned)c * 16u);
                process_step(i, (2 * i) % HCH, w);
            }
        }

        // ---- consume the pass ----
        // The logits of all Mp rows go into the two H buffers (no longer needed once the
        // products are done) in one piece, and every wavefront folds its rows of H without
        // meeting the others again.
        static_assert(2 * HP * 16 >= (kZR + kZPad) * 4, "the H buffers hold the logits of a pass");
        stamp(2);
        {
            float *z_all = reinterpret_cast<float *>(H_lds);
            __syncthreads();   // every wavefront is done with the H chunks
#pragma clang loop unroll(full)
            for (int mt = 0; mt < MT16; ++mt)
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    float *dst = z_all + (mt * 16 + j) * (kZR + kZPad) + (wave * RB + rb) * 16 + 4 * g;
                    *reinterpret_cast<f32x4_t *>(dst) = acc[rb][mt];
                }
            __syncthreads();
            if (sink == (int)Sink::kLogits) {
                for (int e = tid; e < Mp * kZR; e += NT) {
                    const int m = e / kZR, r = e - m * kZR;
                    if (m < a.M && r < n_valid)
                        a.z_out[(size_t)m * a.z_ld + pass_row0 + r] = z_all[m * (kZR + kZPad) + r];
                }
            } else if (sink != (int)Sink::kStreamOnly) {
                auto row_of = [&](int m) {
                    return FoldRow{z_all + m * (kZR + kZPad), run_ms + 2 * m, run_val + m * a.k, run_id + m * a.k};
                };
                // the last pass of the workgroup writes its result out instead of keeping it
                const bool last = p + G >= a.passes;
                const FoldSink out{!last ? FoldTo::kLds : (mailbox ? FoldTo::kMailbox : FoldTo::kPartials),
                                   a.part, a.mail, (int)blockIdx.x, run_ms, run_val, run_id};
                constexpr bool kQuad = Mp > 2 * WAVES;   // two rows per wavefront would take several rounds
                auto fold_with = [&](auto b32) {   // (bound from 16 groups up to k = 10, from 32 beyond)
                    constexpr bool B32 = decltype(b32)::value;
                    if (p == (int)blockIdx.x)
                        fold_pass<kZR, false, false, kQuad, B32>(z_all, kZR + kZPad, 1, 0, ids_lds, n_valid, a.k, 0, a.M,
                                                                 wave, WAVES, row_of, out, &s_select[wave]);
                    else
                        fold_pass<kZR, true, false, kQuad, B32>(z_all, kZR + kZPad, 1, 0, ids_lds, n_valid, a.k, 0, a.M,
                                                                wave, WAVES, row_of, out, &s_select[wave]);
                };
                if (a.k >= kBound32FromK) fold_with(std::true_type{});
                else fold_with(std::false_type{});
            }
        }
    }

    if (sink == (int)Sink::kLogits || sink == (int)Sink::kStreamOnly) return;

    // (every workgroup's last fold has written its lists and statistics out)
    stamp(3);
    const int gidx = blockIdx.x;
    const Partials part = a.part;   // a local copy keeps the argument block itself in registers
    if (mailbox) {
        // The results are self-validating records; the mergers (one per row of H while there
        // are enough workgroups) poll for them: nothing to count.  The mergers are the LAST
        // workgroups of the grid: workgroups start in order, so once the R <= 128 mergers are on
        // the machine everything else they wait for is running or done, and waits for nothing
        // itself: the wait ends as long as R workgroups fit on the device at once.
        if constexpr (WAVES >= 4) {
            const Mailbox mb = a.mail;
            const int R = G < a.M ? G : a.M;
            if (gidx < G - R) return;
            stamp(4);
            const unsigned spin = LEAN ? kMailSpinLimit : (a.spin_limit ? a.spin_limit : kMailSpinLimit);
            if (a.k >= kBound32FromK)
                merge_rows_mailbox<(WAVES >= 8 ? 8 : 4), true>(mb, part, a.ticket + 1, G, gidx - (G - R), R, a.M, a.k,
                                                               a.token_ids, a.logp, &s_merge, &s_select[0], nullptr, spin);
            else
                merge_rows_mailbox<(WAVES >= 8 ? 8 : 4), false>(mb, part, a.ticket + 1, G, gidx - (G - R), R, a.M, a.k,
                                                                a.token_ids, a.logp, &s_merge, &s_select[0], nullptr, spin);
            __syncthreads();
            stamp(5);
        }
        return;
    }
    if (sink == (int)Sink::kPartialsOnly) return;

    const int R = merger_count(G, a.M);
    const int r = arrive_and_wait(ar, (unsigned)__builtin_amdgcn_readfirstlane((int)turn), G, R, &s_slot,
                                  a.spin_limit ? a.spin_limit : kSpinLimit);
    if (r < 0) return;
    if (r & kWaitTimedOut)
        write_no_result((r & ~kWaitTimedOut) + R * wave, R * WAVES, a.M, a.k, a.token_ids, a.logp);
    else
        final_merge_all(part, G, r + R * wave, R * WAVES, a.M, a.k, a.token_ids, a.logp, &s_select[wave]);
}

constexpr int kLdsBudget = 160 * 1024;
constexpr int kStaticLdsReserve = 12 * 1024;   // room for the kernel's static LDS (selection scratch)

struct Build {
    int mt16, hch;
};
// m tiles -> H chunk length (in half-steps of 64 elements) of the build that serves them
constexpr Build kBuilds[] = {{1, 8}, {2, 8}, {3, 8}, {4, 4}, {6, 4}, {8, 2}};

// the smallest build that covers M rows and whose LDS (it grows with k) fits
const Build *build_for(int M, int k) {
    const int t = (M + 15) / 16;
    for (const Build &b : kBuilds)
        if (t <= b.mt16 && WideLds(b.mt16, b.hch, k).total <= kLdsBudget - kStaticLdsReserve) return &b;
    return nullptr;
}

typedef void (*WideKernel)(WideArgs);
constexpr int kWideWaves = 8;

// the build for `mt16` tiles of 16 rows of H
WideKernel select_kernel(int mt16, bool lean = false) {
    switch (mt16) {
        case 1: return lean ? wide_kernel<1, 1, kWideWaves, 4, 8, true> : wide_kernel<1, 1, kWideWaves, 4, 8>;
        case 2: return lean ? wide_kernel<2, 1, kWideWaves, 4, 8, true> : wide_kernel<2, 1, kWideWaves, 4, 8>;
        case 3: return lean ? wide_kernel<3, 1, kWideWaves, 4, 8, true> : wide_kernel<3, 1, kWideWaves, 4, 8>;
        case 4: return lean ? wide_kernel<4, 1, kWideWaves, 4, 4, true> : wide_kernel<4, 1, kWideWaves, 4, 4>;
        case 6: return lean ? wide_kernel<6, 1, kWideWaves, 4, 4, true> : wide_kernel<6, 1, kWideWaves, 4, 4>;
        case 8: return lean ? wide_kernel<8, 1, kWideWaves, 4, 2, true> : wide_kernel<8, 1, kWideWaves, 4, 2>;
    }
    return nullptr;
}

}  // namespace

// Raises the dynamic LDS limit of every build on the current device (per-device set-up).
fr_status prepare_wide_kernels() {
    for (const Build &b : kBuilds)
        for (int lean = 0; lean < 2; ++lean)
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(select_kernel(b.mt16, lean != 0)),
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    kLdsBudget - kStaticLdsReserve) != hipSuccess) {
                (void)hipGetLastError();
                return FR_ERR_HIP;
            }
    return FR_OK;
}

// Largest slab of H rows (multiple of 16, <= 128) whose per-row state fits LDS for this k.
int mfma_max_rows(int k) {
    int best = 0;
    for (const Build &b : kBuilds)
        if (WideLds(b.mt16, b.hch, k).total <= kLdsBudget - kStaticLdsReserve) best = b.mt16 * 16;
    return best;
}

fr_status launch_mfma(const HeadProblem &p, Sink sink, const fr_tuning *t, hipStream_t s,
                      int *grid_used) {
    const Build *b = build_for(p.M, p.k);
    if (!b) return FR_ERR_UNSUPPORTED;
    const int lds = WideLds(b->mt16, b->hch, p.k).total;
    if (lds > kLdsBudget - kStaticLdsReserve) return FR_ERR_UNSUPPORTED;
    const int cus = device_cu_count();
    if (cus <= 0) return FR_ERR_HIP;

    WideArgs a{};
    a.H = static_cast<const u32x4 *>(p.H);
    a.W = static_cast<const u32x4 *>(p.W);
    a.idx_map = p.idx_map;
    a.M = p.M;
    a.d8 = p.d / 8;
    a.V_rows = p.V_rows;
    a.k = p.k;
    a.steps = (a.d8 + kStep16 - 1) / kStep16;
    a.passes = (p.V_rows + kZR - 1) / kZR;
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
    if (grid_used) *grid_used = grid;

    // Single launch through the result mailbox: its records cover 128 rows of H, 16 list
    // positions and 256 workgroups, and the merge wants four wavefronts per workgroup.
    a.mailbox = sink == Sink::kFusedTopk && p.k <= kMailK && p.M <= kMailRows && grid <= 4 * kWave &&
                !(t && t->no_mailbox);

    // (not for the 128-row build: its lean instance measures 83.8 us against 75.2 us for the general one,
    // the 96-row build the other way round, 60.5 against 68.3 us; the smaller builds gain 0.1 to 0.9 us)
    const bool lean = sink == Sink::kFusedTopk && a.mailbox && !a.trace && a.spin_limit == 0u && b->mt16 != 8;
    const WideKernel kern = select_kernel(b->mt16, lean);
    if (!kern) return FR_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kWideWaves * kWave), lds, s, a);
    const fr_status st = hip_status(hipGetLastError());
    if (st != FR_OK) return st;
    if (sink == Sink::kPartialsOnly) return launch_merge(p, grid, s);
    return FR_OK;
}

}  // namespace frspec
