// Skinny kernel for a handful of H rows (M <= 16): the streaming product of Eq. 4 fused
// with the online log-softmax, the per-row top-k and the id remap.
//
// The product is bound by reading W once from HBM (2*d bytes per vocabulary row against
// 2*M*d flops), so the kernel is organised around the stream of W:
//   * one persistent workgroup per compute unit keeps all M rows of H in LDS;
//   * a wavefront owns a tile of 16 vocabulary rows.  Its 64 lanes form 4 row slots of
//     16 lanes; a slot walks along d, each lane loading 16 bytes (8 bf16) of W per step,
//     so one load instruction fetches 256 contiguous bytes from each of 4 rows (measured:
//     64-byte pieces per row, which would suit the matrix cores directly, stream 10%
//     slower);
//   * W goes straight from HBM to registers through a software pipeline of DEPTH steps,
//     every wavefront starting at a different column (see g_first);
//   * the products of a step run either on the matrix cores (default): the 16 x 128 slab
//     is transposed through a per-wavefront LDS buffer into MFMA operand order and
//     multiplied with 4 x v_mfma_f32_16x16x32_bf16 against H taken from LDS; or on the
//     vector ALUs: packed bf16 dot products with fp32 accumulation in a 4-row x MT
//     register tile, summed over the 16 lanes of a slot with DPP rotations at the end;
//   * the tile's logits go to LDS, never to HBM, and are folded into the workgroup's
//     running (max, sum-exp, top-k) state; on its last pass a workgroup writes that state
//     to the workspace, where a few of the workgroups merge the results of all of them
//     and write the outputs (for k <= 16 through self-validating mailbox records).
// For small vocabularies several wavefronts share a tile and split d between them
// (KS > 1) so that every compute unit still has enough loads in flight.
#include <type_traits>

#include "epilogue.hpp"
#include "internal.hpp"

namespace frspec {
namespace {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float dot2_bf16(unsigned w, unsigned h, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w),
                                           __builtin_bit_cast(bf16x2_t, h), acc, false);
}

// Streaming load of 16 bytes of W: global address space, wave-uniform base, per-lane
// unsigned 32-bit byte offset, non-temporal (W is read once and must not evict H).
typedef const __attribute__((address_space(1))) char *GlobalBytes;
typedef const __attribute__((address_space(1))) u32x4 *GlobalVec;
__device__ __forceinline__ u32x4 load_w(GlobalBytes base, unsigned byte_offset) {
    return __builtin_nontemporal_load(reinterpret_cast<GlobalVec>(base + byte_offset));
}

constexpr int kTileRows = 16;     // vocabulary rows per wavefront tile
constexpr int kRowsPerLane = 4;   // rows served by one lane
constexpr int kLanesAlongD = 16;  // lanes of a row slot (one DPP row)

struct SkinnyArgs {
    long long row_delta[16];   // byte offset of row m of H from `H` (the rows may sit in several blocks)
    const u32x4 *H;
    const u32x4 *W;
    const int *idx_map;
    int M, d8, V_rows, k;
    int tiles;            // 16-row tiles of W (tiled layout only)
    int skew;             // rows moved from every odd workgroup to its even neighbour (skewed build)
    int KS;               // wavefronts sharing one tile along d
    int steps;            // ceil(d8 / 16): steps of 128 elements along d
    int steps_per_split;  // ceil(steps / KS)
    int passes;           // ceil(V_rows / rows per pass)
    int sink;
    unsigned spin_limit;  // polls after which a wait for other workgroups is given up (0: the default)
    Partials part;
    Mailbox mail;
    StepArgs step;
    unsigned *ticket;
    int *token_ids;
    float *logp;
    float *z_out;
    int z_ld;
    long long *trace;     // optional [gridDim.x][8] phase timestamps (100 MHz clock)
};

__host__ __device__ constexpr int round_up(int x, int m) { return (x + m - 1) / m * m; }

// LDS carve-up, in bytes, identical on host and device.
constexpr int kStagePitch16 = kLanesAlongD + 1;   // 272-byte rows: conflict-free fragment reads

struct SkinnyLds {
    int h_off, stage_off, z_off, ids_off, ms_off, val_off, id_off, total;
    // `hrows` rows of H are staged: all MT (zero padded) for the dot-product variant, whose
    // register tiles are MT wide; only the M real ones for the matrix-core variant.
    __host__ __device__ SkinnyLds(int MT, int hrows, int waves, int steps, int k, bool mfma, bool tiled) {
        int o = 0;
        h_off = o;   o += hrows * (steps * kLanesAlongD + 1) * 16;
        stage_off = o; o += (mfma && !tiled) ? waves * kTileRows * kStagePitch16 * 16 : 0;
        z_off = o;   o += (waves * kTileRows * MT + waves * kTileRows) * 4;
        ids_off = o; o += waves * kTileRows * 4;
        ms_off = o;  o += MT * 2 * 4;
        val_off = o; o += MT * k * 4;
        id_off = o;  o += MT * k * 4;
        total = round_up(o, 16);
    }
};

/*
 * SKEW build (single pass per workgroup, row-major W, matrix cores): the eight compute dies do
 * not stream at the same rate (the odd-numbered ones are consistently ~9% slower), workgroups
 * are dealt to the dies in turn, and the kernel ends with the slowest die.  So every odd
 * workgroup hands `skew` of its rows to its even neighbour: a pair of workgroups shares
 * 2 * V_rows / G consecutive rows, the even one takes the first V_rows / G + skew.  A
 * workgroup's rows are cut into 16-row tiles as always; the even workgroup's surplus is a
 * ninth, short tile, streamed by a ninth wavefront that takes no part in the fold.  (A
 * wavefront's pace is set by the latency of its die's memory path, not by its own byte
 * count, so it does not matter which wavefront of a die carries fewer or more rows.)
 */
// B32: the bound of the folds and of the merge from 32 groups (the build for k = 11 .. 16).  A build of
// its own: both instances of that code in one kernel cost the k <= 10 calls 0.3 us.
// LEAN: the build for the plain fused call (single launch through the mailbox, no fused beam-search step,
// no phase trace, default wait limit): those choices are compile-time constants in it, which frees
// registers (212 against 220 vector registers, 162 against 217 scalar spills) and is worth 0.55 us per
// call at every size.  (Fixing the wavefronts per tile along d, or M and k, at compile time as well
// measured no further gain.)
// LEAN = 2: the same with the fused beam-search step (fr_draft_step).
template <int MT, int WAVES, int DEPTH, bool MFMA, bool TILED = false, bool SKEW = false, int HR = 16, bool B32 = false,
          int LEAN = 0>
__global__ __launch_bounds__(WAVES * kWave) void skinny_kernel(SkinnyArgs a) {
    static_assert(MFMA || !TILED, "the tiled layout is the matrix cores' operand order");
    static_assert(!SKEW || (MFMA && !TILED), "the skewed build is the default build plus one wavefront");
    constexpr int FOLD_WAVES = SKEW ? WAVES - 1 : WAVES;
    // The argument block spans several cache lines and the compiler fetches its fields where
    // they are first used, in half a dozen dependent rounds of scalar loads, each a trip to
    // memory (the block is new with every launch).  One load per line, all issued at once,
    // brings the lines into the scalar cache in a single trip; the rounds then hit.
    {
        static_assert(sizeof(SkinnyArgs) <= 6 * 64, "one load per 64-byte line of the argument block");
        typedef const __attribute__((address_space(4))) unsigned *ConstWords;
        ConstWords ka = (ConstWords)__builtin_amdgcn_kernarg_segment_ptr();
        unsigned w0, w1, w2, w3, w4, w5;
        asm volatile(
            "s_load_dword %0, %6, 0x0\n\t"
            "s_load_dword %1, %6, 0x40\n\t"
            "s_load_dword %2, %6, 0x80\n\t"
            "s_load_dword %3, %6, 0xc0\n\t"
            "s_load_dword %4, %6, 0x100\n\t"
            "s_load_dword %5, %6, 0x140\n\t"
            "s_waitcnt lgkmcnt(0)"
            : "=&s"(w0), "=&s"(w1), "=&s"(w2), "=&s"(w3), "=&s"(w4), "=&s"(w5)
            : "s"(ka)
            : "memory");
    }
    // The very first thing: H (see "Start of the stream" below for the order of the loads).
    // Thread t fetches 16-byte column t of every row of H (wave-uniform base + 32-bit lane
    // offset, like W), holds the pieces in registers and writes them to LDS further down.
    // rows of H this build requests (the skewed build's LDS holds at most 11, the vector-ALU
    // builds are compiled per number of rows anyway)
    constexpr int kHRowsMax = SKEW ? 12 : (MFMA ? HR : MT);
    const GlobalBytes Hb = (GlobalBytes)a.H;
    const unsigned hcol = (unsigned)min((int)threadIdx.x, a.d8 - 1) * 16u;   // clamped: always a valid address
    u32x4 hpre[kHRowsMax];
#pragma unroll
    for (int m = 0; m < kHRowsMax; ++m)
        hpre[m] = *reinterpret_cast<GlobalVec>(Hb + (m < a.M ? a.row_delta[m] : 0ll) + hcol);

    extern __shared__ u32x4 smem[];
    char *base = reinterpret_cast<char *>(smem);
    const int hrows = MFMA ? a.M : MT;
    const SkinnyLds L(MT, hrows, WAVES, a.steps, a.k, MFMA, TILED);
    u32x4 *H_lds = reinterpret_cast<u32x4 *>(base + L.h_off);
    u32x4 *stage_lds = reinterpret_cast<u32x4 *>(base + L.stage_off);
    float *z_lds = reinterpret_cast<float *>(base + L.z_off);
    int *ids_lds = reinterpret_cast<int *>(base + L.ids_off);
    float *run_ms = reinterpret_cast<float *>(base + L.ms_off);
    float *run_val = reinterpret_cast<float *>(base + L.val_off);
    int *run_id = reinterpret_cast<int *>(base + L.id_off);
    __shared__ int s_slot;
    __shared__ SelectScratch s_select[WAVES];
    __shared__ MergeScratch s_merge;
    const Partials part = a.part;   // a local copy keeps the argument block itself in registers

    constexpr int ZR_MAX = FOLD_WAVES * kTileRows;   // local rows that the fold's lanes cover
    // four rows of H per folding wavefront only where two would take a second round
    constexpr bool kQuadFold = !SKEW && MT > 2 * FOLD_WAVES;
    // the default build also carries the fold for passes of 64 rows (two wavefronts per tile)
    constexpr bool kHalfFold = MFMA && !TILED && !SKEW && WAVES == 8 && !kQuadFold;
    constexpr int kStep16 = kLanesAlongD;        // 16-byte chunks per row per step
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);   // wave-uniform by construction
    const int lk = lane & (kLanesAlongD - 1);
    const int rs = lane / kLanesAlongD;
    // 16-byte chunks per row of H in LDS: the row padded to whole steps, plus one chunk so
    // that the rows start 4 banks apart (the matrix-core fragments are read down a column of
    // H: lanes l % 16 = row; without the skew all rows of a column share their banks)
    const int hcols = a.steps * kStep16;
    const int hpitch = hcols + 1;
    const int KS = a.KS;
    const int ZR = (WAVES / KS) * kTileRows;     // vocabulary rows per pass
    const int tile_in_pass = wave / KS;
    const int ks = wave - tile_in_pass * KS;
    const int G = gridDim.x;
    // SKEW: this workgroup's own row range
    int blk_row0 = 0, blk_rows = 0;
    if constexpr (SKEW) {
        const int B = a.V_rows / G, odd = (int)blockIdx.x & 1;
        blk_row0 = ((int)blockIdx.x >> 1) * 2 * B + (odd ? B + a.skew : 0);
        blk_rows = odd ? B - a.skew : B + a.skew;
    }
    const bool has_tile = !SKEW || tile_in_pass * kTileRows < blk_rows;   // wave-uniform
    auto stamp = [&](int slot) {
        if constexpr (LEAN == 0)
            if (a.trace && tid == 0) a.trace[blockIdx.x * 8 + slot] = (long long)__builtin_amdgcn_s_memrealtime();
    };
    const int sink = LEAN != 0 ? (int)Sink::kFusedTopk : a.sink;
    stamp(0);
    // which arrival counter this call uses: asked for now, needed at the very end
    const Arrival ar(a.ticket);
    // single launch, k <= 16, at most 256 workgroups: results travel as mailbox records
    const bool mailbox = LEAN != 0 || (sink == (int)Sink::kFusedTopk && a.k <= kSmallKMax && G <= 4 * kWave);
    const unsigned turn = (sink == (int)Sink::kFusedTopk && !mailbox) ? ar.turn() : 0u;

    // Step range of this wavefront along d, split into a pipelined part (whole groups of
    // DEPTH full steps, no bounds handling at all) and leftovers (at most DEPTH - 1 steps,
    // plus the ragged last step when d is not a multiple of 128).
    const int s_begin = ks * a.steps_per_split;
    const int s_end = has_tile ? min(a.steps, s_begin + a.steps_per_split) : s_begin;
    const int full_end = min(s_end, a.d8 / kStep16);
    const int groups = full_end > s_begin ? (full_end - s_begin) / DEPTH : 0;
    const int s_pipe_end = s_begin + groups * DEPTH;
    // Every wavefront walks its groups of steps cyclically from a different starting group.
    // All wavefronts advance at about the same pace; if they also started at the same
    // column, the whole device would at any moment read addresses that agree modulo the
    // row pitch and load the memory channels unevenly.  The sum over d does not depend
    // on the order of the steps.
    const int g_first = groups > 0 ? (int)((wave + blockIdx.x) % (unsigned)groups) : 0;

    // W is addressed as a wave-uniform base plus a per-lane 32-bit byte offset (the host
    // guarantees the matrix is smaller than 4 GiB): offset of (row, chunk lk of step
    // s_begin) for the 4 rows of this lane.
    // Tiled layout: a 16-row tile of W is one contiguous run of 1 KiB blocks, one per 32
    // elements of d, each block already in the lane order of the matrix cores' A operand
    // (lane l: row l % 16, elements 8 * (l / 16) .. + 7 of the block).  The 4 loads of a step
    // are then 4 consecutive blocks: 4 KiB of contiguous memory per wavefront and step.
    const GlobalBytes Wb = (GlobalBytes)a.W;
    auto row_offsets = [&](int pass, unsigned (&wo)[kRowsPerLane]) {
        if constexpr (TILED) {
            const int tile = min(pass * (WAVES / KS) + tile_in_pass, a.tiles - 1);
#pragma unroll
            for (int r = 0; r < kRowsPerLane; ++r)
                wo[r] = (unsigned)tile * ((unsigned)a.d8 * (kTileRows * 16u)) +
                        (unsigned)(s_begin * kRowsPerLane + r) * 1024u + (unsigned)lane * 16u;
        } else {
            const int tile_row0 = (SKEW ? blk_row0 : pass * ZR) + tile_in_pass * kTileRows + rs * kRowsPerLane;
            const int last_row = SKEW ? blk_row0 + blk_rows - 1 : a.V_rows - 1;
#pragma unroll
            for (int r = 0; r < kRowsPerLane; ++r) {
                const int row = min(tile_row0 + r, last_row);
                wo[r] = ((unsigned)row * (unsigned)a.d8 + (unsigned)(s_begin * kStep16 + lk)) * 16u;
            }
        }
    };
    constexpr unsigned kStepBytes = TILED ? kRowsPerLane * 1024u : kStep16 * 16;
    constexpr unsigned kGroupBytes = DEPTH * kStepBytes;

    // Start of the stream.  Loads return in issue order, so the (small, L2-resident) H is
    // requested first and W right behind it: H can then be written to LDS while the first
    // W stages are still on their way, and the first products start as soon as W arrives.
    // Requested the other way round, H would queue behind 16 W loads per lane.
    // Thread t fetches 16-byte column t of every row of H (wave-uniform base + 32-bit lane
    // offset, like W), holds the pieces in registers and writes them to LDS further down.
    // Every load between here and the first products is issued UNCONDITIONALLY (rows past M
    // re-read row 0, rows past the pass are clamped): a load under a branch leaves the
    // compiler without the number of loads outstanding behind it, and it then waits for
    // all of them (vmcnt(0)), i.e. for the whole first batch of W, before H goes to LDS.
    constexpr int NT = WAVES * kWave;
    // token id of local row `tid` of a pass (asked for before the loads of that pass's W)
    const int *idx_or_null = a.idx_map;
    auto request_id = [&](int pass) {
        const int row = min((SKEW ? blk_row0 : pass * ZR) + (tid < ZR_MAX + 16 ? tid : 0), a.V_rows - 1);
        return idx_or_null ? __builtin_nontemporal_load(idx_or_null + row) : row;
    };
    int id_next = request_id((int)blockIdx.x < a.passes ? (int)blockIdx.x : 0);
    u32x4 wb[DEPTH][kRowsPerLane];
    unsigned wo[kRowsPerLane];
    const int first_pass = (int)blockIdx.x;
    int p = first_pass;   // (the host launches no more workgroups than there are passes)
    // The first DEPTH stages of W, also unconditionally: when the row has fewer steps than
    // the pipeline is deep the surplus loads are clamped into the matrix and never used.
    {
        const unsigned w_last = ((unsigned)(TILED ? a.tiles * kTileRows : a.V_rows) * (unsigned)a.d8 - 1u) * 16u;
        row_offsets(p, wo);
#pragma unroll
        for (int u = 0; u < DEPTH; ++u)
#pragma unroll
            for (int r = 0; r < kRowsPerLane; ++r)
                wb[u][r] = load_w(Wb, min(wo[r] + g_first * kGroupBytes + u * kStepBytes, w_last));
    }
    // stage H (zero padded to whole steps, and to MT rows where the tiles need it).  Every
    // piece of H is waited for here, in issue order and in straight-line code, whether it is
    // written or not: the count of loads behind it (those of W) is then exact, and no
    // register of an unwritten row is still awaited when it is reused.
#pragma unroll
    for (int m = 0; m < kHRowsMax; ++m) {
        asm volatile("" : "+v"(hpre[m]));
        if (m < hrows && tid < hcols)
            H_lds[m * hpitch + tid] = (tid < a.d8 && m < a.M) ? hpre[m] : zero_u32x4();
    }
    asm volatile("" : "+v"(id_next));   // (requested before H: here by now, and known to be)
    for (int c = tid + NT; c < hcols; c += NT) {   // columns past the first NT: not held in registers
#pragma unroll
        for (int m = 0; m < 16; ++m)
            if (m < hrows) {
                u32x4 v = zero_u32x4();
                if (m < a.M && c < a.d8) v = *reinterpret_cast<GlobalVec>(Hb + a.row_delta[m] + (unsigned)c * 16u);
                H_lds[m * hpitch + c] = v;
            }
    }
    // (the running state needs no reset: a workgroup's first pass overwrites all of it)
    __syncthreads();
    stamp(1);

    for (; p < a.passes && (!SKEW || p == first_pass); p += G) {
        const int pass_row0 = SKEW ? blk_row0 : p * ZR;
        const int n_valid = SKEW ? blk_rows : min(ZR, a.V_rows - pass_row0);
        if (tid < n_valid) ids_lds[tid] = id_next;

        // Accumulators.  Vector-ALU variant: the lane's share (16 bytes per step) of 4 rows x
        // MT rows of H.  Matrix-core variant: one 16 x 16 tile, lane (j, g) = column m = j,
        // rows 4g..4g+3.
        float acc[MFMA ? 1 : kRowsPerLane][MFMA ? 1 : MT];
        f32x4_t accm = {0.f, 0.f, 0.f, 0.f};
        if constexpr (!MFMA) {
#pragma unroll
            for (int r = 0; r < kRowsPerLane; ++r)
#pragma unroll
                for (int m = 0; m < MT; ++m) acc[r][m] = 0.0f;
        }

        // One step: 16 bytes of each of the lane's 4 rows (together the wavefront holds
        // 16 rows x 128 elements) against the M rows of H.  `c0` is the index of the step's
        // first 16-byte chunk along d.
        auto compute = [&](const u32x4 (&w)[kRowsPerLane], int c0) {
            if constexpr (MFMA && TILED) {
                // the 4 loads of the step are the A operands of its 4 products as they are
                const int hrow = lk < a.M ? lk : a.M - 1;   // columns >= M are never read back
                bf16x8_t bf[4];
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
                    bf[kk] = __builtin_bit_cast(bf16x8_t, H_lds[hrow * hpitch + c0 + kk * 4 + rs]);
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
                    accm = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, w[kk]), bf[kk],
                                                                   accm, 0, 0, 0);
            } else if constexpr (MFMA) {
                // Transpose through LDS into MFMA operand order: the loads deliver
                // (row slot, 16-byte chunk) per lane, the A operand wants (row, 8-element
                // group).  Only this wavefront touches its staging rows and LDS executes a
                // wavefront's operations in order, so no barrier is needed.
                u32x4 *st = stage_lds + wave * (kTileRows * kStagePitch16);
#pragma unroll
                for (int r = 0; r < kRowsPerLane; ++r)
                    st[(rs * kRowsPerLane + r) * kStagePitch16 + lk] = w[r];
                const int j = lk, g = rs;   // operand coordinates of this lane
                const int hrow = j < a.M ? j : a.M - 1;   // columns >= M are never read back
                bf16x8_t af[4], bf[4];
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    af[kk] = __builtin_bit_cast(bf16x8_t, st[j * kStagePitch16 + kk * 4 + g]);
                    bf[kk] = __builtin_bit_cast(bf16x8_t, H_lds[hrow * hpitch + c0 + kk * 4 + g]);
                }
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
                    accm = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[kk], bf[kk], accm, 0, 0, 0);
            } else {
                const u32x4 *hp = H_lds + c0 + lk;
                u32x4 h[MT];
#pragma unroll
                for (int m = 0; m < MT; ++m) h[m] = hp[m * hpitch];
#pragma unroll
                for (int r = 0; r < kRowsPerLane; ++r)
#pragma unroll
                    for (int m = 0; m < MT; ++m) {
                        float t = acc[r][m];
                        t = dot2_bf16(w[r].x, h[m].x, t);
                        t = dot2_bf16(w[r].y, h[m].y, t);
                        t = dot2_bf16(w[r].z, h[m].z, t);
                        t = dot2_bf16(w[r].w, h[m].w, t);
                        acc[r][m] = t;
                    }
            }
        };

        if (groups > 0) {
            const int c_begin = s_begin * kStep16;
            int grp = g_first;
            // Steady state: consume stage u, then refill it with the same stage of the next
            // group.  The scheduling barriers keep the refill where it is written: left
            // alone, the scheduler sinks all loads to the end of the body (shorter live
            // ranges) and the wavefront then waits for every load it has just issued.
            for (int it = 0; it < groups - 1; ++it) {
                const int nxt = (grp + 1 == groups) ? 0 : grp + 1;
                const int cg = c_begin + grp * (DEPTH * kStep16);
                const unsigned nofs = (unsigned)nxt * kGroupBytes;
#pragma unroll
                for (int u = 0; u < DEPTH; ++u) {
                    compute(wb[u], cg + u * kStep16);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int r = 0; r < kRowsPerLane; ++r)
                        wb[u][r] = load_w(Wb, wo[r] + nofs + u * kStepBytes);
                    __builtin_amdgcn_sched_barrier(0);
                }
                grp = nxt;
            }
            // drain; the stages freed here start on the next pass of this workgroup
            const int cg = c_begin + grp * (DEPTH * kStep16);
            const bool has_next = !SKEW && p + G < a.passes;   // (the skewed build has one pass)
            if (has_next) {
                id_next = request_id(p + G);
                row_offsets(p + G, wo);
                const unsigned nofs = (unsigned)g_first * kGroupBytes;
#pragma unroll
                for (int u = 0; u < DEPTH; ++u) {
                    compute(wb[u], cg + u * kStep16);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int r = 0; r < kRowsPerLane; ++r)
                        wb[u][r] = load_w(Wb, wo[r] + nofs + u * kStepBytes);
                    __builtin_amdgcn_sched_barrier(0);
                }
                asm volatile("" : "+v"(id_next));   // wait for it here, where the loads behind it are counted
            } else {
#pragma unroll
                for (int u = 0; u < DEPTH; ++u) compute(wb[u], cg + u * kStep16);
            }
        }
        if (s_pipe_end < s_end) {
            // Leftover steps, not pipelined.  A chunk index past the end of the row is
            // clamped: the bytes loaded are valid finite weights and the matching H chunk
            // in LDS is zero.
            unsigned wr[kRowsPerLane];
            row_offsets(p, wr);
            for (int s = s_pipe_end; s < s_end; ++s) {
                // byte offset of step s relative to step s_begin (tiled: whole steps only, the
                // host admits the layout only for d a multiple of 128)
                const unsigned c = TILED ? (unsigned)(s - s_begin) * kStepBytes
                                         : (unsigned)(min(s * kStep16 + lk, a.d8 - 1) - (s_begin * kStep16 + lk)) * 16u;
                u32x4 w[kRowsPerLane];
#pragma unroll
                for (int r = 0; r < kRowsPerLane; ++r) w[r] = load_w(Wb, wr[r] + c);
                compute(w, s * kStep16);
            }
        }

        if constexpr (MFMA) {
            // lane (j, g) owns rows 4g..4g+3 of column m = j
            if (lk < a.M) {
                float *dst = z_lds + (ks * MT + lk) * ZR + tile_in_pass * kTileRows + 4 * rs;
                *reinterpret_cast<f32x4_t *>(dst) = accm;
            }
        } else {
            // sum the 16 lanes of each row slot; lane 0 of the slot stores the tile's logits
#pragma unroll
            for (int r = 0; r < kRowsPerLane; ++r)
#pragma unroll
                for (int m = 0; m < MT; ++m) acc[r][m] = row16_sum(acc[r][m]);
            if (lk == 0) {
                const int rl = tile_in_pass * kTileRows + rs * kRowsPerLane;
#pragma unroll
                for (int m = 0; m < MT; ++m)
#pragma unroll
                    for (int r = 0; r < kRowsPerLane; ++r)
                        z_lds[(ks * MT + m) * ZR + rl + r] = acc[r][m];
            }
        }
        __syncthreads();
        stamp(2);

        // ---- consume the pass ----
        if (sink == (int)Sink::kLogits) {
            for (int i = tid; i < a.M * ZR; i += WAVES * kWave) {
                const int m = i / ZR, r = i - m * ZR;
                if (r < n_valid) {
                    float z = 0.0f;
                    for (int s = 0; s < KS; ++s) z += z_lds[(s * MT + m) * ZR + r];
                    a.z_out[(size_t)m * a.z_ld + pass_row0 + r] = z;
                }
            }
        } else if (sink != (int)Sink::kStreamOnly) {
            auto row_of = [&](int m) {
                return FoldRow{z_lds + m * ZR, run_ms + 2 * m, run_val + m * a.k, run_id + m * a.k};
            };
            // the last pass of the workgroup writes its result out instead of keeping it
            const bool last = p + G >= a.passes;
            const FoldSink out{!last ? FoldTo::kLds : (mailbox ? FoldTo::kMailbox : FoldTo::kPartials),
                               part, a.mail, (int)blockIdx.x, run_ms, run_val, run_id};
            bool folded = false;
            if constexpr (kHalfFold) {
                // two wavefronts per tile: a pass is 64 rows, and a fold laid out for 64 rows has half the
                // logits per lane of the one laid out for 128 (of which half the lanes would hold none)
                if (KS == 2) {
                    if (p == first_pass)
                        fold_pass<ZR_MAX / 2, false, false, false, B32>(z_lds, ZR, KS, MT * ZR, ids_lds, n_valid, a.k, 0, a.M,
                                                                   wave, FOLD_WAVES, row_of, out, &s_select[wave]);
                    else
                        fold_pass<ZR_MAX / 2, true, false, false, B32>(z_lds, ZR, KS, MT * ZR, ids_lds, n_valid, a.k, 0, a.M,
                                                                  wave, FOLD_WAVES, row_of, out, &s_select[wave]);
                    folded = true;
                } else if (KS == 4) {
                    // four wavefronts per tile: 32 rows per pass, folded in the layout for 64 (two logits per
                    // lane, half the lanes empty) instead of the one for 128: -0.6 us at 8192 rows
                    if (p == first_pass)
                        fold_pass<ZR_MAX / 2, false, false, false, B32>(z_lds, ZR, KS, MT * ZR, ids_lds, n_valid, a.k, 0, a.M,
                                                                        wave, FOLD_WAVES, row_of, out, &s_select[wave]);
                    else
                        fold_pass<ZR_MAX / 2, true, false, false, B32>(z_lds, ZR, KS, MT * ZR, ids_lds, n_valid, a.k, 0, a.M,
                                                                       wave, FOLD_WAVES, row_of, out, &s_select[wave]);
                    folded = true;
                }
            }
            if (folded || (SKEW && wave >= FOLD_WAVES)) {
                // (done; or the ninth wavefront, which only streams)
            } else if (p == first_pass) {
                fold_pass<ZR_MAX, false, SKEW, kQuadFold, B32>(z_lds, ZR, KS, MT * ZR, ids_lds, n_valid, a.k, 0, a.M, wave,
                                               FOLD_WAVES, row_of, out, &s_select[wave]);
            } else {
                fold_pass<ZR_MAX, true, SKEW, kQuadFold, B32>(z_lds, ZR, KS, MT * ZR, ids_lds, n_valid, a.k, 0, a.M, wave,
                                              FOLD_WAVES, row_of, out, &s_select[wave]);
            }
        }
        if (p + G < a.passes) {
            // (with a pipelined stream the ids of the next pass were requested together with its W)
            if (groups == 0 && !SKEW) {
                id_next = request_id(p + G);
                asm volatile("" : "+v"(id_next));
            }
            __syncthreads();
        }
    }

    if (sink == (int)Sink::kLogits || sink == (int)Sink::kStreamOnly) return;
    stamp(3);
    if (sink == (int)Sink::kPartialsOnly) return;

    // ---- some of the workgroups merge all partials (single launch) ----
    const int R = merger_count(G, a.M);
    if (mailbox) {
        // Mailbox records announce themselves: nothing to wait for, nothing to count.  The
        // mergers are fixed, every 8th workgroup while there are enough (workgroups are
        // dealt to the 8 dies in turn, so these share the first die), counted from the END of
        // the grid: workgroups start in order, so once the R <= 16 mergers are on the machine
        // everything else they wait for is running or done, and waits for nothing itself.
        // They start polling for the others' records as soon as their own are out.
        const int spread = 8 * (R - 1) < G ? 8 : 1;
        const int b = (int)blockIdx.x;
        const int top = (G - 1) / spread * spread;   // the last workgroup that can be a merger
        const int r = (top - b) / spread;
        if (b > top || b % spread != 0 || r >= R) return;
        stamp(4);
        const unsigned spin = LEAN != 0 ? kMailSpinLimit : (a.spin_limit ? a.spin_limit : kMailSpinLimit);
        unsigned long long *const step_rec = LEAN == 1 ? nullptr : a.step.rec;
        merge_rows_mailbox<(WAVES >= 8 ? 8 : 4), B32>(a.mail, part, a.ticket + 1, G, r, R, a.M, a.k, a.token_ids, a.logp, &s_merge,
                                                      &s_select[0], step_rec, spin);
        // the first merger also runs the beam-search expansion of the step, if one was asked for
        if (step_rec && r == 0 && wave == 0)
            expand_step_fused(a.step, a.M, a.k, reinterpret_cast<unsigned long long *>(s_select), a.ticket + 1, spin);
    } else {
        const int r = arrive_and_wait(ar, (unsigned)__builtin_amdgcn_readfirstlane((int)turn), G, R, &s_slot,
                                      a.spin_limit ? a.spin_limit : kSpinLimit);
        stamp(4);
        if (r < 0) return;
        if (r & kWaitTimedOut)
            write_no_result((r & ~kWaitTimedOut) + R * wave, R * WAVES, a.M, a.k, a.token_ids, a.logp);
        else
            final_merge_general(part, G, r + R * wave, R * WAVES, a.M, a.k, a.token_ids, a.logp, &s_select[wave]);
    }
    __syncthreads();
    stamp(5);
}

// ---------------------------------------------------------------- host side ---

constexpr int kLdsBudget = 160 * 1024;   // bytes of LDS per workgroup on gfx950
constexpr int kStaticLdsReserve = 16 * 1024;   // room for the kernel's static LDS (selection scratch)

constexpr int kMTBuckets[] = {1, 2, 4, 6, 8, 10, 12, 16};

int bucket_for(int M) {
    for (int b : kMTBuckets)
        if (M <= b) return b;
    return -1;
}

typedef void (*SkinnyKernel)(SkinnyArgs);

// The dot-product variant is compiled per width of its register tile.
template <int WAVES, int DEPTH>
SkinnyKernel dot_kernel(int MT) {
    switch (MT) {
        case 1: return skinny_kernel<1, WAVES, DEPTH, false>;
        case 2: return skinny_kernel<2, WAVES, DEPTH, false>;
        case 4: return skinny_kernel<4, WAVES, DEPTH, false>;
        case 6: return skinny_kernel<6, WAVES, DEPTH, false>;
        case 8: return skinny_kernel<8, WAVES, DEPTH, false>;
        case 10: return skinny_kernel<10, WAVES, DEPTH, false>;
        case 12: return skinny_kernel<12, WAVES, DEPTH, false>;
        case 16: return skinny_kernel<16, WAVES, DEPTH, false>;
    }
    return nullptr;
}

struct Variant {
    int waves, depth;
    bool mfma;
    bool tiled;
};
// Build variants: waves per workgroup, pipeline depth, and whether the products run on
// the matrix cores or on the packed-bf16 dot instruction of the vector ALUs.  The matrix
// cores win at every M on this chip (the dot instruction issues at about 70% of the plain
// FMA rate and its work competes with the address arithmetic of the stream), so they are
// the default; the vector-ALU build is kept as the measured alternative.
//   0  matrix cores, 8 waves, 4 stages        (default)
//   1  matrix cores, 4 waves, 8 stages        (default when H is too large for 8 staging rows)
//   2  matrix cores, 8 waves, 3 stages
//   3  matrix cores, 8 waves, 6 stages
//   4  vector ALUs, 8 waves, 4 stages (2 stages when more than 10 rows of H: registers)
//   5  vector ALUs, 8 waves, 3 stages
//   6  matrix cores, tiled W, 8 waves, 4 stages   (default for the tiled layout)
//   7  matrix cores, tiled W, 8 waves, 6 stages
//   8  matrix cores, tiled W, 8 waves, 8 stages
//   9  matrix cores, 8 + 1 waves, 4 stages, rows skewed between neighbouring workgroups
//      (chosen automatically when every workgroup has exactly one pass)
constexpr Variant kVariants[] = {{8, 4, true, false}, {4, 8, true, false}, {8, 3, true, false},
                                 {8, 6, true, false}, {8, 4, false, false}, {8, 3, false, false},
                                 {8, 4, true, true}, {8, 6, true, true}, {8, 8, true, true},
                                 {9, 4, true, false}};
constexpr int kSkewVariant = 9;
constexpr int kSkewDefaultRows = 4;
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);
constexpr int kMfmaTile = 16;   // the matrix-core variant is compiled once, for up to 16 rows

// The kernel build behind a variant, for M rows of H (MT: width of the vector-ALU tile).
template <bool B32, int LEAN>
SkinnyKernel lean_kernel(int M) {
    if (M <= 2) return skinny_kernel<16, 8, 4, true, false, false, 2, B32, LEAN>;
    if (M <= 4) return skinny_kernel<16, 8, 4, true, false, false, 4, B32, LEAN>;
    if (M <= 8) return skinny_kernel<16, 8, 4, true, false, false, 8, B32, LEAN>;
    if (M <= 10) return skinny_kernel<16, 8, 4, true, false, false, 10, B32, LEAN>;
    if (M <= 12) return skinny_kernel<16, 8, 4, true, false, false, 12, B32, LEAN>;
    return skinny_kernel<16, 8, 4, true, false, false, 16, B32, LEAN>;
}

// lean: 0 = the general build, 1 = the build for the plain fused call, 2 = for the call with the fused
// beam-search step (k <= 10 only)
SkinnyKernel select_kernel(int variant, int M, int MT, bool b32 = false, int lean = 0) {
    if (variant == 0 && lean == 1) return b32 ? lean_kernel<true, 1>(M) : lean_kernel<false, 1>(M);
    if (variant == 0 && lean == 2 && !b32) return lean_kernel<false, 2>(M);
    if (variant == 0 && b32) {   // the default build for k = 11 .. 16
        if (M <= 2) return skinny_kernel<kMfmaTile, 8, 4, true, false, false, 2, true>;
        if (M <= 4) return skinny_kernel<kMfmaTile, 8, 4, true, false, false, 4, true>;
        if (M <= 8) return skinny_kernel<kMfmaTile, 8, 4, true, false, false, 8, true>;
        if (M <= 10) return skinny_kernel<kMfmaTile, 8, 4, true, false, false, 10, true>;
        if (M <= 12) return skinny_kernel<kMfmaTile, 8, 4, true, false, false, 12, true>;
        return skinny_kernel<kMfmaTile, 8, 4, true, false, false, 16, true>;
    }
    switch (variant) {
        case 0:
            // the default build exists once per number of H rows it requests at its start
            if (M <= 2) return skinny_kernel<kMfmaTile, 8, 4, true, false, false, 2>;
            if (M <= 4) return skinny_kernel<kMfmaTile, 8, 4, true, false, false, 4>;
            if (M <= 8) return skinny_kernel<kMfmaTile, 8, 4, true, false, false, 8>;
            if (M <= 10) return skinny_kernel<kMfmaTile, 8, 4, true, false, false, 10>;
            if (M <= 12) return skinny_kernel<kMfmaTile, 8, 4, true, false, false, 12>;
            return skinny_kernel<kMfmaTile, 8, 4, true>;
        case 1: return skinny_kernel<kMfmaTile, 4, 8, true>;
        case 2: return skinny_kernel<kMfmaTile, 8, 3, true>;
        case 3: return skinny_kernel<kMfmaTile, 8, 6, true>;
        case 4: return MT > 10 ? dot_kernel<8, 2>(MT) : dot_kernel<8, 4>(MT);
        case 5: return dot_kernel<8, 3>(MT);
        case 6: return skinny_kernel<kMfmaTile, 8, 4, true, true>;
        case 7: return skinny_kernel<kMfmaTile, 8, 6, true, true>;
        case 8: return skinny_kernel<kMfmaTile, 8, 8, true, true>;
        case 9: return skinny_kernel<kMfmaTile, 9, 4, true, false, true>;
    }
    return nullptr;
}

int lds_bytes(int M, int d, int k, int variant) {
    const int steps = (d / 8 + kLanesAlongD - 1) / kLanesAlongD;
    const Variant &v = kVariants[variant];
    const int MT = v.mfma ? kMfmaTile : bucket_for(M);
    return SkinnyLds(MT, v.mfma ? M : MT, v.waves, steps, k, v.mfma, v.tiled).total;
}

bool variant_fits(int M, int d, int k, int variant) {
    return lds_bytes(M, d, k, variant) <= kLdsBudget - kStaticLdsReserve;
}

// -1 if no build of the skinny kernel can hold this problem's H in LDS
int default_variant(int M, int d, int k, bool vector_alu, bool tiled) {
    if (tiled) return variant_fits(M, d, k, 6) ? 6 : -1;
    if (vector_alu) return variant_fits(M, d, k, 4) ? 4 : -1;
    if (variant_fits(M, d, k, 0)) return 0;
    if (variant_fits(M, d, k, 1)) return 1;
    return -1;
}

}  // namespace

// Raises the dynamic LDS limit of every build on the current device (part of the per-device
// set-up; a launch never changes a function attribute).
fr_status prepare_skinny_kernels() {
    for (int variant = 0; variant < kNumVariants; ++variant)
        for (int M = 1; M <= kSkinnyMaxM; ++M) {
            for (int build = 0; build < 6; ++build) {   // 16 / 32 groups of the bound x general / lean / lean with step
                const SkinnyKernel kern = select_kernel(variant, M, kVariants[variant].mfma ? kMfmaTile : bucket_for(M),
                                                        (build & 1) != 0, build >> 1);
                if (!kern) return FR_ERR_HIP;
                if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                        kLdsBudget - kStaticLdsReserve) != hipSuccess) {
                    (void)hipGetLastError();
                    return FR_ERR_HIP;
                }
            }
        }
    return FR_OK;
}

bool skinny_fits(int M, int d, int k) {
    return M <= kSkinnyMaxM && default_variant(M, d, k, false, false) >= 0;
}

bool skinny_fits_eight_waves(int M, int d, int k) { return M <= kSkinnyMaxM && variant_fits(M, d, k, 0); }

fr_status launch_skinny(const HeadProblem &p, Sink sink, const fr_tuning *t, hipStream_t s) {
    if (p.M > kSkinnyMaxM) return FR_ERR_UNSUPPORTED;
    const bool vector_alu = t && t->path == 1;
    if (p.tiled && (vector_alu || p.d % 128 != 0)) return FR_ERR_UNSUPPORTED;
    int variant = default_variant(p.M, p.d, p.k, vector_alu, p.tiled);
    if (t && t->variant > 0) {
        if (t->variant > kNumVariants) return FR_ERR_INVALID_ARG;
        variant = t->variant - 1;
        if (kVariants[variant].tiled != p.tiled) return FR_ERR_INVALID_ARG;   // a build reads one layout
        if (!variant_fits(p.M, p.d, p.k, variant)) return FR_ERR_UNSUPPORTED;
    }
    if (variant < 0) return FR_ERR_UNSUPPORTED;
    const bool mfma = kVariants[variant].mfma;
    const int MT = mfma ? kMfmaTile : bucket_for(p.M);
    const int waves = kVariants[variant].waves;
    const int cus = device_cu_count();
    if (cus <= 0) return FR_ERR_HIP;

    SkinnyArgs a{};
    a.H = static_cast<const u32x4 *>(p.H);
    for (int m = 0; m < 16; ++m)
        a.row_delta[m] = p.scattered_rows ? p.row_delta[m] : static_cast<long long>(m) * p.d * 2;
    a.W = static_cast<const u32x4 *>(p.W);
    a.idx_map = p.idx_map;
    a.M = p.M;
    a.d8 = p.d / 8;
    a.V_rows = p.V_rows;
    a.k = p.k;
    a.tiles = (p.V_rows + kTileRows - 1) / kTileRows;
    a.steps = (a.d8 + kLanesAlongD - 1) / kLanesAlongD;

    // Wavefronts that share a tile and split d between them (see the rule below).
    int KS = 1;
    if (variant == kSkewVariant) {
        if (t && t->ksplit > 1) return FR_ERR_INVALID_ARG;
    } else if (t && t->ksplit > 0) {
        KS = t->ksplit;
        if (KS > waves || (KS & (KS - 1)) != 0) return FR_ERR_INVALID_ARG;
    } else {
        auto passes_for = [&](int ks) {
            const int zr = (waves / ks) * kTileRows;
            return (p.V_rows + zr - 1) / zr;
        };
        // Measured rule (d = 4096, 256 compute units): while the passes do not fill three quarters of
        // the compute units, halve them; once there is a pass for every compute unit, two half-size
        // passes per workgroup stream faster than one (-0.5 us at 32768 rows, -1.5 us at 65536 and
        // 128256, -6 us at 49152, where one-tile passes leave half the device idle in a second round).
        if (passes_for(1) >= cus) {
            if (2 <= waves && 4 <= a.steps) KS = 2;
        } else {
            while (KS < waves && KS * 2 <= a.steps && 4 * passes_for(KS) < 3 * cus) KS *= 2;
        }
    }
    a.KS = KS;
    a.steps_per_split = (a.steps + KS - 1) / KS;
    // (a forced skewed build counts passes like the default build it replaces: 8 tiles each)
    const int ZR = ((variant == kSkewVariant ? 8 : waves) / KS) * kTileRows;
    a.passes = (p.V_rows + ZR - 1) / ZR;
    a.sink = (int)sink;
    a.part.ms = p.ws.part_ms;
    a.part.val = p.ws.part_val;
    a.part.id = p.ws.part_id;
    a.ticket = p.ws.ticket;
    a.mail.rec = p.ws.mail_rec;
    a.mail.st = p.ws.mail_st;
    if (p.step) {
        // the expansion rides on the mailbox merge: k <= 16, one launch, at most 256 workgroups
        if (sink != Sink::kFusedTopk || p.k > kSmallKMax || cus > 4 * kWave || p.M * p.k > kStepRows * kMailK)
            return FR_ERR_UNSUPPORTED;
        a.step = *p.step;
        a.step.rec = p.ws.step_rec;
    }
    a.token_ids = p.token_ids;
    a.logp = p.logp;
    a.z_out = p.z_out;
    a.z_ld = p.z_ld;
    a.trace = t ? static_cast<long long *>(t->trace) : nullptr;
    a.spin_limit = t && t->spin_limit > 0 ? (unsigned)t->spin_limit : 0u;

    int grid = a.passes < cus ? a.passes : cus;
    if (t && t->grid > 0) grid = t->grid < a.passes ? t->grid : a.passes;
    if (grid > kGridMax) grid = kGridMax;

    // The skewed build can replace the default one when every workgroup has exactly one full
    // pass (as at V_rows = 128 * compute units): see the kernel's comment.  It is opt-in
    // (fr_tuning.skew > 0): measured, the even dies do finish ~2 us ahead of the odd ones and
    // the finish times do follow the row counts, but the ninth wavefront (168 instead of 226
    // registers per lane, three wavefronts on one SIMD) costs about as much as the balance gains.
    const int want_skew = t ? t->skew : 0;
    const bool forced = variant == kSkewVariant;
    if ((variant == 0 && want_skew > 0 && !(t && (t->variant > 0 || t->ksplit > 0 || t->grid > 0))) || forced) {
        const int rows = want_skew > 0 ? want_skew : kSkewDefaultRows;
        const int B = p.V_rows / cus;
        const bool ok = KS == 1 && a.passes == cus && grid == cus && (cus % 2) == 0 && p.V_rows == B * cus &&
                        B + rows <= 9 * kTileRows && B - rows >= 1 && cus <= kGridMax && p.M <= 12 &&
                        variant_fits(p.M, p.d, p.k, kSkewVariant);
        if (ok) {
            variant = kSkewVariant;
            a.skew = rows;
        } else if (forced) {
            return FR_ERR_UNSUPPORTED;
        }
    }
    const int lds = lds_bytes(p.M, p.d, p.k, variant);

    const bool lean = sink == Sink::kFusedTopk && p.k <= kSmallKMax && grid <= 4 * kWave && !a.trace && a.spin_limit == 0u;
    const SkinnyKernel kern = select_kernel(variant, a.M, MT, p.k >= kBound32FromK && p.k <= kSmallKMax,
                                            !lean ? 0 : a.step.rec ? 2 : 1);
    if (!kern) return FR_ERR_INVALID_ARG;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kVariants[variant].waves * kWave), lds, s, a);
    const fr_status st = hip_status(hipGetLastError());
    if (st != FR_OK) return st;
    if (sink == Sink::kPartialsOnly) return launch_merge(p, grid, s);
    return FR_OK;
}

}  // namespace frspec
