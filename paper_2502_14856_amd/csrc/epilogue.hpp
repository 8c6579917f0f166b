// Online log-softmax statistics, per-row top-k and the merge of per-workgroup partials.
//
// A workgroup owns a set of vocabulary rows.  For every row m of H it keeps, in LDS,
//   run_ms[m]  = (mx, S): running maximum of its logits and sum of exp(z - mx),
//   run_val/run_id[m][0..k): its k best (logit, token id) pairs, best first,
// folded pass by pass (fold_pass).  On the workgroup's last pass the state goes to the
// workspace, where a few workgroups of the same launch merge the G partial results of every
// row into log Z (Eq. 4's normaliser over the subset) and the final k candidates, and write
// token ids and log-probabilities.  Two ways to the workspace and back:
//   * k <= 16, G <= 256, skinny kernel: self-validating mailbox records, merged by
//     merge_rows_mailbox (and, on request, expanded by expand_step_fused);
//   * otherwise: plain partial arrays plus an arrival counter (arrive_and_wait), merged by
//     final_merge_all, in the same launch or in a second one.
// fold_pair_fast / merge_rows_mailbox are the fast paths; block_fold_rows / final_merge_rows
// are the general ones (any k, any number of tied values).
#pragma once

#include "internal.hpp"
#include "wave_ops.hpp"

namespace frspec {

constexpr int kGridMax = 512;                 // upper bound on workgroups per launch
constexpr int kHeadsPerLane = kGridMax / kWave;

// Per-workgroup partial results in the workspace.  The workgroup index is the fastest
// dimension so that the merge reads the same field of consecutive workgroups from
// consecutive addresses:
//   ms [M][2][kGridMax]   (running max, sum of exp)
//   val[M][k][kGridMax]   id[M][k][kGridMax]   (candidate lists, best first)
struct Partials {
    float *ms;
    float *val;
    int *id;
};
__device__ __forceinline__ size_t part_index(int field, int g) {
    return (size_t)field * kGridMax + g;
}

// The partials cross compute dies whose L2 caches are not coherent with each other.  A
// device-scope fence would write back and invalidate a whole L2 from every wavefront;
// instead every access to a partial is a relaxed device-scope atomic, which the hardware
// performs at the point of coherence (write-through store, cache-missing load).
template <typename T>
__device__ __forceinline__ void publish(T *p, T v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ T observe(const T *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
/*
 * Mailbox of the skinny kernel's single-launch path: the same partial results as 8-byte
 * records that say by themselves whether they have been written.  A record is all ones
 * while empty; a workgroup fills its records with single 8-byte stores (whole or not at
 * all for any reader), the merging workgroup polls the records it needs until none is
 * empty, and empties them again once it has read them.  Between calls every record is
 * empty, so no counter, no flag and no wait for a store to be acknowledged stands
 * between a workgroup's last result and the merge.
 *   rec[m][t][g]  list position t of row m from workgroup g: (value bits << 32) | id
 *   st[m][g]      (running max bits << 32) | (sum-of-exp bits)
 * A token id is never -1 and the statistics are canonicalised, so no real record is all ones.
 */
struct Mailbox {
    unsigned long long *rec;
    unsigned long long *st;
};
constexpr int kStepRows = 16;                 // rows of H whose results the fused expansion collects
constexpr unsigned long long kMailEmpty = ~0ull;
constexpr unsigned kMailSpinLimit = 1u << 20;   // rounds of about a microsecond before giving up
__device__ __forceinline__ size_t mail_rec_index(int m, int t, int g) {
    return (size_t)(m * kMailK + t) * kGridMax + g;
}
__device__ __forceinline__ size_t mail_st_index(int m, int g) { return (size_t)m * kGridMax + g; }
__device__ __forceinline__ unsigned long long mail_pack(float hi, unsigned lo) {
    return ((unsigned long long)__builtin_bit_cast(unsigned, hi) << 32) | lo;
}
__device__ __forceinline__ unsigned long long mail_pack_stats(float mx, float S) {
    unsigned s = __builtin_bit_cast(unsigned, S);
    if (s == 0xFFFFFFFFu) s = 0x7FC00000u;   // a NaN is a NaN; this one is taken
    return mail_pack(mx, s);
}
__device__ __forceinline__ float mail_hi(unsigned long long r) {
    return __builtin_bit_cast(float, (unsigned)(r >> 32));
}
__device__ __forceinline__ float mail_lo_f32(unsigned long long r) {
    return __builtin_bit_cast(float, (unsigned)r);
}

// Blocks the wavefront until its outstanding stores have been acknowledged.
__device__ __forceinline__ void wait_stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Arrival words at the start of the workspace.  Two arrival counters take turns from call
// to call (`parity` says whose turn it is), each on a cache line of its own.
constexpr int kMaxMergers = 32;          // far fewer than the workgroups resident at once
constexpr unsigned kSpinLimit = 1u << 22;   // polls of ~0.2 us each before giving up
struct Arrival {
    unsigned *parity;
    unsigned *error;    // sticky: set to 1 if a bounded wait ever ran out
    unsigned *count;    // count[0] and count[32]
    __device__ explicit Arrival(unsigned *header) : parity(header), error(header + 1), count(header + 32) {}
    // Which counter this call uses; read by every workgroup when it starts.
    __device__ unsigned turn() const { return __hip_atomic_load(parity, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
};

/*
 * The merge of the partials is shared by the first R = min(G, M, kMaxMergers) workgroups
 * to arrive: number r of those merges rows r, r + R, ... of H once all G have arrived.
 * The early finishers have nothing else left to do, and the last workgroup to arrive (the
 * one everybody waits for) only posts its arrival: the mergers see it one memory hop later.
 *
 * An arriving workgroup draws its arrival number from this call's counter; the mergers
 * poll that counter, several polls in flight, until it shows G.  The workgroup that draws
 * the last number clears the OTHER counter (last used by the previous call, which is long
 * over) and hands the turn to it, so the next call starts from zero and no merger has to
 * write, or wait for, anything once its rows are out.
 *
 * Every thread of a workgroup calls this after publishing its partials; `turn` is the
 * value read when the workgroup started.  Returns -1 in workgroups that do not merge
 * (they are finished), else r, after all G workgroups have arrived; r | kWaitTimedOut if the
 * wait was given up after `spin_limit` polls (the caller then reports "no result" for its rows).  At most kMaxMergers
 * workgroups ever wait, the workgroups they wait for need nothing from them, and a
 * waiting workgroup occupies one compute unit of many, so the wait cannot starve a
 * workgroup that has not been scheduled yet; it is bounded all the same.
 */
constexpr int kWaitTimedOut = 1 << 30;   // set in arrive_and_wait's result when its wait ran out
__device__ __forceinline__ int arrive_and_wait(const Arrival &ar, unsigned turn, int G, int R, int *s_slot,
                                               unsigned spin_limit) {
    wait_stores_done();
    __syncthreads();
    if (threadIdx.x == 0) {
        turn &= 1u;
        unsigned *mine = ar.count + 32 * turn;
        const unsigned a = __hip_atomic_fetch_add(mine, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (a == (unsigned)(G - 1)) {
            __hip_atomic_store(ar.count + 32 * (turn ^ 1u), 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(ar.parity, turn ^ 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        int r = a < (unsigned)R ? (int)a : -1;
        if (r >= 0) {
            auto poll = [mine]() { return __hip_atomic_load(mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
            unsigned q0 = poll(), q1 = poll(), q2 = poll(), q3 = poll();   // oldest first
            unsigned polls = 0;
            while (q0 < (unsigned)G) {
                q0 = q1;
                q1 = q2;
                q2 = q3;
                q3 = poll();
                __builtin_amdgcn_s_sleep(1);
                if (++polls > spin_limit) {
                    __hip_atomic_store(ar.error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    r |= kWaitTimedOut;
                    break;
                }
            }
        }
        *s_slot = r;
    }
    __syncthreads();
    return *s_slot;
}

// "No result" for rows first, first + stride, ... of the outputs: what a merger writes when a
// bounded wait ran out, so that a caller who ignores the sticky error word at least sees no
// plausible-looking candidates.  One wavefront; k <= 64.
__device__ __forceinline__ void write_no_result(int first, int stride, int M, int k, int *token_ids, float *logp) {
    const int lane = lane_id();
    for (int m = first; m < M; m += stride)
        if (lane < k) {
            token_ids[(size_t)m * k + lane] = INT_MAX;
            logp[(size_t)m * k + lane] = kNegInf;
        }
}

__device__ __forceinline__ int merger_count(int G, int M) {
    int R = G < M ? G : M;
    return R < kMaxMergers ? R : kMaxMergers;
}

// Where one row of H keeps its running state in LDS, and where its logits of the
// current pass are.
struct FoldRow {
    const float *z_pass;   // KS slices of the pass's logits (slice stride z_slice_stride)
    float *run_ms;         // [2]
    float *run_val;        // [k]
    int *run_id;           // [k]
};

/*
 * One wavefront folds one pass worth of logits of NS rows of H into their running state.
 *   z_pass   LDS, KS slices; the logit of local row r is the sum over the slices, taken in
 *            slice order
 *   ids_pass LDS, token id of each local vocabulary row (already remapped)
 *   n_valid  number of local rows that exist (the rest are padding)
 *   WITH_RUN false on a workgroup's first pass: the running lists are still empty and do
 *            not need to compete
 */
template <int ZR, int NS, bool WITH_RUN>
__device__ __forceinline__ void block_fold_rows(const FoldRow (&row)[NS], int KS, int z_slice_stride,
                                                const int *ids_pass, int n_valid, int k,
                                                SelectScratch *sc) {
    constexpr int CP = ZR / kWave;
    constexpr int CPL = CP + (WITH_RUN ? 1 : 0);
    static_assert(ZR % kWave == 0, "pass rows must be a multiple of the wave size");
    const int lane = lane_id();
    float v[NS][CPL];
    int id[NS][CPL], pl[NS][CPL];
    bool have[NS][CPL];
    float mx[NS], S[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        float local_max = kNegInf;
#pragma unroll
        for (int c = 0; c < CP; ++c) {
            const int r = lane + kWave * c;
            float z = 0.0f;
            for (int q = 0; q < KS; ++q) z += row[s].z_pass[q * z_slice_stride + r];
            const bool ok = r < n_valid;
            have[s][c] = ok;
            v[s][c] = ok ? z : kNegInf;
            id[s][c] = ok ? ids_pass[r] : INT_MAX;
            pl[s][c] = 0;
            local_max = fmaxf(local_max, v[s][c]);
        }
        const float old_mx = WITH_RUN ? row[s].run_ms[0] : kNegInf;
        const float old_S = WITH_RUN ? row[s].run_ms[1] : 0.0f;
        mx[s] = fmaxf(old_mx, wave_max_f32(local_max));
        float part = 0.0f;
#pragma unroll
        for (int c = 0; c < CP; ++c) part += exp_diff(v[s][c], mx[s]);
        S[s] = old_S * exp_diff(old_mx, mx[s]) + wave_sum_f32(part);
        if (WITH_RUN) {   // the running list competes as k more candidates
            v[s][CPL - 1] = (lane < k) ? row[s].run_val[lane] : kNegInf;
            id[s][CPL - 1] = (lane < k) ? row[s].run_id[lane] : INT_MAX;
            have[s][CPL - 1] = id[s][CPL - 1] != INT_MAX;
            pl[s][CPL - 1] = 0;
        }
    }
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        bool decided = false;
        if (k <= kSmallKMax) {
            unsigned hi[CPL], lo[CPL];
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                hi[c] = have[s][c] ? key_hi_of(v[s][c]) : 0u;
                lo[c] = ~(unsigned)id[s][c];
            }
            unsigned long long mine;
            int mine_pl, rank, n;
            decided = wave_topk_small<CPL>(hi, lo, pl[s], k, sc, mine, mine_pl, rank, n);
            if (decided) {
                if (lane < k && lane >= n) {   // fewer candidates than k: the tail stays empty
                    row[s].run_val[lane] = kNegInf;
                    row[s].run_id[lane] = INT_MAX;
                }
                if (lane < n && rank < k) {
                    row[s].run_val[rank] = value_of_key_hi((unsigned)(mine >> 32));
                    row[s].run_id[rank] = (int)~(unsigned)mine;
                }
            }
        }
        if (!decided) {   // large k, or too many tied survivors
            float v1[1][CPL], ov[1];
            int id1[1][CPL], pl1[1][CPL], oid[1], opl1[1];
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                v1[0][c] = v[s][c];
                id1[0][c] = id[s][c];
                pl1[0][c] = 0;
            }
            wave_select_topk<1, CPL>(v1, id1, pl1, k, ov, oid, opl1);
            if (lane < k) {
                row[s].run_val[lane] = ov[0];
                row[s].run_id[lane] = oid[0];
            }
        }
        if (lane == 0) {
            row[s].run_ms[0] = mx[s];
            row[s].run_ms[1] = S[s];
        }
    }
}

// ---------------------------------------------------------------------------------------
// Fast paths for k <= kSmallKMax (16).  Both rest on the same bound: split the candidates
// into 16 groups; the k-th largest of the 16 group maxima is a lower bound of the k-th best
// candidate overall (k different groups hold a candidate at least that good), so only the
// candidates at or above it, k plus a few in expectation, need to be ranked.  The 16 group
// maxima sit in the 16 lanes of a DPP row, where the k-th largest takes 15 row rotations.
// ---------------------------------------------------------------------------------------

typedef float fvec4 __attribute__((ext_vector_type(4)));
typedef float fvec2 __attribute__((ext_vector_type(2)));
typedef int ivec4 __attribute__((ext_vector_type(4)));
typedef int ivec2 __attribute__((ext_vector_type(2)));
typedef unsigned long long u64x2 __attribute__((ext_vector_type(2)));

// C consecutive 4-byte words of LDS, as one access.
template <int C, typename T, typename V4, typename V2>
__device__ __forceinline__ void lds_words(const T *p, T (&out)[C]) {
    static_assert(C == 1 || C == 2 || C == 4 || C == 8, "1, 2, 4 or 8 words per lane");
    if constexpr (C == 8) {
        const V4 a = *reinterpret_cast<const V4 *>(p), b = *reinterpret_cast<const V4 *>(p + 4);
        out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
        out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
    } else if constexpr (C == 4) {
        const V4 v = *reinterpret_cast<const V4 *>(p);
        out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
    } else if constexpr (C == 2) {
        const V2 v = *reinterpret_cast<const V2 *>(p);
        out[0] = v.x; out[1] = v.y;
    } else {
        out[0] = *p;
    }
}

// Where a fold puts its results: the workgroup's running state in LDS, or, on the
// workgroup's last pass, straight into the workspace (slot g of the partials, or of the
// mailbox).
enum class FoldTo : int { kLds = 0, kPartials = 1, kMailbox = 2 };
struct FoldSink {
    FoldTo to;
    Partials part;
    Mailbox mail;
    int g;
    float *run_ms;
    float *run_val;
    int *run_id;
    __device__ __forceinline__ void entry(int m, int k, int slot, float v, int id) const {
        if (to == FoldTo::kMailbox) {
            publish(mail.rec + mail_rec_index(m, slot, g), mail_pack(v, (unsigned)id));
        } else if (to == FoldTo::kPartials) {
            publish(part.val + part_index(m * k + slot, g), v);
            publish(part.id + part_index(m * k + slot, g), id);
        } else {
            run_val[m * k + slot] = v;
            run_id[m * k + slot] = id;
        }
    }
    __device__ __forceinline__ void stats(int m, float mx, float S) const {
        if (to == FoldTo::kMailbox) {
            publish(mail.st + mail_st_index(m, g), mail_pack_stats(mx, S));
        } else if (to == FoldTo::kPartials) {
            publish(part.ms + part_index(m * 2, g), mx);
            publish(part.ms + part_index(m * 2 + 1, g), S);
        } else {
            run_ms[2 * m] = mx;
            run_ms[2 * m + 1] = S;
        }
    }
};

/*
 * One wavefront folds one pass of logits of TWO rows of H at once, one per half of the
 * wavefront: lane (h, l32) works on row `m` (the same for the 32 lanes of a half;
 * `active` false if that row does not exist) and holds C = ZR_MAX / 32 consecutive local
 * vocabulary rows, plus entry l32 of the row's running list when WITH_RUN.  A group is
 * the pair of lanes (l32, l32 ^ 16).
 *   z_lds   logits of the pass, row m at z_lds + (m - m_base) * z_row_stride (+ q *
 *           z_slice_stride for slice q of a split d); the logit is the sum of the slices in
 *           slice order
 * Returns false, having written nothing, when more than 32 candidates of a row survive
 * the bound (heavily tied values, or fewer than k populated groups): the caller then
 * takes the general path for both rows.
 */
template <int ZR_MAX, bool WITH_RUN, bool WITH_EXTRA = false, bool B32 = false>
__device__ __forceinline__ bool fold_pair_fast(const float *z_lds, int z_row_stride, int m_base, int KS,
                                               int z_slice_stride, const int *ids_pass, int n_valid, int k, int m,
                                               bool active, const FoldSink &out, SelectScratch *sc) {
    constexpr int C = ZR_MAX / 32;
    constexpr int CPL = C + (WITH_RUN ? 1 : 0) + (WITH_EXTRA ? 1 : 0);
    const int lane = lane_id(), h = lane >> 5, l32 = lane & 31;
    const int mm = active ? m : m_base;
    // WITH_EXTRA: the pass has up to 16 more local rows than the ZR_MAX that the lanes cover C
    // at a time (slots ZR_MAX .. ZR_MAX + 15); lane l32 < 16 takes slot ZR_MAX + l32 as one
    // more candidate

    float z[C];
#pragma unroll
    for (int c = 0; c < C; ++c) z[c] = 0.0f;
    const float *zp = z_lds + (mm - m_base) * z_row_stride + l32 * C;
    for (int q = 0; q < KS; ++q) {
        float t[C];
        lds_words<C, float, fvec4, fvec2>(zp + q * z_slice_stride, t);
#pragma unroll
        for (int c = 0; c < C; ++c) z[c] += t[c];
    }
    int id[C];
    lds_words<C, int, ivec4, ivec2>(ids_pass + l32 * C, id);
    float z_x = 0.0f;
    int id_x = INT_MAX;
    bool ok_x = false;
    if (WITH_EXTRA) {
        const int rx = ZR_MAX + (l32 & 15);   // always inside the rows of the pass's z block
        ok_x = active && l32 < 16 && rx < n_valid;
        for (int q = 0; q < KS; ++q) z_x += z_lds[(mm - m_base) * z_row_stride + q * z_slice_stride + rx];
        id_x = ids_pass[ok_x ? rx : 0];
    }
    const int kk = l32 < k ? l32 : k - 1;
    float old_mx = kNegInf, old_S = 0.0f, run_v = kNegInf;
    int run_i = INT_MAX;
    if (WITH_RUN) {
        old_mx = out.run_ms[2 * mm];
        old_S = out.run_ms[2 * mm + 1];
        run_v = out.run_val[mm * k + kk];
        run_i = out.run_id[mm * k + kk];
        if (!(active && l32 < k)) run_i = INT_MAX;
    }

    // online softmax statistics of the row (Eq. 4's normaliser, accumulated per pass)
    float v[C];
    bool ok[C];
    float lmax = kNegInf;
#pragma unroll
    for (int c = 0; c < C; ++c) {
        ok[c] = active && (l32 * C + c < n_valid);
        v[c] = ok[c] ? z[c] : kNegInf;
        lmax = fmaxf(lmax, v[c]);
    }
    const float v_x = ok_x ? z_x : kNegInf;
    if (WITH_EXTRA) lmax = fmaxf(lmax, v_x);
    const float mx = fmaxf(old_mx, row16_max_f32(max_xor16_f32(lmax)));
    float part = 0.0f;
#pragma unroll
    for (int c = 0; c < C; ++c) part += exp_diff(v[c], mx);
    if (WITH_EXTRA) part += exp_diff(v_x, mx);
    part = sum_xor16_f32(part);
    const float S = old_S * exp_diff(old_mx, mx) + row16_sum_all(part);

    // candidates as keys, and the bound
    unsigned hi[CPL], lo[CPL];
#pragma unroll
    for (int c = 0; c < C; ++c) {
        hi[c] = ok[c] ? key_hi_of(v[c]) : 0u;
        lo[c] = ~(unsigned)id[c];
    }
    if (WITH_EXTRA) {
        hi[C] = ok_x ? key_hi_of(v_x) : 0u;
        lo[C] = ~(unsigned)id_x;
    }
    if (WITH_RUN) {
        hi[CPL - 1] = run_i != INT_MAX ? key_hi_of(run_v) : 0u;
        lo[CPL - 1] = ~(unsigned)run_i;
    }
    unsigned lm = hi[0];
#pragma unroll
    for (int c = 1; c < CPL; ++c) lm = max(lm, hi[c]);
    // (groups: the 16 lane pairs (l, l ^ 16) of the half; from k = 11 on every lane of its own)
    const unsigned L = B32 ? half32_kth_largest_u32(lm, k) : row16_kth_largest_u32(max_xor16_u32(lm), k);

    // survivors of each half, packed into its 32 scratch slots
    sc->key[lane] = 0ull;
    int n0 = 0, n1 = 0;
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        const bool sv = hi[c] != 0u && hi[c] >= L;
        const unsigned long long mask = __ballot(sv);
        const int c_lo = __popc((unsigned)mask), c_hi = __popc((unsigned)(mask >> 32));
        const int before = (int)__builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32),
                                                          __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u));
        const int pos = h ? before - c_lo + n1 : before + n0;
        if (sv && pos < 32) sc->key[h * 32 + pos] = make_key(hi[c], lo[c]);
        n0 += c_lo;
        n1 += c_hi;
    }
    if (n0 > 32 || n1 > 32) return false;

    // rank = number of better survivors of the same row (the unused slots hold zero keys)
    const unsigned long long mine = sc->key[lane];
    const u64x2 *kp = reinterpret_cast<const u64x2 *>(sc->key + h * 32);
    const int nmax = n0 > n1 ? n0 : n1;
    int rank = 0;
#pragma unroll 4
    for (int j = 0; j < nmax; j += 2) {
        const u64x2 two = kp[j >> 1];
        rank += two.x > mine;
        rank += two.y > mine;
    }
    if (active) {
        const int n_h = h ? n1 : n0;
        if (mine != 0ull && rank < k)
            out.entry(m, k, rank, value_of_key_hi((unsigned)(mine >> 32)), (int)~(unsigned)mine);
        if (l32 >= n_h && l32 < k) out.entry(m, k, l32, kNegInf, INT_MAX);   // fewer candidates than k
        if (l32 == 0) out.stats(m, mx, S);
    }
    return true;
}

/*
 * The same for FOUR rows of H at once, one per quarter of the wavefront (a DPP row of 16
 * lanes): lane (r, l16) works on row `m` (the same for the 16 lanes of a quarter) and holds
 * C = ZR_MAX / 16 consecutive local vocabulary rows, plus entry l16 of the row's running
 * list when WITH_RUN.  A group is one lane, so the 16 group maxima already sit in the 16
 * lanes of the row.  Up to 32 survivors per row, two per lane when they are ranked.
 */
template <int ZR_MAX, bool WITH_RUN, bool B32 = false>
__device__ __forceinline__ bool fold_quad_fast(const float *z_lds, int z_row_stride, int m_base, int KS,
                                               int z_slice_stride, const int *ids_pass, int n_valid, int k, int m,
                                               bool active, const FoldSink &out, SelectScratch *sc) {
    constexpr int C = ZR_MAX / 16;
    constexpr int CPL = C + (WITH_RUN ? 1 : 0);
    const int lane = lane_id(), r = lane >> 4, l16 = lane & 15;
    const int mm = active ? m : m_base;

    float z[C];
#pragma unroll
    for (int c = 0; c < C; ++c) z[c] = 0.0f;
    const float *zp = z_lds + (mm - m_base) * z_row_stride + l16 * C;
    for (int q = 0; q < KS; ++q) {
        float t[C];
        lds_words<C, float, fvec4, fvec2>(zp + q * z_slice_stride, t);
#pragma unroll
        for (int c = 0; c < C; ++c) z[c] += t[c];
    }
    int id[C];
    lds_words<C, int, ivec4, ivec2>(ids_pass + l16 * C, id);
    const int kk = l16 < k ? l16 : k - 1;
    float old_mx = kNegInf, old_S = 0.0f, run_v = kNegInf;
    int run_i = INT_MAX;
    if (WITH_RUN) {
        old_mx = out.run_ms[2 * mm];
        old_S = out.run_ms[2 * mm + 1];
        run_v = out.run_val[mm * k + kk];
        run_i = out.run_id[mm * k + kk];
        if (!(active && l16 < k)) run_i = INT_MAX;
    }

    // online softmax statistics of the row (Eq. 4's normaliser, accumulated per pass)
    float v[C];
    bool ok[C];
    float lmax = kNegInf;
#pragma unroll
    for (int c = 0; c < C; ++c) {
        ok[c] = active && (l16 * C + c < n_valid);
        v[c] = ok[c] ? z[c] : kNegInf;
        lmax = fmaxf(lmax, v[c]);
    }
    const float mx = fmaxf(old_mx, row16_max_f32(lmax));
    float part = 0.0f;
#pragma unroll
    for (int c = 0; c < C; ++c) part += exp_diff(v[c], mx);
    const float S = old_S * exp_diff(old_mx, mx) + row16_sum_all(part);

    // candidates as keys, and the bound: the k-th largest of the 16 lane maxima
    unsigned hi[CPL], lo[CPL];
#pragma unroll
    for (int c = 0; c < C; ++c) {
        hi[c] = ok[c] ? key_hi_of(v[c]) : 0u;
        lo[c] = ~(unsigned)id[c];
    }
    if (WITH_RUN) {
        hi[CPL - 1] = run_i != INT_MAX ? key_hi_of(run_v) : 0u;
        lo[CPL - 1] = ~(unsigned)run_i;
    }
    unsigned L;
    if constexpr (B32) {
        // 32 groups: the two halves of the lane's logits (the entry of the running list joins the second)
        unsigned la = hi[0], lb = hi[C / 2];
#pragma unroll
        for (int c = 1; c < C / 2; ++c) la = max(la, hi[c]);
#pragma unroll
        for (int c = C / 2 + 1; c < CPL; ++c) lb = max(lb, hi[c]);
        L = row16x2_kth_largest_u32(la, lb, k);
    } else {
        unsigned lm = hi[0];
#pragma unroll
        for (int c = 1; c < CPL; ++c) lm = max(lm, hi[c]);
        L = row16_kth_largest_u32(lm, k);
    }

    // survivors of each row, packed into its 32 scratch slots
    sc->key[lane] = 0ull;
    sc->key[kWave + lane] = 0ull;
    const unsigned below = (1u << l16) - 1u;
    int n = 0;   // survivors of this lane's row so far
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        const bool sv = hi[c] != 0u && hi[c] >= L;
        const unsigned field = (unsigned)(__ballot(sv) >> (16 * r)) & 0xFFFFu;
        const int pos = n + __popc(field & below);
        if (sv && pos < 32) sc->key[r * 32 + pos] = make_key(hi[c], lo[c]);
        n += __popc(field);
    }
    if (__any(n > 32)) return false;

    // rank = number of better survivors of the same row (the unused slots hold zero keys);
    // lane l16 ranks the survivors in slots l16 and 16 + l16
    const unsigned long long mine_a = sc->key[r * 32 + l16], mine_b = sc->key[r * 32 + 16 + l16];
    const u64x2 *kp = reinterpret_cast<const u64x2 *>(sc->key + r * 32);
    const int nmax = max(max(__builtin_amdgcn_readlane(n, 0), __builtin_amdgcn_readlane(n, 16)),
                         max(__builtin_amdgcn_readlane(n, 32), __builtin_amdgcn_readlane(n, 48)));
    int rank_a = 0, rank_b = 0;
#pragma unroll 4
    for (int j = 0; j < nmax; j += 2) {
        const u64x2 two = kp[j >> 1];
        rank_a += two.x > mine_a;
        rank_a += two.y > mine_a;
        rank_b += two.x > mine_b;
        rank_b += two.y > mine_b;
    }
    if (active) {
        if (mine_a != 0ull && rank_a < k)
            out.entry(m, k, rank_a, value_of_key_hi((unsigned)(mine_a >> 32)), (int)~(unsigned)mine_a);
        if (mine_b != 0ull && rank_b < k)
            out.entry(m, k, rank_b, value_of_key_hi((unsigned)(mine_b >> 32)), (int)~(unsigned)mine_b);
        if (l16 >= n && l16 < k) out.entry(m, k, l16, kNegInf, INT_MAX);   // fewer candidates than k
        if (l16 == 0) out.stats(m, mx, S);
    }
    return true;
}

// General fold of one row by one whole wavefront, kept out of line: any k, any number of
// tied values.  The row's state stays in LDS; on the workgroup's last pass it is also
// written out.
template <int ZR, bool WITH_RUN>
__device__ __noinline__ void fold_row_general(FoldRow row, int KS, int z_slice_stride, const int *ids_pass,
                                              int n_valid, int k, SelectScratch *sc, FoldSink out, int m) {
    const FoldRow rows[1] = {row};
    block_fold_rows<ZR, 1, WITH_RUN>(rows, KS, z_slice_stride, ids_pass, n_valid, k, sc);
    if (out.to != FoldTo::kLds) {
        const int lane = lane_id();
        if (lane < k) out.entry(m, k, lane, row.run_val[lane], row.run_id[lane]);
        if (lane == 0) out.stats(m, row.run_ms[0], row.run_ms[1]);
    }
}

/*
 * Folds one pass into the running state of rows m_base <= m < m_end of H, or, on the
 * workgroup's last pass, writes the result out (see FoldSink).  While k <= 16, wavefront w
 * of `waves` takes rows m_base + w and m_base + w + waves (then + 2 * waves, ...), two at a
 * time in its two halves; with QUAD, rows m_base + 4w .. 4w + 3 (then + 4 * waves, ...), four
 * at a time in its quarters.  A fold is one long chain of dependent instructions and LDS
 * round trips, and the four-row one is the longer chain: QUAD pays off where the rows
 * would otherwise take more than one round per wavefront.
 */
template <int ZR_MAX, bool WITH_RUN, bool WITH_EXTRA = false, bool QUAD = false, bool B32 = false, typename RowOf>
__device__ __forceinline__ void fold_pass(const float *z_lds, int z_row_stride, int KS, int z_slice_stride,
                                          const int *ids_pass, int n_valid, int k, int m_base, int m_end, int wave,
                                          int waves, RowOf row_of, const FoldSink &out, SelectScratch *sc) {
    // the general fold covers 64 local rows per lane slot: one more slot takes the extra rows
    constexpr int ZR_GEN = WITH_EXTRA ? ZR_MAX + kWave : ZR_MAX;
    static_assert(!(QUAD && WITH_EXTRA), "the four-row fold takes no extra rows");
    if (QUAD && k <= kSmallKMax) {
        for (int mb = m_base; mb < m_end; mb += 4 * waves) {
            const int m0 = mb + 4 * wave;
            if (m0 >= m_end) break;
            const int m = m0 + (lane_id() >> 4);
            if (fold_quad_fast<ZR_MAX, WITH_RUN, B32>(z_lds, z_row_stride, m_base, KS, z_slice_stride, ids_pass, n_valid, k,
                                                 m, m < m_end, out, sc))
                continue;
            for (int i = 0; i < 4 && m0 + i < m_end; ++i)
                fold_row_general<ZR_GEN, WITH_RUN>(row_of(m0 + i), KS, z_slice_stride, ids_pass, n_valid, k, sc, out,
                                                   m0 + i);
        }
    } else if (k <= kSmallKMax) {
        for (int mb = m_base; mb < m_end; mb += 2 * waves) {
            const int m_lo = mb + wave, m_hi = mb + wave + waves;
            if (m_lo >= m_end) break;
            const int m = (lane_id() >> 5) ? m_hi : m_lo;
            if (fold_pair_fast<ZR_MAX, WITH_RUN, WITH_EXTRA, B32>(z_lds, z_row_stride, m_base, KS, z_slice_stride,
                                                             ids_pass, n_valid, k, m, m < m_end, out, sc))
                continue;
            fold_row_general<ZR_GEN, WITH_RUN>(row_of(m_lo), KS, z_slice_stride, ids_pass, n_valid, k, sc, out, m_lo);
            if (m_hi < m_end)
                fold_row_general<ZR_GEN, WITH_RUN>(row_of(m_hi), KS, z_slice_stride, ids_pass, n_valid, k, sc, out,
                                                   m_hi);
        }
    } else {
        for (int m = m_base + wave; m < m_end; m += waves)
            fold_row_general<ZR_GEN, WITH_RUN>(row_of(m), KS, z_slice_stride, ids_pass, n_valid, k, sc, out, m);
    }
}


// Candidate number c of the triangle {(i, t): i + t < k}, rows i listed one after the
// other (row i holds k - i entries and starts at i*k - i(i-1)/2).
__device__ __forceinline__ void triangle_coords(int c, int k, int &i, int &t) {
    const float b = (float)(2 * k + 1);
    i = (int)((b - __builtin_sqrtf(b * b - 8.0f * (float)c)) * 0.5f);
    i = i < 0 ? 0 : (i > k - 1 ? k - 1 : i);
    auto start = [k](int r) { return r * k - r * (r - 1) / 2; };
    if (i + 1 < k && start(i + 1) <= c) ++i;   // the float root may be off by one either way
    if (i > 0 && start(i) > c) --i;
    t = c - start(i);
}

/*
 * One wavefront merges the G partial results of NS rows of H and writes their outputs.
 * Every partial list is sorted, so the k best overall lie in the k lists with the best
 * heads, and list number i (by head) can contribute at most k - i entries: the search
 * space shrinks from G*k to k(k+1)/2 candidates.  HPL = ceil(G / 64) heads per lane.
 * All loads are issued unconditionally from clamped (always valid) addresses so that
 * they overlap; what a lane must not see is masked afterwards.
 */
template <int NS, int HPL>
__device__ __forceinline__ void final_merge_rows(const Partials &P, int G, const int (&m)[NS], int k,
                                                 int *token_ids, float *logp, SelectScratch *sc) {
    const int lane = lane_id();
    float hv[NS][HPL];
    int hid[NS][HPL], hg[NS][HPL];
    float logZ[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        // log Z = mx + log sum_g S_g exp(mx_g - mx)
        float mxs[HPL], Ss[HPL];
#pragma unroll
        for (int q = 0; q < HPL; ++q) {
            const int g = lane + kWave * q;
            const int gs = g < G ? g : G - 1;
            mxs[q] = observe(P.ms + part_index(m[s] * 2, gs));
            Ss[q] = observe(P.ms + part_index(m[s] * 2 + 1, gs));
            hv[s][q] = observe(P.val + part_index(m[s] * k, gs));
            hid[s][q] = observe(P.id + part_index(m[s] * k, gs));
        }
        float lmx = kNegInf;
#pragma unroll
        for (int q = 0; q < HPL; ++q) {
            const bool ok = lane + kWave * q < G;
            mxs[q] = ok ? mxs[q] : kNegInf;
            Ss[q] = ok ? Ss[q] : 0.0f;
            hv[s][q] = ok ? hv[s][q] : kNegInf;
            hid[s][q] = ok ? hid[s][q] : INT_MAX;
            hg[s][q] = ok ? lane + kWave * q : -1;
            lmx = fmaxf(lmx, mxs[q]);
        }
        const float mx = wave_max_f32(lmx);
        float part = 0.0f;
#pragma unroll
        for (int q = 0; q < HPL; ++q) part += Ss[q] * exp_diff(mxs[q], mx);
        logZ[s] = mx + __logf(wave_sum_f32(part));
    }

    const int n_cand = k * (k + 1) / 2;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        // ---- the k lists with the best heads: sc->pl[i] = workgroup of list number i
        bool decided = false;
        if (k <= kSmallKMax) {
            unsigned hi[HPL], lo[HPL];
#pragma unroll
            for (int q = 0; q < HPL; ++q) {
                hi[q] = hid[s][q] != INT_MAX ? key_hi_of(hv[s][q]) : 0u;
                lo[q] = ~(unsigned)hid[s][q];
            }
            unsigned long long mine;
            int mine_pl, rank, n;
            decided = wave_topk_small<HPL>(hi, lo, hg[s], k, sc, mine, mine_pl, rank, n);
            if (decided) {
                if (lane < k) sc->pl[lane] = -1;   // slots of missing lists (fewer than k)
                if (lane < n && rank < k) sc->pl[rank] = mine_pl;
            }
        }
        if (!decided) {
            float v1[1][HPL], lv[1];
            int id1[1][HPL], pl1[1][HPL], lid[1], lg1[1];
#pragma unroll
            for (int q = 0; q < HPL; ++q) {
                v1[0][q] = hv[s][q];
                id1[0][q] = hid[s][q];
                pl1[0][q] = hg[s][q];
            }
            wave_select_topk<1, HPL>(v1, id1, pl1, k, lv, lid, lg1);
            if (lane < k) sc->pl[lane] = lg1[0];
        }

        // ---- candidates (i, t), i + t < k
        auto fetch = [&](int c, float &cv, int &cid) {
            int i, t;
            triangle_coords(c < n_cand ? c : 0, k, i, t);
            const int g = sc->pl[i];
            const bool ok = (c < n_cand) && (g >= 0) && (g < G);
            const size_t at = part_index(m[s] * k + t, ok ? g : 0);
            cv = observe(P.val + at);
            cid = observe(P.id + at);
            cv = ok ? cv : kNegInf;
            cid = ok ? cid : INT_MAX;
        };
        if (k <= kSmallKMax) {
            if (n_cand <= kWave) {
                // up to k = 10 the candidates sit one per lane: rank them all directly
                float cv;
                int cid;
                fetch(lane, cv, cid);
                const unsigned long long mine =
                    cid != INT_MAX ? make_key(key_hi_of(cv), ~(unsigned)cid) : 0ull;
                const int rank = wave_rank_all(mine, sc);
                int n = (int)__popcll(__ballot(mine != 0ull));
                if (lane < k && lane >= n) {
                    token_ids[(size_t)m[s] * k + lane] = INT_MAX;
                    logp[(size_t)m[s] * k + lane] = kNegInf;
                }
                if (mine != 0ull && rank < k) {
                    token_ids[(size_t)m[s] * k + rank] = cid;
                    logp[(size_t)m[s] * k + rank] = cv - logZ[s];
                }
            } else {
                constexpr int C2 = 3;   // 16 * 17 / 2 = 136 candidates at most
                float cv[C2];
                int cid[C2], cpl[C2];
#pragma unroll
                for (int q = 0; q < C2; ++q) fetch(lane + kWave * q, cv[q], cid[q]);
                unsigned hi[C2], lo[C2];
#pragma unroll
                for (int q = 0; q < C2; ++q) {
                    hi[q] = cid[q] != INT_MAX ? key_hi_of(cv[q]) : 0u;
                    lo[q] = ~(unsigned)cid[q];
                    cpl[q] = 0;
                }
                unsigned long long mine;
                int mine_pl, rank, n;
                if (wave_topk_small<C2>(hi, lo, cpl, k, sc, mine, mine_pl, rank, n)) {
                    if (lane < k && lane >= n) {
                        token_ids[(size_t)m[s] * k + lane] = INT_MAX;
                        logp[(size_t)m[s] * k + lane] = kNegInf;
                    }
                    if (lane < n && rank < k) {
                        token_ids[(size_t)m[s] * k + rank] = (int)~(unsigned)mine;
                        logp[(size_t)m[s] * k + rank] = value_of_key_hi((unsigned)(mine >> 32)) - logZ[s];
                    }
                } else {
                    float v1[1][C2], ov[1];
                    int id1[1][C2], pl1[1][C2], oid[1], opl[1];
#pragma unroll
                    for (int q = 0; q < C2; ++q) {
                        v1[0][q] = cv[q];
                        id1[0][q] = cid[q];
                        pl1[0][q] = 0;
                    }
                    wave_select_topk<1, C2>(v1, id1, pl1, k, ov, oid, opl);
                    if (lane < k) {
                        token_ids[(size_t)m[s] * k + lane] = oid[0];
                        logp[(size_t)m[s] * k + lane] = ov[0] - logZ[s];
                    }
                }
            }
        } else {
            // Large k: the candidates stay in memory.  Round j picks the best candidate that
            // is strictly after the previous winner in the (value, id) order; ids are
            // distinct, so this walks the sorted order without marking anything.
            float ov = kNegInf;
            int oid = INT_MAX;
            float pv = __builtin_huge_valf();
            int pid = -1;
            for (int j = 0; j < k; ++j) {
                float bv = kNegInf;
                int bi = INT_MAX;
                for (int q = 0; q * kWave < n_cand; ++q) {
                    float cv;
                    int cid;
                    fetch(lane + kWave * q, cv, cid);
                    const bool after_prev = cand_before(pv, pid, cv, cid);
                    if (after_prev && cand_before(cv, cid, bv, bi)) {
                        bv = cv;
                        bi = cid;
                    }
                }
                const float wmax = wave_max_f32(bv);
                const int wid = wave_min_i32(bv == wmax ? bi : INT_MAX);
                if (lane == j) {
                    ov = wmax;
                    oid = wid;
                }
                pv = wmax;
                pid = wid;
            }
            if (lane < k) {
                token_ids[(size_t)m[s] * k + lane] = oid;
                logp[(size_t)m[s] * k + lane] = ov - logZ[s];
            }
        }
    }
}

template <int NS>
__device__ __forceinline__ void final_merge_dispatch(const Partials &P, int G, const int (&m)[NS],
                                                     int k, int *token_ids, float *logp,
                                                     SelectScratch *sc) {
    if (G <= kWave) final_merge_rows<NS, 1>(P, G, m, k, token_ids, logp, sc);
    else if (G <= 2 * kWave) final_merge_rows<NS, 2>(P, G, m, k, token_ids, logp, sc);
    else if (G <= 4 * kWave) final_merge_rows<NS, 4>(P, G, m, k, token_ids, logp, sc);
    else final_merge_rows<NS, kHeadsPerLane>(P, G, m, k, token_ids, logp, sc);
}

// Merges rows m = first, first + stride, ... < M, two at a time where possible.
__device__ __forceinline__ void final_merge_all(const Partials &P, int G, int first, int stride, int M, int k,
                                       int *token_ids, float *logp, SelectScratch *sc) {
    int m = first;
    for (; m + stride < M; m += 2 * stride) {
        const int ms[2] = {m, m + stride};
        final_merge_dispatch<2>(P, G, ms, k, token_ids, logp, sc);
    }
    if (m < M) {
        const int ms[1] = {m};
        final_merge_dispatch<1>(P, G, ms, k, token_ids, logp, sc);
    }
}


// Scratch of the fast merge, one per workgroup.
struct alignas(16) MergeScratch {
    unsigned long long key[kWave];
    unsigned count;
    float logZ;
    unsigned timed_out;   // a fetching wavefront gave up waiting for this row's records
};

// The general merge of a set of rows by one wavefront, kept out of line.
__device__ __noinline__ void final_merge_general(Partials P, int G, int first, int stride, int M, int k,
                                                 int *token_ids, float *logp, SelectScratch *sc) {
    final_merge_all(P, G, first, stride, M, k, token_ids, logp, sc);
}

/*
 * The beam-search expansion of a draft step (Section 2 of the paper) fused into the LM head's
 * launch.  The merger of every row of H hands the row's k results on as records
 * step_rec[m][t] = (logp bits << 32) | token, all ones while empty; the first merger, when
 * its own rows are out, collects all M * k of them, forms the cumulative scores
 * node_score[m] + logp, appends the candidates to the search history and returns the `width`
 * best as the next nodes: what fr_beam_expand does in a launch of its own.
 */

// One wavefront; keys: LDS, at least M * k + 2 entries, 16-byte aligned.
__device__ __forceinline__ void expand_step_fused(const StepArgs &st, int M, int k, unsigned long long *keys,
                                                  unsigned *error, unsigned spin_limit) {
    constexpr int CPL = kStepRows * kMailK / kWave;   // 4 candidates per lane at most
    const int lane = lane_id(), C = M * k;
    unsigned long long r[CPL];
    int row[CPL], at[CPL];
    bool inb[CPL];
#pragma unroll
    for (int q = 0; q < CPL; ++q) {
        const int c = lane + kWave * q;
        inb[q] = c < C;
        row[q] = inb[q] ? c / k : 0;
        at[q] = row[q] * kMailK + (inb[q] ? c - row[q] * k : 0);
        r[q] = observe(st.rec + at[q]);
    }
    for (unsigned polls = 0;; ++polls) {
        bool again = false;
#pragma unroll
        for (int q = 0; q < CPL; ++q)
            if (inb[q] && r[q] == kMailEmpty) {
                r[q] = observe(st.rec + at[q]);
                again = true;
            }
        if (!__any(again)) break;
        if (polls > spin_limit) {
            // given up: no next nodes, the history stays as it was
            if (lane == 0) __hip_atomic_store(error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            for (int w = lane; w < st.width; w += kWave) {
                st.next_score[w] = kNegInf;
                st.next_token[w] = INT_MAX;
                st.next_hist[w] = -1;
            }
            return;
        }
        __builtin_amdgcn_s_sleep(1);
    }
    float score[CPL];
#pragma unroll
    for (int q = 0; q < CPL; ++q) {
        const int c = lane + kWave * q;
        if (inb[q]) {
            publish(st.rec + at[q], kMailEmpty);
            score[q] = st.node_score[row[q]] + mail_hi(r[q]);   // the one rounding of the cumulative score
            st.hist_score[st.hist_offset + c] = score[q];
            st.hist_token[st.hist_offset + c] = (int)(unsigned)r[q];
            st.hist_parent[st.hist_offset + c] = st.node_hist[row[q]];
        }
    }
    // Only the `width` best are wanted, not every candidate's rank: the candidates fall into 16 groups
    // (lanes l, l + 16, l + 32, l + 48, all their candidates); the width-th largest group maximum is a
    // lower bound of the width-th best score; the candidates at or above it (width plus a few) are
    // packed into `keys` and ranked among themselves.
    unsigned khi[CPL];
    unsigned lm = 0u;
#pragma unroll
    for (int q = 0; q < CPL; ++q) {
        khi[q] = inb[q] ? key_hi_of(score[q]) : 0u;
        lm = max(lm, khi[q]);
    }
    const unsigned gm = max_xor32_u32(max_xor16_u32(lm));
    const unsigned bound = st.width <= 16 ? row16_kth_largest_u32(gm, st.width) : 0u;
    int n = 0;
    bool sv[CPL];
#pragma unroll
    for (int q = 0; q < CPL; ++q) {
        sv[q] = khi[q] != 0u && khi[q] >= bound;
        const unsigned long long mask = __ballot(sv[q]);
        const int pos = n + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u));
        if (sv[q]) keys[pos] = make_key(khi[q], ~(unsigned)(lane + kWave * q));
        n += (int)__popcll(mask);
    }
    if (lane == 0) keys[n] = 0ull;
    // (one wavefront: its LDS operations execute in order, no barrier needed)
    const u64x2 *kp = reinterpret_cast<const u64x2 *>(keys);
#pragma unroll
    for (int q = 0; q < CPL; ++q) {
        if (__ballot(sv[q]) == 0ull) continue;
        const unsigned long long mine = sv[q] ? make_key(khi[q], ~(unsigned)(lane + kWave * q)) : ~0ull;
        int rank = 0;
        for (int j = 0; j < n; j += 2) {
            const u64x2 two = kp[j >> 1];
            rank += two.x > mine;
            rank += two.y > mine;
        }
        if (sv[q] && rank < st.width) {
            st.next_score[rank] = score[q];
            st.next_token[rank] = (int)(unsigned)r[q];
            st.next_hist[rank] = (int)(st.hist_offset + lane + kWave * q);
        }
    }
}

/*
 * A workgroup merges the G <= 256 mailbox records of rows first, first + stride, ... of H,
 * k <= 16.  Four wavefronts (one per SIMD; the others only keep the barriers company)
 * fetch, and keep fetching until none is empty: entry t of all G lists for the list
 * positions t = wave, wave + 4, ...; the G list heads (position 0), for the bound; and,
 * the last of the four, the softmax statistics.  The groups of the bound are the 16 sets
 * of heads {g : g mod 16 = j}.  Each wavefront keeps those of its entries that reach the
 * bound (k plus a few survive, out of G * k: most registers hold none, and those are
 * skipped), the survivors meet in LDS, and the first wavefront ranks them and writes
 * the outputs.  The records are emptied for the next call on the way.
 */
template <int NW = 4, bool B32 = false>   // NW fetching wavefronts: 4 or 8, at most the wavefronts of the workgroup
__device__ __forceinline__ void merge_rows_mailbox(const Mailbox &mb, const Partials &P, unsigned *error, int G,
                                                   int first, int stride, int M, int k, int *token_ids,
                                                   float *logp, MergeScratch *ms, SelectScratch *sc,
                                                   unsigned long long *step_rec, unsigned spin_limit) {
    constexpr int HPL = 4;                      // G <= 256
    static_assert(NW == 4 || NW == 8, "list positions are dealt out evenly");
    constexpr int TPW = kMailK / NW;            // list positions per fetching wavefront
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x / kWave);
    for (int m = first; m < M; m += stride) {
        if (wave == 0) {
            ms->key[lane] = 0ull;
            if (lane == 0) {
                ms->count = 0u;
                ms->timed_out = 0u;
            }
        }
        __syncthreads();
        unsigned long long ent[TPW][HPL], head[HPL], stt[HPL];
        const unsigned long long *hrow = mb.rec + mail_rec_index(m, 0, 0);
        const unsigned long long *srow = mb.st + mail_st_index(m, 0);
        if (wave < NW) {
            // ---- fetch until no record is empty; unconditional first round from clamped
            // addresses, then only what is still missing
#pragma unroll
            for (int q = 0; q < HPL; ++q) {
                const int g = lane + kWave * q, gs = g < G ? g : G - 1;
#pragma unroll
                for (int j = 0; j < TPW; ++j) {
                    const int t = wave + j * NW, ts = t < k ? t : 0;
                    ent[j][q] = observe(mb.rec + mail_rec_index(m, ts, gs));
                }
                head[q] = observe(hrow + gs);
                stt[q] = wave == NW - 1 ? observe(srow + gs) : 0ull;
            }
            for (unsigned polls = 0;; ++polls) {
                bool again = false;
#pragma unroll
                for (int q = 0; q < HPL; ++q) {
                    const int g = lane + kWave * q;
                    const bool real_g = g < G;
#pragma unroll
                    for (int j = 0; j < TPW; ++j) {
                        const int t = wave + j * NW;
                        if (real_g && t < k && ent[j][q] == kMailEmpty) {
                            ent[j][q] = observe(mb.rec + mail_rec_index(m, t, g));
                            again = true;
                        }
                    }
                    if (real_g && head[q] == kMailEmpty) {
                        head[q] = observe(hrow + g);
                        again = true;
                    }
                    if (real_g && stt[q] == kMailEmpty) {
                        stt[q] = observe(srow + g);
                        again = true;
                    }
                }
                if (!__any(again)) break;
                if (polls > spin_limit) {
                    if (lane == 0) {
                        __hip_atomic_store(error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        ms->timed_out = 1u;
                    }
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }

            // ---- the bound (every fetching wavefront computes the same one).  Maxima are
            // taken as floats (a NaN head just does not take part) and ordered as keys.
            float lmax = kNegInf;
#pragma unroll
            for (int q = 0; q < HPL; ++q) lmax = fmaxf(lmax, lane + kWave * q < G ? mail_hi(head[q]) : kNegInf);
            // (from k = 11 on 32 groups, {g : g mod 32 = j})
            unsigned gm = max_xor32_u32(key_hi_of(lmax));
            const float bound = value_of_key_hi(B32 ? half32_kth_largest_u32(gm, k)
                                                        : row16_kth_largest_u32(max_xor16_u32(gm), k));

            // ---- survivors among this wavefront's entries: not below the bound (a NaN
            // is not below anything, and ranks first like in the key order).  First all
            // the survivor masks, then ONE reservation of LDS slots for the wavefront, then
            // the few registers that hold a survivor are written out.
            unsigned long long mk[TPW][HPL];
            unsigned total = 0u;
#pragma unroll
            for (int j = 0; j < TPW; ++j)
#pragma unroll
                for (int q = 0; q < HPL; ++q) {
                    const int id = (int)(unsigned)ent[j][q];
                    const float v = mail_hi(ent[j][q]);
                    const bool real = (wave + j * NW < k) && (lane + kWave * q < G) && id != INT_MAX && id != -1;
                    mk[j][q] = __ballot(real && !(v < bound));
                    total += (unsigned)__popcll(mk[j][q]);
                }
            if (total != 0u) {
                unsigned base = 0u;
                if (lane == 0) base = atomicAdd(&ms->count, total);
                int at = __builtin_amdgcn_readfirstlane((int)base);
#pragma unroll
                for (int j = 0; j < TPW; ++j)
#pragma unroll
                    for (int q = 0; q < HPL; ++q) {
                        const unsigned long long m1 = mk[j][q];
                        if (m1 != 0ull) {
                            const int pos = at + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m1 >> 32),
                                                                                __builtin_amdgcn_mbcnt_lo((unsigned)m1, 0u));
                            if (((m1 >> lane) & 1ull) && pos < kWave)
                                ms->key[pos] = make_key(key_hi_of(mail_hi(ent[j][q])), ~(unsigned)ent[j][q]);
                            at += (int)__popcll(m1);
                        }
                    }
            }
            if (wave == NW - 1) {
                // log Z = mx + log sum_g S_g exp(mx_g - mx)
                float mxs[HPL], Ss[HPL];
                float lmx = kNegInf;
#pragma unroll
                for (int q = 0; q < HPL; ++q) {
                    const bool ok = lane + kWave * q < G;
                    mxs[q] = ok ? mail_hi(stt[q]) : kNegInf;
                    Ss[q] = ok ? mail_lo_f32(stt[q]) : 0.0f;
                    lmx = fmaxf(lmx, mxs[q]);
                }
                const float mx = wave_max_f32(lmx);
                float part = 0.0f;
#pragma unroll
                for (int q = 0; q < HPL; ++q) part += Ss[q] * exp_diff(mxs[q], mx);
                const float logZ = mx + __logf(wave_sum_f32(part));
                if (lane == 0) ms->logZ = logZ;
            }
        }
        __syncthreads();
        if (ms->timed_out != 0u) {
            // A wait ran out: this row has no result (and the records that may still arrive stay
            // in the mailbox: the workspace has to be prepared again before its next use).
            if (wave == 0) {
                write_no_result(m, M, M, k, token_ids, logp);
                if (step_rec && lane < k) publish(step_rec + m * kMailK + lane, mail_pack(kNegInf, (unsigned)INT_MAX));
            }
            __syncthreads();   // (every wavefront has read the flag before the next row resets it)
            continue;
        }

        // Every fetching wavefront has its records in registers: they are emptied for the next
        // call by all wavefronts but the first, which ranks and writes the outputs meanwhile
        // (emptying needs the addresses only, so the wavefronts that fetched nothing help).
        {
            const int helpers = (int)blockDim.x / kWave - 1;
            if (wave > 0) {
                for (int t = wave - 1; t < k; t += helpers)
#pragma unroll
                    for (int q = 0; q < HPL; ++q)
                        if (lane + kWave * q < G) publish(mb.rec + mail_rec_index(m, t, lane + kWave * q), kMailEmpty);
                if (wave == helpers)
#pragma unroll
                    for (int q = 0; q < HPL; ++q)
                        if (lane + kWave * q < G) publish(mb.st + mail_st_index(m, lane + kWave * q), kMailEmpty);
            }
        }

        const int n = __builtin_amdgcn_readfirstlane((int)ms->count);
        if (n <= kWave) {
            if (wave == 0) {
                const unsigned long long mine = ms->key[lane];
                const float logZ = ms->logZ;
                const u64x2 *kp = reinterpret_cast<const u64x2 *>(ms->key);
                int rank = 0;
#pragma unroll 4
                for (int j = 0; j < n; j += 2) {
                    const u64x2 two = kp[j >> 1];
                    rank += two.x > mine;
                    rank += two.y > mine;
                }
                if (mine != 0ull && rank < k) {
                    const int tok = (int)~(unsigned)mine;
                    const float lp = value_of_key_hi((unsigned)(mine >> 32)) - logZ;
                    token_ids[(size_t)m * k + rank] = tok;
                    logp[(size_t)m * k + rank] = lp;
                    if (step_rec) publish(step_rec + m * kMailK + rank, mail_pack(lp, (unsigned)tok));
                }
                if (lane >= n && lane < k) {   // fewer candidates than k in the whole subset
                    token_ids[(size_t)m * k + lane] = INT_MAX;
                    logp[(size_t)m * k + lane] = kNegInf;
                    if (step_rec) publish(step_rec + m * kMailK + lane, mail_pack(kNegInf, (unsigned)INT_MAX));
                }
            }
        } else {
            // Too many survivors (heavily tied values): hand the row to the general merge
            // through the plain partial arrays.
            if (wave < NW) {
#pragma unroll
                for (int q = 0; q < HPL; ++q) {
                    const int g = lane + kWave * q;
                    if (g < G) {
#pragma unroll
                        for (int j = 0; j < TPW; ++j) {
                            const int t = wave + j * NW;
                            if (t < k) {
                                publish(P.val + part_index(m * k + t, g), mail_hi(ent[j][q]));
                                publish(P.id + part_index(m * k + t, g), (int)(unsigned)ent[j][q]);
                            }
                        }
                        if (wave == NW - 1) {
                            publish(P.ms + part_index(m * 2, g), mail_hi(stt[q]));
                            publish(P.ms + part_index(m * 2 + 1, g), mail_lo_f32(stt[q]));
                        }
                    }
                }
            }
            wait_stores_done();
            __syncthreads();
            if (wave == 0) {
                final_merge_general(P, G, m, M, M, k, token_ids, logp, sc);   // this row only
                if (step_rec) {   // hand the row on from where the general merge wrote it
                    wait_stores_done();
                    if (lane < k)
                        publish(step_rec + m * kMailK + lane,
                                mail_pack(observe(logp + (size_t)m * k + lane),
                                          (unsigned)observe(token_ids + (size_t)m * k + lane)));
                }
            }
        }
    }
}

}  // namespace frspec
