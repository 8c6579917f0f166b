// Online log-softmax statistics, per-row top-k and the merge of per-workgroup partials.
//
// A workgroup owns a set of vocabulary rows.  For every row m of H it keeps, in LDS,
//   run_ms[m]  = (mx, S): running maximum of its logits and sum of exp(z - mx),
//   run_val/run_id[m][0..k): its k best (logit, token id) pairs, best first.
// At the end these go to the workspace; one wavefront per row m then merges the G
// workgroups' partials into log Z (Eq. 4's normaliser over the subset), the final k
// candidates, and writes token ids and log-probabilities.
#pragma once

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
// Blocks the wavefront until its outstanding stores have been acknowledged.
__device__ __forceinline__ void wait_stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Arrival words at the start of the workspace (all zero between calls).
struct Arrival {
    unsigned *ticket;   // workgroups that have published their partials
    unsigned *done;     // merging workgroups that have finished
    unsigned *error;    // sticky: set to 1 if a bounded wait ever ran out
};
constexpr int kMaxMergers = 32;          // far fewer than the workgroups resident at once
constexpr unsigned kSpinLimit = 1u << 22;   // polls of ~0.5 us each before giving up

/*
 * The merge of the partials is shared by the last R = min(G, M, kMaxMergers) workgroups
 * to arrive: workgroup number r of those merges rows r, r + R, ... of H.  One workgroup
 * merging every row would run M single-wavefront jobs on the four SIMDs of one compute
 * unit; spread over R compute units the jobs run side by side.
 *
 * Every thread of a workgroup calls this after publishing its partials.  Returns -1 in
 * workgroups that are not among the last R (they are finished), else r, after all G
 * workgroups have arrived.  The wait is on workgroups that are already running and need
 * nothing from the waiters, and at most kMaxMergers workgroups ever wait, so it cannot
 * starve a workgroup that has not been scheduled yet; it is bounded all the same.
 */
__device__ __forceinline__ int arrive_and_wait(const Arrival &ar, int G, int R, int *s_slot) {
    wait_stores_done();
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned a = __hip_atomic_fetch_add(ar.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int r = (int)a - (G - R);
        if (r >= 0) {
            unsigned polls = 0;
            while (__hip_atomic_load(ar.ticket, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < (unsigned)G) {
                __builtin_amdgcn_s_sleep(4);
                if (++polls > kSpinLimit) {
                    __hip_atomic_store(ar.error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
            }
        }
        *s_slot = r;
    }
    __syncthreads();
    return *s_slot;
}

// Called by every thread of a merging workgroup when its rows are written; the last
// merger to finish clears the arrival words for the next call.
__device__ __forceinline__ void merger_done(const Arrival &ar, int R) {
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned d = __hip_atomic_fetch_add(ar.done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (d == (unsigned)(R - 1)) {
            __hip_atomic_store(ar.done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(ar.ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
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

// Folds rows m = first, first + stride, ... < M of H, two at a time where possible.
template <int ZR, bool WITH_RUN, typename RowOf>
__device__ __forceinline__ void block_fold_all(int first, int stride, int M, RowOf row_of, int KS,
                                               int z_slice_stride, const int *ids_pass, int n_valid,
                                               int k, SelectScratch *sc) {
    int m = first;
    for (; m + stride < M; m += 2 * stride) {
        const FoldRow rows[2] = {row_of(m), row_of(m + stride)};
        block_fold_rows<ZR, 2, WITH_RUN>(rows, KS, z_slice_stride, ids_pass, n_valid, k, sc);
    }
    if (m < M) {
        const FoldRow rows[1] = {row_of(m)};
        block_fold_rows<ZR, 1, WITH_RUN>(rows, KS, z_slice_stride, ids_pass, n_valid, k, sc);
    }
}

/*
 * One wavefront merges the G partial results of NS rows of H and writes their outputs.
 * Every partial list is sorted, so the k best overall lie in the k lists with the best
 * heads, and list number i (by head) can contribute at most k - i entries: the search
 * space shrinks from G*k to k(k+1)/2 candidates.  HPL = ceil(G / 64) heads per lane.
 */
#ifdef FRSPEC_MERGE_TRACE
#define FRSPEC_MERGE_STAMP(i) \
    do { if (lane_id() == 0) FRSPEC_MERGE_TRACE[i] = (long long)__builtin_readcyclecounter(); } while (0)
#else
#define FRSPEC_MERGE_STAMP(i) do { } while (0)
#endif

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
    FRSPEC_MERGE_STAMP(0);
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
    FRSPEC_MERGE_STAMP(1);
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
        FRSPEC_MERGE_STAMP(2);

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
                FRSPEC_MERGE_STAMP(3);
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
                FRSPEC_MERGE_STAMP(3);
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
        FRSPEC_MERGE_STAMP(4);
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

}  // namespace frspec
