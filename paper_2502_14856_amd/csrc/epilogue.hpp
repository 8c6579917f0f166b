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

// Arrival of one workgroup (all its threads call this after publishing its partials);
// returns true in every thread of the last workgroup to arrive.
__device__ __forceinline__ bool arrive_is_last(unsigned *ticket, int G, int *s_flag) {
    wait_stores_done();
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned old = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *s_flag = (old == (unsigned)(G - 1));
    }
    __syncthreads();
    return *s_flag != 0;
}
__device__ __forceinline__ void reset_ticket(unsigned *ticket) {
    __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
                                                const int *ids_pass, int n_valid, int k) {
    constexpr int CP = ZR / kWave;
    constexpr int CPL = CP + (WITH_RUN ? 1 : 0);
    static_assert(ZR % kWave == 0, "pass rows must be a multiple of the wave size");
    const int lane = lane_id();
    float v[NS][CPL];
    int id[NS][CPL], pl[NS][CPL];
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
            pl[s][CPL - 1] = 0;
        }
    }
    float ov[NS];
    int oid[NS], opl[NS];
    wave_select_topk<NS, CPL>(v, id, pl, k, ov, oid, opl);
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        if (lane < k) {
            row[s].run_val[lane] = ov[s];
            row[s].run_id[lane] = oid[s];
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
                                               int k) {
    int m = first;
    for (; m + stride < M; m += 2 * stride) {
        const FoldRow rows[2] = {row_of(m), row_of(m + stride)};
        block_fold_rows<ZR, 2, WITH_RUN>(rows, KS, z_slice_stride, ids_pass, n_valid, k);
    }
    if (m < M) {
        const FoldRow rows[1] = {row_of(m)};
        block_fold_rows<ZR, 1, WITH_RUN>(rows, KS, z_slice_stride, ids_pass, n_valid, k);
    }
}

/*
 * One wavefront merges the G partial results of NS rows of H and writes their outputs.
 * Every partial list is sorted, so the k best overall lie in the k lists with the best
 * heads, and list number i (by head) can contribute at most k - i entries: the search
 * space shrinks from G*k to k(k+1)/2 candidates.  HPL = ceil(G / 64) heads per lane.
 */
template <int NS, int HPL>
__device__ __forceinline__ void final_merge_rows(const Partials &P, int G, const int (&m)[NS], int k,
                                                 int *token_ids, float *logp) {
    const int lane = lane_id();
    float hv[NS][HPL];
    int hid[NS][HPL], hg[NS][HPL];
    float logZ[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        // log Z = mx + log sum_g S_g exp(mx_g - mx)
        float mxs[HPL], Ss[HPL];
        float lmx = kNegInf;
#pragma unroll
        for (int q = 0; q < HPL; ++q) {
            const int g = lane + kWave * q;
            const bool ok = g < G;
            const int gs = ok ? g : 0;
            mxs[q] = ok ? observe(P.ms + part_index(m[s] * 2, gs)) : kNegInf;
            Ss[q] = ok ? observe(P.ms + part_index(m[s] * 2 + 1, gs)) : 0.0f;
            hv[s][q] = ok ? observe(P.val + part_index(m[s] * k, gs)) : kNegInf;
            hid[s][q] = ok ? observe(P.id + part_index(m[s] * k, gs)) : INT_MAX;
            hg[s][q] = ok ? g : -1;
            lmx = fmaxf(lmx, mxs[q]);
        }
        const float mx = wave_max_f32(lmx);
        float part = 0.0f;
#pragma unroll
        for (int q = 0; q < HPL; ++q) part += Ss[q] * exp_diff(mxs[q], mx);
        logZ[s] = mx + __logf(wave_sum_f32(part));
    }

    // the k lists with the best heads; lane i learns the workgroup of list number i
    float lv[NS];
    int lid[NS], lg[NS];
    wave_select_topk<NS, HPL>(hv, hid, hg, k, lv, lid, lg);

    // candidates (i, t), i + t < k, enumerated row by row of the triangle
    const int n_cand = k * (k + 1) / 2;
    float ov[NS];
    int oid[NS], opl[NS];
    auto fetch = [&](int s, int c, float &cv, int &cid) {
        // triangle row i starts at offset i*k - i(i-1)/2
        int i = 0, off = 0;
        while (i + 1 < k && off + (k - i) <= c) {
            off += k - i;
            ++i;
        }
        const int t = c - off;
        const int g = __shfl(lg[s], i);
        const bool ok = (c < n_cand) && (g >= 0) && (g < G);
        const size_t at = part_index(m[s] * k + (ok ? t : 0), ok ? g : 0);
        cv = ok ? observe(P.val + at) : kNegInf;
        cid = ok ? observe(P.id + at) : INT_MAX;
    };
    if (n_cand <= kWave) {
        float v[NS][1];
        int id[NS][1], pl[NS][1];
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            fetch(s, lane, v[s][0], id[s][0]);
            pl[s][0] = 0;
        }
        wave_select_topk<NS, 1>(v, id, pl, k, ov, oid, opl);
    } else if (n_cand <= 4 * kWave) {
        float v[NS][4];
        int id[NS][4], pl[NS][4];
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                fetch(s, lane + kWave * q, v[s][q], id[s][q]);
                pl[s][q] = 0;
            }
        wave_select_topk<NS, 4>(v, id, pl, k, ov, oid, opl);
    } else {
        // Large k: the candidates stay in memory.  Round j picks the best candidate that
        // is strictly after the previous winner in the (value, id) order; ids are
        // distinct, so this walks the sorted order without marking anything.
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            ov[s] = kNegInf;
            oid[s] = INT_MAX;
            float pv = __builtin_huge_valf();
            int pid = -1;
            for (int j = 0; j < k; ++j) {
                float bv = kNegInf;
                int bi = INT_MAX;
                for (int q = 0; q * kWave < n_cand; ++q) {   // uniform trip count: fetch shuffles
                    float cv;
                    int cid;
                    fetch(s, lane + kWave * q, cv, cid);
                    const bool after_prev = cand_before(pv, pid, cv, cid);
                    if (after_prev && cand_before(cv, cid, bv, bi)) {
                        bv = cv;
                        bi = cid;
                    }
                }
                const float wmax = wave_max_f32(bv);
                const int wid = wave_min_i32(bv == wmax ? bi : INT_MAX);
                if (lane == j) {
                    ov[s] = wmax;
                    oid[s] = wid;
                }
                pv = wmax;
                pid = wid;
            }
        }
    }
#pragma unroll
    for (int s = 0; s < NS; ++s)
        if (lane < k) {
            token_ids[(size_t)m[s] * k + lane] = oid[s];
            logp[(size_t)m[s] * k + lane] = ov[s] - logZ[s];
        }
}

template <int NS>
__device__ __forceinline__ void final_merge_dispatch(const Partials &P, int G, const int (&m)[NS],
                                                     int k, int *token_ids, float *logp) {
    if (G <= kWave) final_merge_rows<NS, 1>(P, G, m, k, token_ids, logp);
    else if (G <= 2 * kWave) final_merge_rows<NS, 2>(P, G, m, k, token_ids, logp);
    else if (G <= 4 * kWave) final_merge_rows<NS, 4>(P, G, m, k, token_ids, logp);
    else final_merge_rows<NS, kHeadsPerLane>(P, G, m, k, token_ids, logp);
}

// Merges rows m = first, first + stride, ... < M, two at a time where possible.
__device__ inline void final_merge_all(const Partials &P, int G, int first, int stride, int M, int k,
                                       int *token_ids, float *logp) {
    int m = first;
    for (; m + stride < M; m += 2 * stride) {
        const int ms[2] = {m, m + stride};
        final_merge_dispatch<2>(P, G, ms, k, token_ids, logp);
    }
    if (m < M) {
        const int ms[1] = {m};
        final_merge_dispatch<1>(P, G, ms, k, token_ids, logp);
    }
}

}  // namespace frspec
