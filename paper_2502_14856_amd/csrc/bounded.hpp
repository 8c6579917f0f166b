// The bounded end of the skinny kernel's single-launch path (k <= 16, at most 256 workgroups,
// every workgroup with at least two passes).
//
// After a workgroup's last pass three things stand between the end of its stream and the
// outputs: its fold, the trip of its records to the merging workgroups, and their merge.  Both
// the fold and the merge are long chains of dependent instructions, and nearly all of their
// work is spent on logits that cannot end up among the k best of the row: with 256 workgroups a
// workgroup's k best hold 0.04 winners on average.  So the work is moved ahead of the last pass:
//   * a workgroup publishes the k best of all its passes but the last (the "early list") at the
//     start of its last pass, long before the end of the kernel;
//   * one group of steps before the end of its stream a wavefront fetches the heads of all early
//     lists of its two rows of H and takes the k-th largest of 16 group maxima as the row's bound
//     (the bound of the fast selection, over other workgroups' results: k different groups
//     hold a logit at least that large, so nothing below it is among the k best of the row); a
//     list that is not there yet only weakens the bound;
//   * its last fold is the softmax statistics plus one comparison per logit: the few logits at
//     or above the bound (0.1 per workgroup and row in expectation) go out as they are, in up to
//     three slots beside the statistics record;
//   * the merging workgroup of a row ranks the early lists while the last workgroups still
//     stream; when the last statistics record arrives it only has to add the late survivors
//     that beat its k-th best so far, and the normaliser.
// A workgroup with more than three late survivors in a row writes the k best of its last pass
// as a second list and marks the row; the merger then takes the general merge over both lists
// of every workgroup.  Heavily tied logits end there too.  Outputs are bit for bit those of the
// unbounded path: the same statistics, summed in the same order, and the same key order.
#pragma once

#include "epilogue.hpp"

namespace frspec {

/*
 * Records of the bounded end, all in the mailbox's record array (8192 records per mailbox row):
 *   early[g][m][t]   rows 0 to 7, workgroup-major: the early list of workgroup g for row m of H
 *                    is 16 consecutive records, one 128-byte line
 *   head[m][g]       list position 4 of row 32 + m: the best entry of that list once more
 *   late[m][t][g]    rows 16 + m: the late lists of marked rows
 *   fin[m][s][g]     rows 32 + m, list positions 0 (statistics) and 1 to 3 (late survivors)
 * Why the early lists are workgroup-major: a store instruction to memory that the other compute
 * dies must see is sent line by line, about 80 ns per line it touches (measured: a store of 64
 * records to 64 lines takes 5 us longer than one to 4 lines), and a wavefront's loads do not
 * complete before the stores issued ahead of them.  An early list laid out like the final records
 * (one line per list position) costs the stream 1 to 1.5 us per workgroup; as two lines per
 * wavefront, plus two for the heads, next to nothing.  The heads are there once more, by workgroup
 * within a row, because every wavefront of the grid reads them: contiguous, they are 8 lines a row.
 */
constexpr int kLateRow0 = kMailLateRow0, kFinRow0 = kMailFinRow0, kBoundedMailRows = 48;
constexpr int kLateSlots = 3, kHeadSlot = 1 + kLateSlots;
constexpr int kEarlyRowsOfH = 16;                   // rows of H per workgroup in the early region
constexpr unsigned kMarkedId = 0x7FFFFFFEu;   // "see the late list" (never a token id: ids are < 2^31 - 2)
static_assert(4 * kWave * kEarlyRowsOfH * kMailK <= kLateRow0 * kMailK * kGridMax, "the early region ends before the late lists");

__device__ __forceinline__ unsigned long long *fin_record(const Mailbox &mb, int m, int slot, int g) {
    return mb.rec + mail_rec_index(kFinRow0 + m, slot, g);
}
__device__ __forceinline__ size_t early_index(int g, int m, int t) {
    return ((size_t)g * kEarlyRowsOfH + m) * kMailK + t;
}

/*
 * What a wavefront sends out at the start of the workgroup's last pass for its two rows of H, one
 * per half (lane (h, l32): row m = wave + 8h), from the running state that the previous fold left
 * in LDS: the early list (lanes l32 < 16: list position l32) and the head record (the other
 * lanes); the entries then leave the running list (they only compete once more if the last pass
 * has to write late lists).  EVERY lane stores, in one instruction: the kernel waits for its loads
 * of W by count (s_waitcnt vmcnt(N): "all but the N youngest have completed"), loads and stores
 * complete in order, and only a store in straight-line code is counted exactly by the compiler.
 * Lanes without an entry write an empty record where one is (a row of H that does not exist, a
 * list position past k).
 */
__device__ __forceinline__ void post_early_list(const Mailbox &mb, int wave, int M, int k, int g, float *run_val,
                                                int *run_id) {
    const int lane = lane_id(), l32 = lane & 31;
    const int m = wave + 8 * (lane >> 5);
    const int t = l32 < kMailK ? l32 : 0;
    const bool valid = m < M && t < k;
    const int at = valid ? m * k + t : 0;
    const float v = run_val[at];
    const int id = run_id[at];
    const size_t to = l32 < kMailK ? early_index(g, m, t) : mail_rec_index(kFinRow0 + m, kHeadSlot, g);
    publish(mb.rec + to, valid ? mail_pack(v, (unsigned)id) : kMailEmpty);
    if (valid && l32 < kMailK) {
        run_val[at] = kNegInf;
        run_id[at] = INT_MAX;
    }
}

// The head records of row m, four per lane (workgroups lane, lane + 64, ...): the high word of a
// record is the logit, all ones while the record is empty.
__device__ __forceinline__ void request_heads(const Mailbox &mb, int m, int G, unsigned (&w)[4]) {
    const int lane = lane_id();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int g = lane + kWave * q, gs = g < G ? g : G - 1;
        w[q] = observe(reinterpret_cast<const unsigned *>(fin_record(mb, m, kHeadSlot, gs)) + 1);
    }
}

// The bound from those heads, as the high word of a key, the same in every lane: the k-th largest
// of the 16 maxima over the groups {g : (g mod 64) / 4 = j}.  A group holds workgroups of four
// compute dies (workgroup g runs on die g mod 8): the dies do not keep the same pace, and with
// groups of one die each the workgroups of the slow dies, whose records are the ones that may
// still be missing, would empty whole groups.  An empty record, a list without entries and a
// NaN do not take part; with fewer than k populated groups the bound admits everything.
__device__ __forceinline__ unsigned bound_from_heads(const unsigned (&w)[4], int G, int k) {
    const int lane = lane_id();
    float lmax = kNegInf;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const bool there = lane + kWave * q < G && w[q] != 0xFFFFFFFFu;
        lmax = fmaxf(lmax, there ? __builtin_bit_cast(float, w[q]) : kNegInf);
    }
    unsigned qm = key_hi_of(lmax);
    qm = max(qm, (unsigned)dpp_i32<kDppQuadXor1>((int)qm));
    qm = max(qm, (unsigned)dpp_i32<kDppQuadXor2>((int)qm));
    int greater = 0;   // quads whose maximum is strictly larger than this lane's quad maximum
#pragma unroll
    for (int q = 0; q < 16; ++q) greater += (unsigned)__builtin_amdgcn_readlane((int)qm, 4 * q) > qm;
    // the smallest quad maximum that still is among the k largest = the k-th largest
    return wave_min_u32(greater <= k - 1 ? qm : 0xFFFFFFFFu);
}

/*
 * The last fold of a workgroup under a bound, TWO rows of H per wavefront as in fold_pair_fast
 * (lane (h, l32): row `m`, C = ZR_MAX / 32 consecutive local vocabulary rows): the statistics of
 * the pass are folded into the running ones (run_ms, in LDS) and written as the row's final
 * statistics record; the logits at or above `bound` (high word of a key, this lane's row's) go to
 * the late slots.  Returns false, having written nothing, when a row has more than kLateSlots of
 * them: the caller then writes late lists for both rows.
 */
template <int ZR_MAX>
__device__ __forceinline__ bool fold_pair_bounded(const float *z_lds, int z_row_stride, int KS, int z_slice_stride,
                                                  const int *ids_pass, int n_valid, int m, bool active,
                                                  unsigned bound, const float *run_ms, const Mailbox &mail, int g) {
    constexpr int C = ZR_MAX / 32;
    const int lane = lane_id(), h = lane >> 5, l32 = lane & 31;
    const int mm = active ? m : 0;

    float z[C];
#pragma unroll
    for (int c = 0; c < C; ++c) z[c] = 0.0f;
    const float *zp = z_lds + mm * z_row_stride + l32 * C;
    for (int q = 0; q < KS; ++q) {
        float t[C];
        lds_words<C, float, fvec4, fvec2>(zp + q * z_slice_stride, t);
#pragma unroll
        for (int c = 0; c < C; ++c) z[c] += t[c];
    }
    int id[C];
    lds_words<C, int, ivec4, ivec2>(ids_pass + l32 * C, id);
    const float old_mx = run_ms[2 * mm], old_S = run_ms[2 * mm + 1];

    // the statistics, exactly as the unbounded fold takes them
    float v[C];
    bool ok[C];
    float lmax = kNegInf;
#pragma unroll
    for (int c = 0; c < C; ++c) {
        ok[c] = active && (l32 * C + c < n_valid);
        v[c] = ok[c] ? z[c] : kNegInf;
        lmax = fmaxf(lmax, v[c]);
    }
    const float mx = fmaxf(old_mx, row16_max_f32(max_xor16_f32(lmax)));
    float part = 0.0f;
#pragma unroll
    for (int c = 0; c < C; ++c) part += exp_diff(v[c], mx);
    part = sum_xor16_f32(part);
    const float S = old_S * exp_diff(old_mx, mx) + row16_sum_all(part);

    // the late survivors of each half, in the order of their lanes
    bool sv[C];
    int pos[C];
    int n0 = 0, n1 = 0;
#pragma unroll
    for (int c = 0; c < C; ++c) {
        sv[c] = ok[c] && key_hi_of(v[c]) >= bound;
        const unsigned long long mask = __ballot(sv[c]);
        const int c_lo = __popc((unsigned)mask), c_hi = __popc((unsigned)(mask >> 32));
        const int before = (int)__builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32),
                                                          __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u));
        pos[c] = h ? before - c_lo + n1 : before + n0;
        n0 += c_lo;
        n1 += c_hi;
    }
    if (n0 > kLateSlots || n1 > kLateSlots) return false;
    if (active) {
        const int n_h = h ? n1 : n0;
#pragma unroll
        for (int c = 0; c < C; ++c)
            if (sv[c]) publish(fin_record(mail, m, 1 + pos[c], g), mail_pack(v[c], (unsigned)id[c]));
        if (l32 >= n_h && l32 < kLateSlots) publish(fin_record(mail, m, 1 + l32, g), mail_pack(kNegInf, (unsigned)INT_MAX));
        if (l32 == 0) publish(fin_record(mail, m, 0, g), mail_pack_stats(mx, S));
    }
    return true;
}

// Marks rows m (one per half of the wavefront) as "see the late list": position 1 carries the
// mark, the other late slots are written as unused.
__device__ __forceinline__ void mark_rows_late(const Mailbox &mail, int m, bool active, int g) {
    const int l32 = lane_id() & 31;
    if (active && l32 < kLateSlots)
        publish(fin_record(mail, m, 1 + l32, g), mail_pack(kNegInf, l32 == 0 ? kMarkedId : (unsigned)INT_MAX));
}

// Scratch of the bounded merge, one per workgroup.
struct alignas(16) BoundedScratch {
    unsigned long long cand[kWave];   // the k best of the early lists at [0, k), late survivors behind them
    unsigned count;                   // late survivors so far
    unsigned marked;                  // some workgroup wrote a late list for this row
};

/*
 * A workgroup of eight wavefronts merges rows first, first + stride, ... of H (G <= 256, k <= 16).
 * First the early lists, as merge_rows_mailbox merges its records (fetch until none is empty,
 * bound from the heads, survivors to LDS, ranking), but only as far as the k best so far.  Then
 * the final records: six wavefronts fetch the three late slots of all workgroups, the last one
 * the statistics; late survivors that beat the k-th best so far join the k best in LDS, and the
 * first wavefront ranks the two dozen keys and writes the outputs while the others empty the
 * records.  A marked row, more than 64 early survivors or more late survivors than fit go to the
 * general merge through the plain partial arrays: workgroup g's early list in slot g, its late
 * list (or its sorted late survivors) in slot G + g.
 */
__device__ __forceinline__ void merge_rows_bounded(const Mailbox &mb, const Partials &P, unsigned *error, int G,
                                                   int first, int stride, int M, int k, int *token_ids, float *logp,
                                                   MergeScratch *ms, BoundedScratch *bs, SelectScratch *sc,
                                                   unsigned long long *step_rec, unsigned spin_limit,
                                                   long long *trace = nullptr) {
    constexpr int NW = 8, HPL = 4;
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x / kWave);
    for (int m = first; m < M; m += stride) {
        if (wave == 0) {
            ms->key[lane] = 0ull;
            bs->cand[lane] = 0ull;
            if (lane == 0) {
                ms->count = 0u;
                ms->timed_out = 0u;
                bs->count = 0u;
                bs->marked = 0u;
            }
        }
        __syncthreads();
        // ---- the early lists: fetch until no record is empty, bound, survivors.  A quarter of a
        // wavefront fetches the 16 list positions of one workgroup (one line), a wavefront those of
        // 32 workgroups in eight loads; every wavefront also fetches all heads, for the bound.
        {
            constexpr int LPW = 8;   // loads per wavefront: 4 workgroups each
            unsigned long long ent[LPW], head[HPL];
            const int t = lane & (kMailK - 1);
            const unsigned long long *hrow = fin_record(mb, m, kHeadSlot, 0);
            int ge[LPW];
#pragma unroll
            for (int j = 0; j < LPW; ++j) {
                ge[j] = 32 * wave + 4 * j + (lane >> 4);
                ent[j] = observe(mb.rec + early_index(ge[j] < G ? ge[j] : G - 1, m, t));
            }
#pragma unroll
            for (int q = 0; q < HPL; ++q) {
                const int g = lane + kWave * q;
                head[q] = observe(hrow + (g < G ? g : G - 1));
            }
            for (unsigned polls = 0;; ++polls) {
                bool again = false;
#pragma unroll
                for (int j = 0; j < LPW; ++j)
                    if (ge[j] < G && t < k && ent[j] == kMailEmpty) {
                        ent[j] = observe(mb.rec + early_index(ge[j], m, t));
                        again = true;
                    }
#pragma unroll
                for (int q = 0; q < HPL; ++q)
                    if (lane + kWave * q < G && head[q] == kMailEmpty) {
                        head[q] = observe(hrow + lane + kWave * q);
                        again = true;
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
            float lmax = kNegInf;
#pragma unroll
            for (int q = 0; q < HPL; ++q) lmax = fmaxf(lmax, lane + kWave * q < G ? mail_hi(head[q]) : kNegInf);
            unsigned gm = key_hi_of(lmax);
            gm = max_xor16_u32(gm);
            gm = max_xor32_u32(gm);
            const float bound = value_of_key_hi(row16_kth_largest_u32(gm, k));
            unsigned long long mk[LPW];
            unsigned total = 0u;
#pragma unroll
            for (int j = 0; j < LPW; ++j) {
                const int id = (int)(unsigned)ent[j];
                const float v = mail_hi(ent[j]);
                const bool real = t < k && ge[j] < G && id != INT_MAX && id != -1;
                mk[j] = __ballot(real && !(v < bound));
                total += (unsigned)__popcll(mk[j]);
            }
            if (total != 0u) {
                unsigned base = 0u;
                if (lane == 0) base = atomicAdd(&ms->count, total);
                int at = __builtin_amdgcn_readfirstlane((int)base);
#pragma unroll
                for (int j = 0; j < LPW; ++j) {
                    const unsigned long long m1 = mk[j];
                    if (m1 != 0ull) {
                        const int pos = at + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m1 >> 32),
                                                                            __builtin_amdgcn_mbcnt_lo((unsigned)m1, 0u));
                        if (((m1 >> lane) & 1ull) && pos < kWave)
                            ms->key[pos] = make_key(key_hi_of(mail_hi(ent[j])), ~(unsigned)ent[j]);
                        at += (int)__popcll(m1);
                    }
                }
            }
        }
        __syncthreads();
        const int n_early = __builtin_amdgcn_readfirstlane((int)ms->count);
        if (wave == 0 && n_early <= kWave) {
            const unsigned long long mine = ms->key[lane];
            const u64x2 *kp = reinterpret_cast<const u64x2 *>(ms->key);
            int rank = 0;
#pragma unroll 4
            for (int j = 0; j < n_early; j += 2) {
                const u64x2 two = kp[j >> 1];
                rank += two.x > mine;
                rank += two.y > mine;
            }
            if (mine != 0ull && rank < k) bs->cand[rank] = mine;
        }
        __syncthreads();
        if (trace && threadIdx.x == 0) trace[6] = (long long)__builtin_amdgcn_s_memrealtime();

        // ---- the final records
        if (ms->timed_out == 0u) {
            if (wave < 6) {
                const unsigned long long kth = bs->cand[k - 1];   // zero while fewer than k so far
                const int slot = 1 + (wave >> 1);
                const unsigned long long *row = fin_record(mb, m, slot, 0);
                unsigned long long rc[2];
                int g2[2];
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    g2[q] = lane + kWave * (2 * (wave & 1) + q);
                    rc[q] = observe(row + (g2[q] < G ? g2[q] : G - 1));
                }
                for (unsigned polls = 0;; ++polls) {
                    bool again = false;
#pragma unroll
                    for (int q = 0; q < 2; ++q)
                        if (g2[q] < G && rc[q] == kMailEmpty) {
                            rc[q] = observe(row + g2[q]);
                            again = true;
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
                unsigned long long key[2], mk[2];
                unsigned total = 0u;
                bool mark = false;
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const unsigned id = (unsigned)rc[q];
                    const bool there = g2[q] < G && rc[q] != kMailEmpty;
                    mark = mark || (there && id == kMarkedId);
                    key[q] = make_key(key_hi_of(mail_hi(rc[q])), ~id);
                    mk[q] = __ballot(there && id != (unsigned)INT_MAX && id != kMarkedId && key[q] > kth);
                    total += (unsigned)__popcll(mk[q]);
                }
                if (__any(mark) && lane == 0) bs->marked = 1u;
                if (total != 0u) {
                    unsigned base = 0u;
                    if (lane == 0) base = atomicAdd(&bs->count, total);
                    int at = k + __builtin_amdgcn_readfirstlane((int)base);
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        const int pos = at + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(mk[q] >> 32),
                                                                            __builtin_amdgcn_mbcnt_lo((unsigned)mk[q], 0u));
                        if (((mk[q] >> lane) & 1ull) && pos < kWave) bs->cand[pos] = key[q];
                        at += (int)__popcll(mk[q]);
                    }
                }
            } else if (wave == NW - 1) {
                // log Z = mx + log sum_g S_g exp(mx_g - mx), as the unbounded merge sums it
                const unsigned long long *srow = fin_record(mb, m, 0, 0);
                unsigned long long stt[HPL];
#pragma unroll
                for (int q = 0; q < HPL; ++q) {
                    const int g = lane + kWave * q;
                    stt[q] = observe(srow + (g < G ? g : G - 1));
                }
                for (unsigned polls = 0;; ++polls) {
                    bool again = false;
#pragma unroll
                    for (int q = 0; q < HPL; ++q)
                        if (lane + kWave * q < G && stt[q] == kMailEmpty) {
                            stt[q] = observe(srow + lane + kWave * q);
                            again = true;
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
        if (trace && threadIdx.x == 0) trace[7] = (long long)__builtin_amdgcn_s_memrealtime();
        if (ms->timed_out != 0u) {
            // A wait ran out: this row has no result (and records that may still arrive stay in the
            // mailbox: the workspace has to be prepared again before its next use).
            if (wave == 0) {
                write_no_result(m, M, M, k, token_ids, logp);
                if (step_rec && lane < k) publish(step_rec + m * kMailK + lane, mail_pack(kNegInf, (unsigned)INT_MAX));
            }
            __syncthreads();
            continue;
        }

        const int n_late = __builtin_amdgcn_readfirstlane((int)bs->count);
        const bool general = bs->marked != 0u || n_early > kWave || k + n_late > kWave;
        if (!general) {
            if (wave == 0) {
                const unsigned long long mine = bs->cand[lane];
                const float logZ = ms->logZ;
                const u64x2 *kp = reinterpret_cast<const u64x2 *>(bs->cand);
                const int n = k + n_late;
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
                const int real = (int)__popcll(__ballot(mine != 0ull));
                if (lane >= real && lane < k) {   // fewer candidates than k in the whole subset
                    token_ids[(size_t)m * k + lane] = INT_MAX;
                    logp[(size_t)m * k + lane] = kNegInf;
                    if (step_rec) publish(step_rec + m * kMailK + lane, mail_pack(kNegInf, (unsigned)INT_MAX));
                }
            }
        } else {
            // The lists of the general merge.  With the early lists ranked (and emptied): their k
            // best in slot 0, workgroup g's late list and statistics in slot 1 + g.  Otherwise
            // (more than 64 early survivors): workgroup g's early list and statistics in slot g,
            // its late list in slot G + g.
            const int tid = (int)threadIdx.x;
            const bool ranked = n_early <= kWave;
            const int late0 = ranked ? 1 : G;
            if (ranked && tid < k) {
                const unsigned long long kk = bs->cand[tid];
                publish(P.val + part_index(m * k + tid, 0), kk != 0ull ? value_of_key_hi((unsigned)(kk >> 32)) : kNegInf);
                publish(P.id + part_index(m * k + tid, 0), kk != 0ull ? (int)~(unsigned)kk : INT_MAX);
                if (tid == 0) {
                    publish(P.ms + part_index(m * 2, 0), kNegInf);
                    publish(P.ms + part_index(m * 2 + 1, 0), 0.0f);
                }
            }
            if (!ranked && tid < G) {
                const int g = tid;
                for (int t = 0; t < k; ++t) {
                    const unsigned long long e = observe(mb.rec + early_index(g, m, t));
                    publish(P.val + part_index(m * k + t, g), mail_hi(e));
                    publish(P.id + part_index(m * k + t, g), (int)(unsigned)e);
                }
                const unsigned long long st = observe(fin_record(mb, m, 0, g));
                publish(P.ms + part_index(m * 2, g), mail_hi(st));
                publish(P.ms + part_index(m * 2 + 1, g), mail_lo_f32(st));
            } else if (tid >= 4 * kWave && tid - 4 * kWave < G) {
                const int g = tid - 4 * kWave;
                unsigned long long c[kLateSlots];
#pragma unroll
                for (int s = 0; s < kLateSlots; ++s) c[s] = observe(fin_record(mb, m, 1 + s, g));
                if ((unsigned)c[0] == kMarkedId) {
                    for (int t = 0; t < k; ++t) {
                        const unsigned long long *at = mb.rec + mail_rec_index(kLateRow0 + m, t, g);
                        unsigned long long e = observe(at);
                        for (unsigned polls = 0; e == kMailEmpty && polls <= spin_limit; ++polls) {
                            __builtin_amdgcn_s_sleep(1);
                            e = observe(at);
                        }
                        if (e == kMailEmpty) {
                            __hip_atomic_store(error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            e = mail_pack(kNegInf, (unsigned)INT_MAX);
                        }
                        publish(P.val + part_index(m * k + t, late0 + g), mail_hi(e));
                        publish(P.id + part_index(m * k + t, late0 + g), (int)(unsigned)e);
                    }
                } else {
                    // up to three survivors in lane order: sorted, best first (unused slots last)
                    unsigned long long key[kLateSlots];
#pragma unroll
                    for (int s = 0; s < kLateSlots; ++s)
                        key[s] = (unsigned)c[s] == (unsigned)INT_MAX ? 0ull
                                                                     : make_key(key_hi_of(mail_hi(c[s])), ~(unsigned)c[s]);
                    auto order = [&](int a, int b) {
                        if (key[b] > key[a]) {
                            const unsigned long long t = key[a];
                            key[a] = key[b];
                            key[b] = t;
                        }
                    };
                    order(0, 1);
                    order(1, 2);
                    order(0, 1);
                    for (int t = 0; t < k; ++t) {
                        const unsigned long long kk = t == 0 ? key[0] : t == 1 ? key[1] : t == 2 ? key[2] : 0ull;
                        publish(P.val + part_index(m * k + t, late0 + g),
                                kk != 0ull ? value_of_key_hi((unsigned)(kk >> 32)) : kNegInf);
                        publish(P.id + part_index(m * k + t, late0 + g), kk != 0ull ? (int)~(unsigned)kk : INT_MAX);
                    }
                }
                if (ranked) {
                    const unsigned long long st = observe(fin_record(mb, m, 0, g));
                    publish(P.ms + part_index(m * 2, late0 + g), mail_hi(st));
                    publish(P.ms + part_index(m * 2 + 1, late0 + g), mail_lo_f32(st));
                } else {
                    publish(P.ms + part_index(m * 2, late0 + g), kNegInf);
                    publish(P.ms + part_index(m * 2 + 1, late0 + g), 0.0f);
                }
            }
            wait_stores_done();
            __syncthreads();
            if (wave == 0) {
                if (lane == 0) atomicAdd(error + 1, 1u);   // statistics: rows that took the general merge
                final_merge_general(P, ranked ? G + 1 : 2 * G, m, M, M, k, token_ids, logp, sc);   // this row only
                if (step_rec) {   // hand the row on from where the general merge wrote it
                    wait_stores_done();
                    if (lane < k)
                        publish(step_rec + m * kMailK + lane,
                                mail_pack(observe(logp + (size_t)m * k + lane),
                                          (unsigned)observe(token_ids + (size_t)m * k + lane)));
                }
            }
        }
        // Everything of this row has been read: the records are emptied for the next call by all
        // wavefronts but the first (the late lists only where one was written): the early lists a
        // line (one workgroup) per quarter wavefront, the rest by list position.
        if (wave > 0) {
            const int helpers = NW - 1;
            for (int g0 = 4 * (wave - 1); g0 < G; g0 += 4 * helpers) {
                const int g = g0 + (lane >> 4);
                if (g < G) publish(mb.rec + early_index(g, m, lane & (kMailK - 1)), kMailEmpty);
            }
            constexpr int kFinUsed = 1 + kLateSlots + 1;   // statistics, late slots, head record
            const int positions = kFinUsed + (general ? k : 0);
            for (int t = wave - 1; t < positions; t += helpers) {
                const int row = t < kFinUsed ? kFinRow0 + m : kLateRow0 + m;
                const int at = t < kFinUsed ? t : t - kFinUsed;
#pragma unroll
                for (int q = 0; q < HPL; ++q)
                    if (lane + kWave * q < G) publish(mb.rec + mail_rec_index(row, at, lane + kWave * q), kMailEmpty);
            }
        }
    }
}

}  // namespace frspec
