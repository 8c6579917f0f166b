// Two-phase end of the skinny kernel's single-pass case (every workgroup streams its rows
// once: the compressed head of Eq. 4 at V_sub <= 128 rows x compute units).
//
// Inside a compute unit the older wavefront of each SIMD streams ahead of the younger one: the
// first four wavefronts of a workgroup (the first half of its rows) are done when the other
// four still have about a third of their bytes to go.  That idle time is used:
//   phase 1  the four early wavefronts fold their half of the rows as soon as it is complete
//            and publish it (list records, as in the one-phase path); the early wavefronts of
//            the merging workgroups merge the 256 early lists of their row of H and publish
//            the row's THRESHOLD T: the k-th best logit of the early halves.  All of this
//            overlaps with the stream of the late wavefronts.
//   phase 2  when a workgroup's late half is complete, nothing below T can still make the
//            top-k (k candidates at least that good exist already), and in expectation only k
//            logits of ALL late halves together reach T.  The final fold is therefore the
//            softmax statistics plus one comparison per logit (no selection), and a
//            workgroup publishes, per row of H, its statistics and at most two surviving
//            candidates; the final merge polls three records per workgroup instead of
//            twelve, ranks the k early winners with the few survivors, and writes the outputs.
// What does not fit the fast path stays exact through fall-backs: a workgroup without a
// valid T, or with more than two survivors in a row, publishes its late half as a full list
// (flagged in its candidate record); more than 64 final candidates, a flagged list or a failed
// phase-1 merge send the row through the general merge of the plain partial arrays.
#pragma once

#include "epilogue.hpp"

namespace frspec {

// Rows of the result mailbox used by the two phases (row m of H):
//   rec[m]       phase-1 lists            rec[kP2RecRow + m]  late-half lists (fall-back only)
//   st[m]        final statistics         st[kCand0Row + m], st[kCand1Row + m]  survivors
constexpr int kP2RecRow = 16, kCand0Row = 16, kCand1Row = 32;
constexpr int kTwoPhaseMailRows = 48;          // rows of the mailbox the two-phase path touches
constexpr unsigned kCandNoneId = 0x7FFFFFFFu;  // id field of a "no candidate" record (never a token id)
constexpr unsigned kCandMore = 1u;             // flag in its value field: the late half follows as a full list
// Header words of the workspace: call counter, and one threshold record per row of H,
// (call number << 32) | T bits, valid only for the call whose number it carries.
constexpr int kEpochWord = 2, kTboxWord = 96;

struct alignas(16) TwoPhaseLds {
    unsigned long long key[kWave];       // candidate keys: phase-1 survivors, then the final candidates
    unsigned long long p1_top[kMailK];   // the k best of the early halves by rank (0 = none)
    float T[kStepRows];                  // thresholds of the rows of H, where T_mask says so
    float part_mx[4], part_S[4];
    unsigned T_mask;
    unsigned early_arrived;              // sub-barrier of the four early wavefronts (counts up)
    unsigned late_done;                  // late wavefronts whose logits are in LDS
    unsigned p1_count, p1_failed;
    unsigned n_cand, n_flag, timed_out;
};

// Barrier among `n` wavefronts of a workgroup that may not use the hardware barrier (the other
// wavefronts are still streaming): every participant adds one to an LDS counter and waits
// for it to reach `target`.  LDS executes a wavefront's operations in order, so what the
// wavefront wrote before is visible to whoever sees its arrival.
__device__ __forceinline__ void group_sync(unsigned *ctr, unsigned target) {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (lane_id() == 0) __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    while (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < target)
        __builtin_amdgcn_s_sleep(2);
    asm volatile("" ::: "memory");
}

/*
 * Phase-1 merge of row m by the four early wavefronts of a merging workgroup (no hardware
 * barrier).  Fetches the G <= 256 early lists (k <= 16 records each) until none is empty, keeps
 * the entries that reach the bound (the k-th largest of the 16 maxima over the groups of list
 * heads, as in the one-phase merge), ranks them, leaves the k best in tp->p1_top (and as the
 * first k final candidates in tp->key), and publishes the threshold.  More than 64 entries at
 * the bound (massively tied logits): the records stay where they are, tp->p1_failed is set and
 * the threshold published is -inf, which sends every workgroup and the final merge down their
 * general paths.
 */
__device__ __noinline__ void merge_phase1(Mailbox mb, unsigned *error, int G, int m, int k, TwoPhaseLds *tp,
                                             unsigned spin_limit, unsigned epoch, unsigned long long *tbox,
                                             int wave) {
    constexpr int HPL = 4, NW = 4, TPW = kMailK / NW;
    const int lane = lane_id();
    unsigned long long ent[TPW][HPL], head[HPL];
    const unsigned long long *hrow = mb.rec + mail_rec_index(m, 0, 0);
#pragma unroll
    for (int q = 0; q < HPL; ++q) {
        const int g = lane + kWave * q, gs = g < G ? g : G - 1;
#pragma unroll
        for (int j = 0; j < TPW; ++j) {
            const int t = wave + j * NW, ts = t < k ? t : 0;
            ent[j][q] = observe(mb.rec + mail_rec_index(m, ts, gs));
        }
        head[q] = observe(hrow + gs);
    }
    bool gave_up = false;
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
        }
        if (!__any(again)) break;
        if (polls > spin_limit) {
            gave_up = true;
            break;
        }
        __builtin_amdgcn_s_sleep(2);
    }
    if (gave_up && lane == 0) {
        __hip_atomic_store(error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        tp->timed_out = 1u;
    }

    float lmax = kNegInf;
#pragma unroll
    for (int q = 0; q < HPL; ++q) lmax = fmaxf(lmax, lane + kWave * q < G ? mail_hi(head[q]) : kNegInf);
    unsigned gm = key_hi_of(lmax);
    gm = max_xor16_u32(gm);
    gm = max_xor32_u32(gm);
    const float bound = value_of_key_hi(row16_kth_largest_u32(gm, k));

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
        if (lane == 0) base = atomicAdd(&tp->p1_count, total);
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
                        tp->key[pos] = make_key(key_hi_of(mail_hi(ent[j][q])), ~(unsigned)ent[j][q]);
                    at += (int)__popcll(m1);
                }
            }
    }
    group_sync(&tp->early_arrived, 8u);   // (4 arrivals before the early fold, 4 here)

    const int n = __builtin_amdgcn_readfirstlane(
        (int)__hip_atomic_load(&tp->p1_count, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
    const bool dead = __hip_atomic_load(&tp->timed_out, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) != 0u;
    const bool failed = n > kWave || dead;
    if (!failed) {
        // the records are read: empty them for the next call (every wavefront its own)
#pragma unroll
        for (int q = 0; q < HPL; ++q)
            if (lane + kWave * q < G)
#pragma unroll
                for (int j = 0; j < TPW; ++j)
                    if (wave + j * NW < k)
                        publish(mb.rec + mail_rec_index(m, wave + j * NW, lane + kWave * q), kMailEmpty);
    }
    if (wave != 0) return;
    float T = kNegInf;
    unsigned long long mine = 0ull;
    int rank = 0;
    if (!failed) {
        mine = tp->key[lane];
        const u64x2 *kp = reinterpret_cast<const u64x2 *>(tp->key);
#pragma unroll 4
        for (int j = 0; j < n; j += 2) {
            const u64x2 two = kp[j >> 1];
            rank += two.x > mine;
            rank += two.y > mine;
        }
        // the k-th best value, if there are k
        const unsigned long long kth = __ballot(mine != 0ull && rank == k - 1);
        if (kth != 0ull) {
            const int src = (int)__builtin_ctzll(kth);
            T = value_of_key_hi((unsigned)__builtin_amdgcn_readlane((int)(unsigned)(mine >> 32), src));
        }
    } else if (lane == 0) {
        tp->p1_failed = 1u;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // every lane has its key before the slots are reused
    // the k best by rank, and the same k as the first final candidates
    tp->key[lane] = 0ull;
    if (lane < kMailK) tp->p1_top[lane] = 0ull;
    if (mine != 0ull && rank < k) {
        tp->p1_top[rank] = mine;
        tp->key[rank] = mine;
    }
    if (lane == 0) {
        tp->n_cand = (unsigned)k;
        publish(tbox + m, ((unsigned long long)epoch << 32) | __builtin_bit_cast(unsigned, T));
    }
}

// The first wavefront collects the thresholds of all M rows of H into LDS while the late
// wavefronts of its workgroup are still streaming; it stops when it has them all, or when
// the late wavefronts are done (a row without a threshold takes the fall-back).
__device__ __noinline__ void collect_thresholds(const unsigned long long *tbox, int M, unsigned epoch,
                                                   TwoPhaseLds *tp) {
    const int lane = lane_id();
    const unsigned long long want = M >= 64 ? ~0ull : ((1ull << M) - 1ull);
    unsigned long long have = 0ull;
    for (;;) {
        const unsigned long long rec = observe(tbox + (lane < kStepRows ? lane : 0));
        const bool ok = lane < M && (unsigned)(rec >> 32) == epoch;
        if (ok) tp->T[lane] = __builtin_bit_cast(float, (unsigned)rec);
        have = __ballot(ok);
        if (have == want) break;
        if (__hip_atomic_load(&tp->late_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) >= 4u) break;
        __builtin_amdgcn_s_sleep(16);
    }
    if (lane == 0) tp->T_mask = (unsigned)have;
}

/*
 * Final fold of TWO rows of H by one wavefront, one row per half (lanes 0-31: row m_lo < M,
 * lanes 32-63: row m_hi, which may not exist): the late half of the pass (local rows half ..
 * 2 * half - 1, two per lane) joins the statistics of the early half, which sit in run_ms, and
 * is compared with the row's threshold.  Publishes the row's statistics, and its survivors:
 * up to two as candidate records, otherwise (or without a threshold) the late half as a full
 * list, flagged in the first candidate record.
 */
__device__ __noinline__ void fold_final_pair(const float *z_lds, int ZR, int KS, int z_slice_stride,
                                                const int *ids_lds, int n_valid, int k, int m_lo, int m_hi, int M,
                                                Partials part, Mailbox mail, int g, float *run_ms,
                                                float *run_val, int *run_id, const TwoPhaseLds *tp, bool use_T,
                                                float slack, SelectScratch *sc) {
    constexpr int C = 2;
    const int lane = lane_id(), h = lane >> 5, l32 = lane & 31;
    const int half = ZR >> 1;
    const int m = h ? m_hi : m_lo;
    const bool active = m < M;
    const int mm = active ? m : 0;
    float z[C] = {0.0f, 0.0f};
    const float *zp = z_lds + mm * ZR + half + l32 * C;
    for (int q = 0; q < KS; ++q) {
        float t[C];
        lds_words<C, float, fvec4, fvec2>(zp + q * z_slice_stride, t);
        z[0] += t[0];
        z[1] += t[1];
    }
    int id[C];
    lds_words<C, int, ivec4, ivec2>(ids_lds + half + l32 * C, id);
    const float mx1 = run_ms[2 * mm], S1 = run_ms[2 * mm + 1];
    const bool have_T = use_T && ((tp->T_mask >> mm) & 1u);
    const float Tm = tp->T[mm] - slack;

    bool ok[C];
    float v[C];
    float lmax = kNegInf;
#pragma unroll
    for (int c = 0; c < C; ++c) {
        ok[c] = active && (half + l32 * C + c < n_valid);
        v[c] = ok[c] ? z[c] : kNegInf;
        lmax = fmaxf(lmax, v[c]);
    }
    const float mx = fmaxf(mx1, row16_max_f32(max_xor16_f32(lmax)));
    float p = exp_diff(v[0], mx) + exp_diff(v[1], mx);
    p = sum_xor16_f32(p);
    const float S = S1 * exp_diff(mx1, mx) + row16_sum_all(p);

    // survivors: not below the threshold (a NaN is not below anything)
    unsigned long long mask[C];
    int n0 = 0, n1 = 0, pos[C];
    bool sv[C];
#pragma unroll
    for (int c = 0; c < C; ++c) {
        sv[c] = ok[c] && !(have_T && v[c] < Tm);
        mask[c] = __ballot(sv[c]);
        const int c_lo = __popc((unsigned)mask[c]), c_hi = __popc((unsigned)(mask[c] >> 32));
        const int before = (int)__builtin_amdgcn_mbcnt_hi((unsigned)(mask[c] >> 32),
                                                          __builtin_amdgcn_mbcnt_lo((unsigned)mask[c], 0u));
        pos[c] = h ? before - c_lo + n1 : before + n0;
        n0 += c_lo;
        n1 += c_hi;
    }
    const bool full_lists = n0 > 2 || n1 > 2;   // wave-uniform
    if (active) {
        if (l32 == 0) publish(mail.st + mail_st_index(m, g), mail_pack_stats(mx, S));
        const int n_h = h ? n1 : n0;
        if (!full_lists) {
#pragma unroll
            for (int c = 0; c < C; ++c)
                if (sv[c])
                    publish(mail.st + mail_st_index((pos[c] ? kCand1Row : kCand0Row) + m, g),
                            mail_pack(v[c], (unsigned)id[c]));
            if (l32 < 2 && l32 >= n_h)
                publish(mail.st + mail_st_index((l32 ? kCand1Row : kCand0Row) + m, g),
                        ((unsigned long long)0u << 32) | kCandNoneId);
        } else if (l32 < 2) {
            publish(mail.st + mail_st_index((l32 ? kCand1Row : kCand0Row) + m, g),
                    ((unsigned long long)(l32 ? 0u : kCandMore) << 32) | kCandNoneId);
        }
    }
    if (!full_lists) return;
    // The late half as a sorted list of its own (phase-2 list records): the selecting fold of the
    // one-phase path on the late rows.
    const int n_late = n_valid > half ? n_valid - half : 0;
    const FoldSink out{FoldTo::kMailboxP2, part, mail, g, run_ms, run_val, run_id, kP2RecRow};
    if (fold_pair_fast<64, false, false>(z_lds + half, ZR, 0, KS, z_slice_stride, ids_lds + half, n_late, k, m, active,
                                         out, sc))
        return;
    fold_row_general<64, false>(FoldRow{z_lds + m_lo * ZR + half, run_ms + 2 * m_lo, run_val + m_lo * k, run_id + m_lo * k},
                                KS, z_slice_stride, ids_lds + half, n_late, k, sc, out, m_lo);
    if (m_hi < M)
        fold_row_general<64, false>(
            FoldRow{z_lds + m_hi * ZR + half, run_ms + 2 * m_hi, run_val + m_hi * k, run_id + m_hi * k}, KS,
            z_slice_stride, ids_lds + half, n_late, k, sc, out, m_hi);
}

// "No result" for row m, also as hand-over records of the fused expansion.
__device__ __forceinline__ void row_without_result(int m, int M, int k, int *token_ids, float *logp,
                                                   unsigned long long *step_rec) {
    write_no_result(m, M, M, k, token_ids, logp);
    if (step_rec && lane_id() < k) publish(step_rec + m * kMailK + lane_id(), mail_pack(kNegInf, (unsigned)INT_MAX));
}

/*
 * General form of the final merge of row m (all wavefronts of the workgroup; barriers inside):
 * every workgroup's late-half result (its two candidate records, or its flagged full list) and
 * the early halves (the k winners of phase 1, or, if that merge failed, the 256 early lists
 * still in the mailbox) are laid out as sorted lists in the plain partial arrays and merged
 * by the general merge.  All records of the row are emptied.
 */
__device__ __noinline__ void merge_final_general(Mailbox mb, Partials P, unsigned *error, int G, int m, int M, int k,
                                                 int *token_ids, float *logp, TwoPhaseLds *tp, SelectScratch *sc,
                                                 unsigned long long *step_rec, unsigned spin_limit) {
    const int tid = (int)threadIdx.x, lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const bool p1_failed = tp->p1_failed != 0u;
    bool gave_up = false;
    auto wait_for = [&](const unsigned long long *p) {
        unsigned long long r = observe(p);
        for (unsigned polls = 0; r == kMailEmpty && !gave_up; ++polls) {
            if (polls > spin_limit) gave_up = true;
            __builtin_amdgcn_s_sleep(2);
            r = observe(p);
        }
        return r;
    };
    auto put = [&](int t, int slot, float v, int id) {
        publish(P.val + part_index(m * k + t, slot), v);
        publish(P.id + part_index(m * k + t, slot), id);
    };
    for (int g = tid; g < G; g += (int)blockDim.x) {
        unsigned long long *ps = mb.st + mail_st_index(m, g);
        unsigned long long *p0 = mb.st + mail_st_index(kCand0Row + m, g);
        unsigned long long *p1 = mb.st + mail_st_index(kCand1Row + m, g);
        const unsigned long long stt = observe(ps), c0 = observe(p0), c1 = observe(p1);   // (all have arrived)
        publish(P.ms + part_index(m * 2, g), mail_hi(stt));
        publish(P.ms + part_index(m * 2 + 1, g), mail_lo_f32(stt));
        const bool none0 = (unsigned)c0 == kCandNoneId, none1 = (unsigned)c1 == kCandNoneId;
        if (none0 && ((unsigned)(c0 >> 32) & kCandMore)) {
            for (int t = 0; t < k; ++t) {
                unsigned long long *pr = mb.rec + mail_rec_index(kP2RecRow + m, t, g);
                const unsigned long long r = wait_for(pr);
                put(t, g, mail_hi(r), (int)(unsigned)r);
                publish(pr, kMailEmpty);
            }
        } else {
            float va = none0 ? kNegInf : mail_hi(c0), vb = none1 ? kNegInf : mail_hi(c1);
            int ia = none0 ? INT_MAX : (int)(unsigned)c0, ib = none1 ? INT_MAX : (int)(unsigned)c1;
            if (ib != INT_MAX && (ia == INT_MAX || cand_before(vb, ib, va, ia))) {
                const float tv = va;
                const int ti = ia;
                va = vb;
                ia = ib;
                vb = tv;
                ib = ti;
            }
            put(0, g, va, ia);
            if (k > 1) put(1, g, vb, ib);
            for (int t = 2; t < k; ++t) put(t, g, kNegInf, INT_MAX);
        }
        publish(ps, kMailEmpty);
        publish(p0, kMailEmpty);
        publish(p1, kMailEmpty);
        if (p1_failed) {
            // the early list of workgroup g, still in the mailbox, as list number G + g
            for (int t = 0; t < k; ++t) {
                unsigned long long *pr = mb.rec + mail_rec_index(m, t, g);
                const unsigned long long r = wait_for(pr);
                put(t, G + g, mail_hi(r), (int)(unsigned)r);
                publish(pr, kMailEmpty);
            }
            publish(P.ms + part_index(m * 2, G + g), kNegInf);
            publish(P.ms + part_index(m * 2 + 1, G + g), 0.0f);
        }
    }
    if (!p1_failed && tid < k) {
        const unsigned long long key = tp->p1_top[tid];
        put(tid, G, key ? value_of_key_hi((unsigned)(key >> 32)) : kNegInf, key ? (int)~(unsigned)key : INT_MAX);
        if (tid == 0) {
            publish(P.ms + part_index(m * 2, G), kNegInf);
            publish(P.ms + part_index(m * 2 + 1, G), 0.0f);
        }
    }
    wait_stores_done();
    if (__syncthreads_or(gave_up ? 1 : 0)) {
        if (tid == 0) __hip_atomic_store(error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (wave == 0) row_without_result(m, M, k, token_ids, logp, step_rec);
        return;
    }
    if (wave == 0) {
        final_merge_general(P, p1_failed ? 2 * G : G + 1, m, M, M, k, token_ids, logp, sc);   // this row only
        if (step_rec) {
            wait_stores_done();
            if (lane < k)
                publish(step_rec + m * kMailK + lane, mail_pack(observe(logp + (size_t)m * k + lane),
                                                                 (unsigned)observe(token_ids + (size_t)m * k + lane)));
        }
    }
}

/*
 * Final merge of row m by a merging workgroup (eight wavefronts): polls, per workgroup g, the
 * statistics record and the two candidate records until none is empty; log Z from the
 * statistics; the candidates join the k early winners already in tp->key and are ranked by
 * counting; token ids and log-probabilities are written (and handed on to the fused beam-search
 * expansion when step_rec is given).
 */
__device__ __noinline__ void merge_final(Mailbox mb, Partials P, unsigned *error, int G, int m, int M,
                                            int k, int *token_ids, float *logp, TwoPhaseLds *tp, SelectScratch *sc,
                                            unsigned long long *step_rec, unsigned spin_limit) {
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x / kWave);
    const bool first4 = wave < 4;
    const int g = (wave & 3) * kWave + lane, gs = g < G ? g : G - 1;
    const bool real = g < G;
    // wavefronts 0-3: statistics and first candidate of workgroup g; 4-7: its second candidate
    const unsigned long long *pa = mb.st + mail_st_index(first4 ? m : kCand1Row + m, gs);
    const unsigned long long *pb = mb.st + mail_st_index(kCand0Row + m, gs);
    unsigned long long ra = observe(pa), rb = first4 ? observe(pb) : 0ull;
    for (unsigned polls = 0;; ++polls) {
        bool again = false;
        if (real && ra == kMailEmpty) {
            ra = observe(pa);
            again = true;
        }
        if (real && rb == kMailEmpty) {
            rb = observe(pb);
            again = true;
        }
        if (!__any(again)) break;
        if (polls > spin_limit) {
            if (lane == 0) {
                __hip_atomic_store(error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                tp->timed_out = 1u;
            }
            break;
        }
        __builtin_amdgcn_s_sleep(1);
    }
    const unsigned long long cand = first4 ? rb : ra;
    const bool none = (unsigned)cand == kCandNoneId;
    const bool is_cand = real && !none && cand != kMailEmpty;
    const bool more = real && first4 && none && ((unsigned)(cand >> 32) & kCandMore);
    const unsigned long long cmask = __ballot(is_cand);
    if (cmask != 0ull) {
        unsigned base = 0u;
        if (lane == 0) base = atomicAdd(&tp->n_cand, (unsigned)__popcll(cmask));
        const int pos = __builtin_amdgcn_readfirstlane((int)base) +
                        (int)__builtin_amdgcn_mbcnt_hi((unsigned)(cmask >> 32),
                                                       __builtin_amdgcn_mbcnt_lo((unsigned)cmask, 0u));
        if (is_cand && pos < kWave) tp->key[pos] = make_key(key_hi_of(mail_hi(cand)), ~(unsigned)cand);
    }
    if (__any(more) && lane == 0) atomicAdd(&tp->n_flag, 1u);
    if (first4) {
        const float mxg = real ? mail_hi(ra) : kNegInf, Sg = real ? mail_lo_f32(ra) : 0.0f;
        const float wmx = wave_max_f32(mxg);
        const float wS = wave_sum_f32(Sg * exp_diff(mxg, wmx));
        if (lane == 0) {
            tp->part_mx[wave] = wmx;
            tp->part_S[wave] = wS;
        }
    }
    __syncthreads();
    if (tp->timed_out != 0u) {
        if (wave == 0) row_without_result(m, M, k, token_ids, logp, step_rec);
        return;
    }
    const int n = __builtin_amdgcn_readfirstlane((int)tp->n_cand);
    if (tp->n_flag != 0u || n > kWave || tp->p1_failed != 0u) {
        merge_final_general(mb, P, error, G, m, M, k, token_ids, logp, tp, sc, step_rec, spin_limit);
        return;
    }
    if (wave == 0) {
        const float m01 = fmaxf(tp->part_mx[0], tp->part_mx[1]), m23 = fmaxf(tp->part_mx[2], tp->part_mx[3]);
        const float mx = fmaxf(m01, m23);
        const float S = (tp->part_S[0] * exp_diff(tp->part_mx[0], mx) + tp->part_S[1] * exp_diff(tp->part_mx[1], mx)) +
                        (tp->part_S[2] * exp_diff(tp->part_mx[2], mx) + tp->part_S[3] * exp_diff(tp->part_mx[3], mx));
        const float logZ = mx + __logf(S);
        const unsigned long long mine = tp->key[lane];
        const u64x2 *kp = reinterpret_cast<const u64x2 *>(tp->key);
        int rank = 0;
#pragma unroll 4
        for (int j = 0; j < n; j += 2) {
            const u64x2 two = kp[j >> 1];
            rank += two.x > mine;
            rank += two.y > mine;
        }
        const int nz = (int)__popcll(__ballot(mine != 0ull));
        if (mine != 0ull && rank < k) {
            const int tok = (int)~(unsigned)mine;
            const float lp = value_of_key_hi((unsigned)(mine >> 32)) - logZ;
            token_ids[(size_t)m * k + rank] = tok;
            logp[(size_t)m * k + rank] = lp;
            if (step_rec) publish(step_rec + m * kMailK + rank, mail_pack(lp, (unsigned)tok));
        }
        if (lane >= nz && lane < k) {   // fewer candidates than k in the whole subset
            token_ids[(size_t)m * k + lane] = INT_MAX;
            logp[(size_t)m * k + lane] = kNegInf;
            if (step_rec) publish(step_rec + m * kMailK + lane, mail_pack(kNegInf, (unsigned)INT_MAX));
        }
    } else if (real) {
        // the records are read: empty them for the next call
        if (wave < 4) {
            publish(mb.st + mail_st_index(m, g), kMailEmpty);
        } else {
            publish(mb.st + mail_st_index(kCand0Row + m, g), kMailEmpty);
            publish(mb.st + mail_st_index(kCand1Row + m, g), kMailEmpty);
        }
        if (wave == 4) publish(mb.st + mail_st_index(m, lane), kMailEmpty);   // (the first wavefront's share)
    }
}

}  // namespace frspec
