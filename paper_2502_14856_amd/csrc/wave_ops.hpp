// Wavefront-level primitives for gfx950 (64 lanes, DPP rows of 16 lanes).
#pragma once

#include <hip/hip_runtime.h>
#include <limits.h>
#include <stdint.h>

namespace frspec {

// 16 bytes as a native vector (what the 128-bit load/store builtins accept)
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x4 zero_u32x4() { return u32x4{0u, 0u, 0u, 0u}; }

constexpr int kWave = 64;
constexpr float kNegInf = -__builtin_huge_valf();

// DPP control words of the GCN3+/CDNA encoding.
constexpr int kDppQuadXor1 = 0xB1;       // quad_perm:[1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;       // quad_perm:[2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;
constexpr int kDppRowMirror = 0x140;
constexpr int kDppRowRor1 = 0x121;
constexpr int kDppRowRor2 = 0x122;
constexpr int kDppRowRor4 = 0x124;
constexpr int kDppRowRor8 = 0x128;

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    int r = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false);
    return __builtin_bit_cast(float, r);
}
template <int CTRL>
__device__ __forceinline__ int dpp_i32(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false);
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

__device__ __forceinline__ float readlane_f32(float v, int lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

// Sum over each DPP row of 16 lanes; every lane of the row receives the total.
__device__ __forceinline__ float row16_sum(float v) {
    v += dpp_f32<kDppRowRor8>(v);
    v += dpp_f32<kDppRowRor4>(v);
    v += dpp_f32<kDppRowRor2>(v);
    v += dpp_f32<kDppRowRor1>(v);
    return v;
}

// Maximum over the 64 lanes, returned to every lane (wave-uniform).
__device__ __forceinline__ float wave_max_f32(float v) {
    v = fmaxf(v, dpp_f32<kDppQuadXor1>(v));
    v = fmaxf(v, dpp_f32<kDppQuadXor2>(v));
    v = fmaxf(v, dpp_f32<kDppRowHalfMirror>(v));
    v = fmaxf(v, dpp_f32<kDppRowMirror>(v));
    float a = readlane_f32(v, 0), b = readlane_f32(v, 16);
    float c = readlane_f32(v, 32), d = readlane_f32(v, 48);
    return fmaxf(fmaxf(a, b), fmaxf(c, d));
}

__device__ __forceinline__ int wave_min_i32(int v) {
    v = min(v, dpp_i32<kDppQuadXor1>(v));
    v = min(v, dpp_i32<kDppQuadXor2>(v));
    v = min(v, dpp_i32<kDppRowHalfMirror>(v));
    v = min(v, dpp_i32<kDppRowMirror>(v));
    int a = __builtin_amdgcn_readlane(v, 0), b = __builtin_amdgcn_readlane(v, 16);
    int c = __builtin_amdgcn_readlane(v, 32), d = __builtin_amdgcn_readlane(v, 48);
    return min(min(a, b), min(c, d));
}

__device__ __forceinline__ unsigned wave_min_u32(unsigned v) {
    v = min(v, (unsigned)dpp_i32<kDppQuadXor1>((int)v));
    v = min(v, (unsigned)dpp_i32<kDppQuadXor2>((int)v));
    v = min(v, (unsigned)dpp_i32<kDppRowHalfMirror>((int)v));
    v = min(v, (unsigned)dpp_i32<kDppRowMirror>((int)v));
    unsigned a = __builtin_amdgcn_readlane(v, 0), b = __builtin_amdgcn_readlane(v, 16);
    unsigned c = __builtin_amdgcn_readlane(v, 32), d = __builtin_amdgcn_readlane(v, 48);
    return min(min(a, b), min(c, d));
}

// Sum over the 64 lanes in a fixed order, returned to every lane.
__device__ __forceinline__ float wave_sum_f32(float v) {
    v += dpp_f32<kDppQuadXor1>(v);
    v += dpp_f32<kDppQuadXor2>(v);
    v += dpp_f32<kDppRowHalfMirror>(v);
    v += dpp_f32<kDppRowMirror>(v);
    float a = readlane_f32(v, 0), b = readlane_f32(v, 16);
    float c = readlane_f32(v, 32), d = readlane_f32(v, 48);
    return (a + b) + (c + d);
}

// ---- row (16 lanes) and half-wave (32 lanes) primitives ----
// Butterfly reductions over a DPP row: every lane of the row receives the same bits.
__device__ __forceinline__ unsigned row16_max_u32(unsigned v) {
    v = max(v, (unsigned)dpp_i32<kDppQuadXor1>((int)v));
    v = max(v, (unsigned)dpp_i32<kDppQuadXor2>((int)v));
    v = max(v, (unsigned)dpp_i32<kDppRowHalfMirror>((int)v));
    v = max(v, (unsigned)dpp_i32<kDppRowMirror>((int)v));
    return v;
}
__device__ __forceinline__ unsigned row16_min_u32(unsigned v) {
    v = min(v, (unsigned)dpp_i32<kDppQuadXor1>((int)v));
    v = min(v, (unsigned)dpp_i32<kDppQuadXor2>((int)v));
    v = min(v, (unsigned)dpp_i32<kDppRowHalfMirror>((int)v));
    v = min(v, (unsigned)dpp_i32<kDppRowMirror>((int)v));
    return v;
}
__device__ __forceinline__ float row16_max_f32(float v) {
    v = fmaxf(v, dpp_f32<kDppQuadXor1>(v));
    v = fmaxf(v, dpp_f32<kDppQuadXor2>(v));
    v = fmaxf(v, dpp_f32<kDppRowHalfMirror>(v));
    v = fmaxf(v, dpp_f32<kDppRowMirror>(v));
    return v;
}
__device__ __forceinline__ float row16_sum_all(float v) {
    v += dpp_f32<kDppQuadXor1>(v);
    v += dpp_f32<kDppQuadXor2>(v);
    v += dpp_f32<kDppRowHalfMirror>(v);
    v += dpp_f32<kDppRowMirror>(v);
    return v;
}
// v[l] combined with v[l ^ 16] (v[l ^ 32]) in every lane, through the lane-swap instructions
// of the vector ALU (v_permlane16_swap / v_permlane32_swap): given the same value in both
// operands, one result holds v[l] and the other v[l ^ 16] in every lane, in one order or
// the other, which is all a commutative combination needs.  No trip through the LDS pipe.
__device__ __forceinline__ unsigned max_xor16_u32(unsigned v) {
    const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    return max((unsigned)r[0], (unsigned)r[1]);
}
__device__ __forceinline__ unsigned max_xor32_u32(unsigned v) {
    const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return max((unsigned)r[0], (unsigned)r[1]);
}
__device__ __forceinline__ float max_xor16_f32(float v) {
    const auto r = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned, v), __builtin_bit_cast(unsigned, v),
                                                    false, false);
    return fmaxf(__builtin_bit_cast(float, (unsigned)r[0]), __builtin_bit_cast(float, (unsigned)r[1]));
}
__device__ __forceinline__ float sum_xor16_f32(float v) {
    const auto r = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned, v), __builtin_bit_cast(unsigned, v),
                                                    false, false);
    return __builtin_bit_cast(float, (unsigned)r[0]) + __builtin_bit_cast(float, (unsigned)r[1]);
}
// The k-th largest (1 <= k <= 16, counted with multiplicity) of the 16 values held by the
// lanes of a DPP row, returned to every lane of the row: the smallest value that has
// fewer than k strictly larger ones.  Rows are independent of each other.
template <int N>
__device__ __forceinline__ int row16_count_greater(unsigned v) {
    int c = (unsigned)dpp_i32<0x120 + N>((int)v) > v;   // row_ror:N
    if constexpr (N > 1) c += row16_count_greater<N - 1>(v);
    return c;
}
__device__ __forceinline__ unsigned row16_kth_largest_u32(unsigned v, int k) {
    const int greater = row16_count_greater<15>(v);
    return row16_min_u32(greater < k ? v : 0xFFFFFFFFu);
}

// The same over the 32 values held by the lanes of each half of the wavefront (two DPP rows):
// a lane counts the larger ones in its own row by rotations, and in the other row of its half
// by rotations of the value it receives from there (lane-swap instruction, no LDS pipe).
template <int N>
__device__ __forceinline__ int row16_count_greater_than(unsigned w, unsigned v) {
    int c = (unsigned)dpp_i32<0x120 + N>((int)w) > v;   // row_ror:N
    if constexpr (N > 1) c += row16_count_greater_than<N - 1>(w, v);
    return c;
}
__device__ __forceinline__ unsigned half32_kth_largest_u32(unsigned v, int k) {
    const auto sw = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    const unsigned other = (unsigned)sw[0] == v ? (unsigned)sw[1] : (unsigned)sw[0];   // v[l ^ 16]
    const int greater = row16_count_greater<15>(v) + (other > v) + row16_count_greater_than<15>(other, v);
    const unsigned cand = row16_min_u32(greater < k ? v : 0xFFFFFFFFu);
    const auto sm = __builtin_amdgcn_permlane16_swap(cand, cand, false, false);
    return min((unsigned)sm[0], (unsigned)sm[1]);
}
// ... and over the 32 values that the 16 lanes of a DPP row hold two at a time (a, b).
template <int N>
__device__ __forceinline__ void row16_count_greater_pair(unsigned a, unsigned b, int &ga, int &gb) {
    const unsigned ra = (unsigned)dpp_i32<0x120 + N>((int)a), rb = (unsigned)dpp_i32<0x120 + N>((int)b);
    ga += (ra > a) + (rb > a);
    gb += (ra > b) + (rb > b);
    if constexpr (N > 1) row16_count_greater_pair<N - 1>(a, b, ga, gb);
}
__device__ __forceinline__ unsigned row16x2_kth_largest_u32(unsigned a, unsigned b, int k) {
    int ga = b > a, gb = a > b;
    row16_count_greater_pair<15>(a, b, ga, gb);
    return row16_min_u32(min(ga < k ? a : 0xFFFFFFFFu, gb < k ? b : 0xFFFFFFFFu));
}
// From this k on a bound from 16 group maxima admits too much (at k = 16 it is the smallest of them):
// the folds and the merge that have 32 values at hand take the k-th largest of 32 groups instead.
// The choice is a template argument of the folds and of the merge (B32), made once per pass by the
// kernels: as a run-time choice inside them it cost the k <= 10 calls 0.3 us (the compiler computes
// both bounds and selects, or, with the 32-group bound out of line, keeps registers clear for the call).
constexpr int kBound32FromK = 11;

// (value, id) ordering of the candidate lists: larger value first, equal values by
// lower token id.
__device__ __forceinline__ bool cand_before(float va, int ida, float vb, int idb) {
    return (va > vb) || (va == vb && ida < idb);
}

// exp(a - b) that is 0 (not NaN) when a is -inf, whatever b is.
__device__ __forceinline__ float exp_diff(float a, float b) {
    return (a == kNegInf) ? 0.0f : __expf(a - b);
}

// Candidate keys: 64 bits that order like (value descending, token id ascending) when
// compared as unsigned integers, larger = better.  High word: the fp32 value mapped
// monotonically to unsigned (-0 is folded into +0 first, as the float comparison does);
// low word: ~id.  The all-zero key marks an empty slot (no finite or infinite value maps
// to a zero high word).
__device__ __forceinline__ unsigned key_hi_of(float v) {
    const unsigned u = __builtin_bit_cast(unsigned, v + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float value_of_key_hi(unsigned h) {
    const unsigned u = (h & 0x80000000u) ? (h & 0x7FFFFFFFu) : ~h;
    return __builtin_bit_cast(float, u);
}
__device__ __forceinline__ unsigned long long make_key(unsigned hi, unsigned lo) {
    return ((unsigned long long)hi << 32) | lo;
}

// Per-wavefront LDS scratch of the threshold selection below.
struct alignas(16) SelectScratch {
    unsigned long long key[2 * kWave];   // the four-row fold keeps 32 slots per row
    int pl[kWave];
};

constexpr int kSmallKMax = 16;   // largest k the threshold selection handles

/*
 * The k best (k <= 16) of 64*CPL keyed candidates, without k dependent rounds:
 *   1. each quad of lanes takes the maximum value of its 4*CPL candidates; the k-th
 *      largest of the 16 quad maxima, L, is a lower bound of the k-th best value overall
 *      (k different quads hold a value >= L);
 *   2. the candidates with value >= L (at least k, a few more in expectation) are packed
 *      into lanes 0..n-1 through LDS;
 *   3. each survivor counts the survivors that beat it; that count is its rank.
 * On return lane i < n holds one survivor (key, pl) and its rank; the k best are the
 * survivors with rank < k.  Returns false, having decided nothing, if more than 64
 * candidates survive (massively tied values): the caller then falls back to the
 * round-by-round selection.
 */

template <int CPL>
__device__ __forceinline__ bool wave_topk_small(const unsigned (&hi)[CPL], const unsigned (&lo)[CPL],
                                                const int (&pl)[CPL], int k, SelectScratch *sc,
                                                unsigned long long &mine, int &mine_pl, int &rank,
                                                int &n) {
    const int lane = lane_id();
    unsigned qm = hi[0];
#pragma unroll
    for (int c = 1; c < CPL; ++c) qm = max(qm, hi[c]);
    qm = max(qm, (unsigned)dpp_i32<kDppQuadXor1>((int)qm));
    qm = max(qm, (unsigned)dpp_i32<kDppQuadXor2>((int)qm));
    int greater = 0;   // quads whose maximum is strictly larger than this lane's quad maximum
#pragma unroll
    for (int q = 0; q < 16; ++q) greater += (unsigned)__builtin_amdgcn_readlane((int)qm, 4 * q) > qm;
    // the smallest quad maximum that still is among the k largest = the k-th largest
    const unsigned L = wave_min_u32(greater <= k - 1 ? qm : 0xFFFFFFFFu);

    n = 0;
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        const bool sv = hi[c] != 0u && hi[c] >= L;
        const unsigned long long mask = __ballot(sv);
        const int pos = n + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32),
                                                           __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u));
        if (sv && pos < kWave) {
            sc->key[pos] = make_key(hi[c], lo[c]);
            sc->pl[pos] = pl[c];
        }
        n += (int)__popcll(mask);
    }
    if (n > kWave) return false;

    mine = lane < n ? sc->key[lane] : 0ull;
    mine_pl = lane < n ? sc->pl[lane] : -1;
    rank = 0;
    // every survivor is compared with every survivor; the keys are read back from LDS
    // (same address in all lanes: a broadcast), several reads in flight at a time
#pragma unroll 8
    for (int j = 0; j < n; ++j) rank += sc->key[j] > mine;
    return true;
}

// Rank of each lane's key among the keys of all 64 lanes (number of strictly larger keys);
// empty lanes pass key 0.  For candidate sets that already sit one per lane.
__device__ __forceinline__ int wave_rank_all(unsigned long long mine, SelectScratch *sc) {
    sc->key[lane_id()] = mine;
    int rank = 0;
#pragma unroll 16
    for (int j = 0; j < kWave; ++j) rank += sc->key[j] > mine;
    return rank;
}

/*
 * Selection of the k best of 64*CPL candidates held CPL per lane in registers, for NS
 * independent problems at once (the problems share nothing; running them in one loop lets
 * the scheduler overlap their dependent DPP / readlane chains).
 * Rank j of problem s ends in lane j (out_*[s]), j < k <= 64.  Candidates are consumed
 * (overwritten with the sentinel).  `pl` is an opaque payload carried with each candidate.
 * Every lane executes exactly k rounds whatever the data, so NaNs cannot stall it.
 */
template <int NS, int CPL>
__device__ __forceinline__ void wave_select_topk(float (&v)[NS][CPL], int (&id)[NS][CPL],
                                                 int (&pl)[NS][CPL], int k, float (&out_v)[NS],
                                                 int (&out_id)[NS], int (&out_pl)[NS]) {
    const int lane = lane_id();
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        out_v[s] = kNegInf;
        out_id[s] = INT_MAX;
        out_pl[s] = -1;
    }
    for (int j = 0; j < k; ++j) {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            float bv = v[s][0];
            int bi = id[s][0], bp = pl[s][0], bc = 0;
#pragma unroll
            for (int c = 1; c < CPL; ++c) {
                bool better = cand_before(v[s][c], id[s][c], bv, bi);
                bv = better ? v[s][c] : bv;
                bi = better ? id[s][c] : bi;
                bp = better ? pl[s][c] : bp;
                bc = better ? c : bc;
            }
            const float wmax = wave_max_f32(bv);
            bool mine = (bv == wmax);
            unsigned long long mask = __ballot(mine);
            if (__popcll(mask) > 1) {   // equal values in several lanes: lower id wins
                int mid = wave_min_i32(mine ? bi : INT_MAX);
                mask = __ballot(mine && bi == mid);
            }
            const int win = (mask == 0ull) ? 0 : (int)__builtin_ctzll(mask);
            const float wv = readlane_f32(bv, win);
            const int wid = __builtin_amdgcn_readlane(bi, win);
            const int wpl = __builtin_amdgcn_readlane(bp, win);
            if (lane == j) {
                out_v[s] = wv;
                out_id[s] = wid;
                out_pl[s] = wpl;
            }
            const bool me = (lane == win);
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                bool kill = me && (c == bc);
                v[s][c] = kill ? kNegInf : v[s][c];
                id[s][c] = kill ? INT_MAX : id[s][c];
                pl[s][c] = kill ? -1 : pl[s][c];
            }
        }
    }
}

}  // namespace frspec
