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

// (value, id) ordering of the candidate lists: larger value first, equal values by
// lower token id.
__device__ __forceinline__ bool cand_before(float va, int ida, float vb, int idb) {
    return (va > vb) || (va == vb && ida < idb);
}

// exp(a - b) that is 0 (not NaN) when a is -inf, whatever b is.
__device__ __forceinline__ float exp_diff(float a, float b) {
    return (a == kNegInf) ? 0.0f : __expf(a - b);
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
