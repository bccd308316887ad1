// Wave-level building blocks for kernels that keep one ring rank per lane (N = 64): DPP rotates and
// reductions, and the seeded initial tour built inside the wave.
#pragma once
#include "cc_device.h"

namespace cc {
namespace w64 {
using namespace ccd;

constexpr int kN = 64;

// DPP controls (gfx9 encoding)
constexpr int kDppQuadSwap1 = 0xB1;     // quad_perm:[1,0,3,2]
constexpr int kDppQuadSwap2 = 0x4E;     // quad_perm:[2,3,0,1]
constexpr int kDppWaveRol1 = 0x134;     // lane p <- lane p+1 (cyclic over 64 lanes)
constexpr int kDppWaveRor1 = 0x13C;     // lane p <- lane p-1 (cyclic over 64 lanes)
constexpr int kDppRowMirror = 0x140;
constexpr int kDppRowHalfMirror = 0x141;
constexpr int kDppRowBcast15 = 0x142;
constexpr int kDppRowBcast31 = 0x143;

template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ int dpp(int old, int v) {
    return __builtin_amdgcn_update_dpp(old, v, CTRL, ROW_MASK, 0xf, false);
}
// full-wave rotates read a valid lane everywhere, so the "old" operand is irrelevant (bound_ctrl set)
__device__ __forceinline__ int from_next_lane(int v) {
    return __builtin_amdgcn_update_dpp(v, v, kDppWaveRol1, 0xf, 0xf, true);
}
__device__ __forceinline__ int from_prev_lane(int v) {
    return __builtin_amdgcn_update_dpp(v, v, kDppWaveRor1, 0xf, 0xf, true);
}
__device__ __forceinline__ long long from_next_lane(long long v) {
    const int lo = from_next_lane((int)(unsigned)(unsigned long long)v);
    const int hi = from_next_lane((int)((unsigned long long)v >> 32));
    return (long long)(((unsigned long long)(unsigned)hi << 32) | (unsigned)lo);
}

// Minimum over the wave, returned as a wave-uniform value.
__device__ __forceinline__ int wave_min_uniform(int v) { return wave_min(v); }
__device__ __forceinline__ long long wave_min_uniform(long long v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        const long long o = __shfl_xor(v, m, kWave);
        v = o < v ? o : v;
    }
    return v;
}

// Calls f(lo, hi) exactly once for every pair lo < hi of 0 .. 63, spread over a workgroup of 256 threads: lane l of
// wave w takes the pairs {l, l + j} at the cyclic distances j = 1 + w, 5 + w, .. (the distance 32 by its lower 32
// lanes only).  When the pair indexes a 64 x 64 matrix of words in LDS, consecutive lanes touch consecutive banks in
// both triangles.  Used to fold the two triangles of a staged matrix in place; the caller synchronises around it.
template <class F>
__device__ __forceinline__ void for_each_pair_64(int tid, F f) {
    const int lane = tid & 63, wv = tid >> 6;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        const int j = 1 + wv + 4 * s;            // 1 .. 32 over the four waves
        const int b = (lane + j) & 63;
        if (j < 32 || lane < 32) f(min(lane, b), max(lane, b));
    }
}

// Mirrors the upper triangle of a 64 x 64 matrix in LDS into the lower one, so that a search reads a symmetric
// matrix whatever the caller's buffer holds.
__device__ __forceinline__ void mirror_upper_triangle_64(int32_t* m, int tid) {
    for_each_pair_64(tid, [&](int lo, int hi) { m[hi * kN + lo] = m[lo * kN + hi]; });
}

// Seeded Fisher-Yates shuffle without a serial chain across lanes.  Lane v follows node v: at step k
// (k = 63 .. 1) ranks k and j_k swap, so a node sitting at rank k moves to j_k and a node sitting at
// j_k moves to k, where it stays (later steps only touch ranks below k).  Swap partners are drawn in
// parallel, one per lane, and broadcast step by step; a forward lane permute finally turns
// "node -> rank" into "rank -> node".
__device__ __forceinline__ int init_tour_in_wave(uint64_t seed, uint32_t r, int lane) {
    const int partner = lane ? shuffle_partner(seed, r, lane) : 0;
    int pos = lane;
#pragma unroll
    for (int k = kN - 1; k >= 1; --k) {
        const int j = __builtin_amdgcn_readlane(partner, k);
        const int moved = (pos == k) ? j : pos;
        pos = (pos == j) ? k : moved;
    }
    return __builtin_amdgcn_ds_permute(pos << 2, lane);
}

}  // namespace w64
}  // namespace cc
