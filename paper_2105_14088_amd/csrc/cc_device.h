// Device-side helpers shared by the kernels of the rank-order search library (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ccd {

constexpr int kWave = 64;

// SplitMix64 (Steele, Lea, Flood 2014): n-th output of a generator started at state `seed` is the
// finaliser applied to seed + n * gamma.
__device__ __forceinline__ uint64_t splitmix64_at(uint64_t seed, uint64_t n) {
    uint64_t z = seed + n * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Swap partner of step k of restart r's Fisher-Yates shuffle (see cc.h, cc_2opt_search).
__device__ __forceinline__ int shuffle_partner(uint64_t seed, uint32_t r, int k) {
    uint64_t ctr = (((uint64_t)r << 32) | (uint32_t)k) + 1u;
    uint64_t u = splitmix64_at(seed, ctr) >> 32;
    return (int)((u * (uint64_t)(k + 1)) >> 32);
}

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// Butterfly reductions over the 64 lanes of a wave; every lane ends with the result.
__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
    return v;
}
__device__ __forceinline__ int wave_max(int v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v = max(v, __shfl_xor(v, m, kWave));
    return v;
}
__device__ __forceinline__ long long wave_sum64(long long v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
    return v;
}
__device__ __forceinline__ unsigned long long wave_min_u64(unsigned long long v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        unsigned long long o = __shfl_xor(v, m, kWave);
        v = o < v ? o : v;
    }
    return v;
}

}  // namespace ccd
