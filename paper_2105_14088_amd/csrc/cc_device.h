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

// Flat index of entry (min(x, y), max(x, y)) for the flat index e = x * n + y: the ring-sum searches read the matrix
// through its upper triangle, so their deltas are exact for the matrix they see and every descent ends even when the
// caller's matrix is not symmetric.
__device__ __forceinline__ int upper_index(int e, int n) {
    const int x = e / n, y = e - x * n;
    return min(x, y) * n + max(x, y);
}

// a + b + c as one instruction.  Written out because the compiler, seeing several such sums that share two of their
// terms, prefers to form the shared pair once and then spends two instructions on every sum.
__device__ __forceinline__ int add3(int a, int b, int c) {
    int r;
    asm("v_add3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// Rank whose node moves to rank p when move `id` of the ring search is applied (ids as in cc.h, cc_local_search):
// id = i*n + j < n*n reverses ranks i .. j; id = n*n + (variant*n + s)*n + g takes the L ranks s .. s+L-1 out and
// puts them back, kept or reversed, behind the node of rank g (variant 0: L = 1; 1, 2: L = 2; 3, 4: L = 3; even
// variants above 0 reverse the segment).
__device__ __forceinline__ int move_source(int p, int id, int n) {
    if (id < n * n) {
        const int i = id / n, j = id - i * n;
        return (p >= i && p <= j) ? i + j - p : p;
    }
    const int x = id - n * n;
    const int g = x % n, s = (x / n) % n, variant = x / (n * n);
    const int L = variant == 0 ? 1 : (variant + 3) >> 1;
    const bool rev = variant != 0 && (variant & 1) == 0;
    if (g > s) {                                   // towards higher ranks: the segment ends at rank g
        if (p >= s && p <= g - L) return p + L;
        if (p > g - L && p <= g) return rev ? s + L - 1 - (p - (g - L + 1)) : s + (p - (g - L + 1));
    } else {                                       // towards lower ranks: it starts behind rank g
        if (p > g && p <= g + L) return rev ? s + L - 1 - (p - (g + 1)) : s + (p - (g + 1));
        if (p > g + L && p <= s + L - 1) return p - L;
    }
    return p;
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// Reductions over the 64 lanes of a wave; every lane ends with the result.  The 32-bit forms use six DPP steps
// (pairs, quads, half rows, rows: every lane of a row then holds the row's result; then the rows are chained through
// their last lanes, so lane 63 ends with the total, which is broadcast).  Each step reads the register the previous
// one wrote, which needs two wait states before a DPP read.  All 64 lanes must be active.
#define CC_WAVE_REDUCE_DPP(op)                                                      \
    asm volatile("s_nop 1\n\t" op " %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t" \
                 "s_nop 1\n\t" op " %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t" \
                 "s_nop 1\n\t" op " %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"     \
                 "s_nop 1\n\t" op " %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\t"          \
                 "s_nop 1\n\t" op " %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"        \
                 "s_nop 1\n\t" op " %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"        \
                 "s_nop 1"                                                          \
                 : "+v"(v))
__device__ __forceinline__ int wave_sum(int v) {
    CC_WAVE_REDUCE_DPP("v_add_u32_dpp");
    return __builtin_amdgcn_readlane(v, 63);
}
__device__ __forceinline__ int wave_max(int v) {
    CC_WAVE_REDUCE_DPP("v_max_i32_dpp");
    return __builtin_amdgcn_readlane(v, 63);
}
__device__ __forceinline__ int wave_min(int v) {
    CC_WAVE_REDUCE_DPP("v_min_i32_dpp");
    return __builtin_amdgcn_readlane(v, 63);
}
// Three maxima at once: the three chains are interleaved, so the instructions of the other two fill the wait
// states a chain needs between its steps.  Lane 63 ends with each total.
__device__ __forceinline__ void wave_max3(int& a, int& b, int& c) {
#define CC_STEP3(ctrl)                                         \
    "v_max_i32_dpp %0, %0, %0 " ctrl " bank_mask:0xf\n\t"    \
    "v_max_i32_dpp %1, %1, %1 " ctrl " bank_mask:0xf\n\t"    \
    "v_max_i32_dpp %2, %2, %2 " ctrl " bank_mask:0xf\n\t"
    asm volatile("s_nop 1\n\t" CC_STEP3("quad_perm:[1,0,3,2] row_mask:0xf") CC_STEP3("quad_perm:[2,3,0,1] row_mask:0xf")
                     CC_STEP3("row_half_mirror row_mask:0xf") CC_STEP3("row_mirror row_mask:0xf")
                         CC_STEP3("row_bcast:15 row_mask:0xa") CC_STEP3("row_bcast:31 row_mask:0xc") "s_nop 1"
                 : "+v"(a), "+v"(b), "+v"(c));
#undef CC_STEP3
    a = __builtin_amdgcn_readlane(a, 63);
    b = __builtin_amdgcn_readlane(b, 63);
    c = __builtin_amdgcn_readlane(c, 63);
}
// Three maxima over each half of the wave at once (lanes 0..31 and 32..63 separately): the chain above without its
// last step.  Lane 31 ends with the lower halves' maxima, lane 63 with the upper halves'.
__device__ __forceinline__ void half_wave_max3(int& a, int& b, int& c) {
#define CC_STEP3(ctrl)                                         \
    "v_max_i32_dpp %0, %0, %0 " ctrl " bank_mask:0xf\n\t"    \
    "v_max_i32_dpp %1, %1, %1 " ctrl " bank_mask:0xf\n\t"    \
    "v_max_i32_dpp %2, %2, %2 " ctrl " bank_mask:0xf\n\t"
    asm volatile("s_nop 1\n\t" CC_STEP3("quad_perm:[1,0,3,2] row_mask:0xf") CC_STEP3("quad_perm:[2,3,0,1] row_mask:0xf")
                     CC_STEP3("row_half_mirror row_mask:0xf") CC_STEP3("row_mirror row_mask:0xf")
                         CC_STEP3("row_bcast:15 row_mask:0xa") "s_nop 1"
                 : "+v"(a), "+v"(b), "+v"(c));
#undef CC_STEP3
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
