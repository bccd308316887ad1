// Cost matrix from latency probes (Section 4.2): per ordered pair of nodes the RTT at a given percentile
// of its K samples (nearest rank), then c[a][b] <- max(c[a][b], c[b][a]).
//
// Every sample is read from HBM exactly once and then lives in a register.  One wavefront per ordered
// pair: it loads the pair's K samples (up to 256 per lane, all loads in flight together) and finds the
// sample of rank k by descending over the value's bits from the top set bit of the largest sample: with
// candidate x = prefix | bit, the bit is kept iff fewer than k samples are below x.  Counting costs a
// compare and an add-with-carry per 64 samples plus one DPP reduction per bit; there is no barrier and no
// LDS traffic in the descent.  The two directions of a pair are the two waves of one workgroup, which
// meet once, through LDS, for the symmetrisation.
#include "cc_device.h"
#include "cc_internal.h"

namespace cc {
using namespace ccd;

namespace {

constexpr int kCostMax = (1 << 21) - 1;

// acc += (v.x < cand) + (v.y < cand) + (v.z < cand) + (v.w < cand) per lane: each term is a compare into the carry
// flag and an add-with-carry.
__device__ __forceinline__ void count_below(int& acc, const int4& v, int cand) {
    asm("v_cmp_lt_i32 vcc, %1, %5\n\t"
        "v_addc_co_u32 %0, vcc, 0, %0, vcc\n\t"
        "v_cmp_lt_i32 vcc, %2, %5\n\t"
        "v_addc_co_u32 %0, vcc, 0, %0, vcc\n\t"
        "v_cmp_lt_i32 vcc, %3, %5\n\t"
        "v_addc_co_u32 %0, vcc, 0, %0, vcc\n\t"
        "v_cmp_lt_i32 vcc, %4, %5\n\t"
        "v_addc_co_u32 %0, vcc, 0, %0, vcc"
        : "+v"(acc)
        : "v"(v.x), "v"(v.y), "v"(v.z), "v"(v.w), "v"(cand)
        : "vcc");
}

// CH: int4 registers per lane (the wave holds up to 256 * CH samples).  VEC4: K is a multiple of 4 and the sample
// array is 16-byte aligned, so the samples can be fetched as int4.
template <int CH, bool VEC4>
__global__ __launch_bounds__(128) void probes_percentile_kernel(const int32_t* __restrict__ samples, int N, int K,
                                                                int rank, int symmetrize,
                                                                int32_t* __restrict__ out) {
    __shared__ int direction_result[2];
    const int lane = threadIdx.x & 63, dir = threadIdx.x >> 6;
    const int a = blockIdx.y, b = blockIdx.x;
    if (a == b) {
        if (threadIdx.x == 0) out[(int64_t)a * N + a] = 0;
        return;
    }
    if (a > b) return;                       // the workgroup of (min, max) covers both directions
    const int from = dir ? b : a, to = dir ? a : b;
    const int32_t* src = samples + ((int64_t)from * N + to) * K;
    constexpr int kPad = 0x7fffffff;         // no candidate exceeds it: padding never counts as "below"
    // tails are fetched from a clamped (valid) address and then replaced by the padding value
    int4 v[CH];
#pragma unroll
    for (int u = 0; u < CH; ++u) {
        const int e = u * 256 + lane * 4;
        if (VEC4) {
            v[u] = *(const int4*)(src + min(e, K - 4));
        } else {
            v[u].x = src[min(e, K - 1)];
            v[u].y = src[min(e + 1, K - 1)];
            v[u].z = src[min(e + 2, K - 1)];
            v[u].w = src[min(e + 3, K - 1)];
        }
    }
    int top = 0;
#pragma unroll
    for (int u = 0; u < CH; ++u) {
        const int e = u * 256 + lane * 4;
        const int x = clampi(v[u].x, 0, kCostMax), y = clampi(v[u].y, 0, kCostMax);
        const int z = clampi(v[u].z, 0, kCostMax), w = clampi(v[u].w, 0, kCostMax);
        top = max(max(top, e < K ? x : 0), max(e + 1 < K ? y : 0, max(e + 2 < K ? z : 0, e + 3 < K ? w : 0)));
        v[u].x = e < K ? x : kPad;
        v[u].y = e + 1 < K ? y : kPad;
        v[u].z = e + 2 < K ? z : kPad;
        v[u].w = e + 3 < K ? w : kPad;
    }
    top = wave_max(top);
    int prefix = 0;
    for (int bit = top ? 31 - __clz(top) : -1; bit >= 0; --bit) {
        const int cand = prefix | (1 << bit);
        int below = 0;
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            count_below(below, v[u], cand);
        }
        if (wave_sum(below) < rank) prefix = cand;   // the sample of rank `rank` is at least cand
    }
    if (lane == 0) direction_result[dir] = prefix;
    __syncthreads();
    if (lane == 0) {
        const int value = symmetrize ? max(direction_result[0], direction_result[1]) : prefix;
        out[(int64_t)from * N + to] = value;
    }
}

}  // namespace

template <int CH>
static hipError_t probes_launch(const int32_t* samples, int N, int K, int rank, bool symmetrize, int32_t* out,
                                hipStream_t s) {
    const bool vec4 = (K & 3) == 0 && ((uintptr_t)samples & 15u) == 0;
    if (vec4)
        hipLaunchKernelGGL((probes_percentile_kernel<CH, true>), dim3(N, N), dim3(128), 0, s, samples, N, K, rank,
                           symmetrize ? 1 : 0, out);
    else
        hipLaunchKernelGGL((probes_percentile_kernel<CH, false>), dim3(N, N), dim3(128), 0, s, samples, N, K, rank,
                           symmetrize ? 1 : 0, out);
    return hipGetLastError();
}

// K <= 16384 (checked by the caller)
hipError_t launch_probes_percentile(const int32_t* samples, int N, int K, int rank, bool symmetrize, int32_t* out,
                                    hipStream_t s) {
    if (K <= 256) return probes_launch<1>(samples, N, K, rank, symmetrize, out, s);
    if (K <= 1024) return probes_launch<4>(samples, N, K, rank, symmetrize, out, s);
    if (K <= 2048) return probes_launch<8>(samples, N, K, rank, symmetrize, out, s);
    if (K <= 4096) return probes_launch<16>(samples, N, K, rank, symmetrize, out, s);
    if (K <= 10240) return probes_launch<40>(samples, N, K, rank, symmetrize, out, s);
    return probes_launch<64>(samples, N, K, rank, symmetrize, out, s);
}

}  // namespace cc
