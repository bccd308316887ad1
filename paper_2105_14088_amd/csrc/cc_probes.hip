// Cost matrix from latency probes (Section 4.2): per ordered pair of nodes the RTT at a given percentile
// of its K samples (nearest rank), then c[a][b] <- max(c[a][b], c[b][a]).
//
// HBM-bound by design: every sample is read from HBM exactly once.  One workgroup per unordered pair
// stages one direction's K samples in LDS and finds the sample of rank k by descending over the value's
// bits from the top set bit of the largest sample: with candidate x = prefix | bit, the bit is kept iff
// fewer than k samples are below x.  Counting is one compare per 64 samples: the compare mask of a
// wavefront is population-counted on the scalar unit, so there are no per-lane counters and no wave
// reduction; the four waves' counts meet in LDS once per bit.
#include "cc_device.h"
#include "cc_internal.h"

namespace cc {
using namespace ccd;

namespace {

constexpr int kCostMax = (1 << 21) - 1;

__global__ __launch_bounds__(256) void probes_percentile_kernel(const int32_t* __restrict__ samples, int N, int K,
                                                                int rank, int symmetrize,
                                                                int32_t* __restrict__ out) {
    extern __shared__ int32_t sm[];          // K samples, padded to a multiple of 1024 with values no candidate exceeds
    __shared__ int wave_count[2][4];
    __shared__ int wave_top[4];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int a = blockIdx.y, b = blockIdx.x;
    if (a == b) {
        if (tid == 0) out[(int64_t)a * N + a] = 0;
        return;
    }
    if (symmetrize && a > b) return;         // the block of (b, a) covers both directions
    const int kpad = (K + 1023) & ~1023;
    int result = 0;
    for (int dir = 0; dir < (symmetrize ? 2 : 1); ++dir) {
        const int32_t* src = samples + ((int64_t)(dir ? b : a) * N + (dir ? a : b)) * K;
        int top = 0;
        for (int e = tid; e < kpad; e += 256) {
            int v = 0x7fffffff;
            if (e < K) {
                v = clampi(src[e], 0, kCostMax);
                top = max(top, v);
            }
            sm[e] = v;
        }
        top = wave_max(top);
        if (lane == 0) wave_top[wv] = top;
        __syncthreads();
        top = max(max(wave_top[0], wave_top[1]), max(wave_top[2], wave_top[3]));
        int prefix = 0, parity = 0;
        for (int bit = top ? 31 - __clz(top) : -1; bit >= 0; --bit) {
            const int cand = prefix | (1 << bit);
            int below = 0;                   // wave-uniform
            for (int e = tid * 4; e < kpad; e += 1024) {
                const int4 v = *(const int4*)(sm + e);
                below += __popcll(__ballot(v.x < cand)) + __popcll(__ballot(v.y < cand)) +
                         __popcll(__ballot(v.z < cand)) + __popcll(__ballot(v.w < cand));
            }
            if (lane == 0) wave_count[parity][wv] = below;
            __syncthreads();
            const int total = wave_count[parity][0] + wave_count[parity][1] + wave_count[parity][2] + wave_count[parity][3];
            if (total < rank) prefix = cand; // the sample of rank `rank` is at least cand
            parity ^= 1;
        }
        result = max(result, prefix);
        __syncthreads();                     // all reads of this direction's samples done before the next is staged
    }
    if (tid == 0) {
        out[(int64_t)a * N + b] = result;
        if (symmetrize) out[(int64_t)b * N + a] = result;
    }
}

}  // namespace

hipError_t launch_probes_percentile(const int32_t* samples, int N, int K, int rank, bool symmetrize, int32_t* out,
                                    hipStream_t s) {
    const size_t lds = sizeof(int32_t) * (size_t)((K + 1023) & ~1023);
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)probes_percentile_kernel,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(probes_percentile_kernel, dim3(N, N), dim3(256), lds, s, samples, N, K, rank,
                       symmetrize ? 1 : 0, out);
    return hipGetLastError();
}

}  // namespace cc
