// Ring search over segment insertions (Or-opt), alone or together with the 2-opt moves, for N = 64, ring-sum
// objective on a symmetric matrix with entries below 2^16: one wavefront per restart, the order in one VGPR
// (lane a holds t[a]), the matrix staged once per workgroup in LDS.  Move set, ids and tie-breaks as in cc.h
// (cc_local_search); other matrices and sizes take the general kernel of cc_local.hip.
//
// Everything is read off the cyclic diagonals D_e[a] = c[t[a+e]][t[a]], e = 1 .. 63, one LDS gather per lane and
// diagonal (D_1 and D_63 are the hops f[a+1] and f[a] themselves).  With the segment starting at rank s = a and the
// gap between ranks g = a+e and g+1, the two edges a segment insertion adds are
//     length 1           D_e[a] + D_{e+1}[a]
//     length 2, kept     D_e[a] + D_e[a+1]            reversed   D_{e-1}[a+1] + D_{e+1}[a]
//     length 3, kept     D_e[a] + D_{e-1}[a+2]        reversed   D_{e-2}[a+2] + D_{e+1}[a]
// i.e. the lane's own gathers and those of its two upper neighbours (two DPP wave rotates per diagonal).  The gaps
// next to the segment are e = -1 .. L-1, the same for every lane, so no move is ever masked: e runs from L to 62.
// The edge the gap opens, f[g+1], travels round the wave with the gap's rank and node as one word (one DPP rotate
// per diagonal), exactly as in the 2-opt kernel for N = 64; a 2-opt move between edges a and a+d is
// D_d[a] + D_d[a-1] plus the word of gap a+d-1, so the 2-opt sweep rides on the same gathers (d = 2 .. 32).
// One running minimum per move variant and lane over keys (edges added - f[g+1]) << 14 | g << 8; the cost of
// cutting the segment out (the same for all gaps) is added after the sweep.  Each lane then picks the best of its
// candidates in id order, the wave takes the smallest delta and, among the lanes that hold it, the smallest id.
#include "cc_device.h"
#include "cc_internal.h"
#include "cc_wave64.h"

namespace cc {
using namespace ccd;

namespace {

using namespace w64;
constexpr int kSh = 14;
constexpr int kIntMax = 0x7fffffff;
constexpr int kNoSegment = 1 << 28;        // cut-out cost of a lane that has no segment of that length

template <bool WITH_2OPT>
__device__ __forceinline__ void descend_local(const int32_t* m, int lane, int& t, long long& cost, int& applied_out) {
    const char* mbytes = (const char*)m;
    const int rank_a = (lane + kN - 1) & (kN - 1);
    long long cur = 0;
    int applied = 0;
    bool first = true;
    for (;;) {
        const int tprev = from_prev_lane(t);
        const int fm = m[t * kN + tprev];                      // f[a] << 14
        if (first) {
            cur = wave_sum64((long long)(fm >> kSh));
            first = false;
        }
        const int f1 = from_next_lane(fm);                     // f[a+1]
        const int rowofs = t * (kN * 4);
        // word of gap g = a: the edge it opens, its rank, its first node's column offset
        int pk = (0 - f1) + ((lane << 8) | (4 * t));

        // ---- gathers: D[e] = c[t[a+e]][t[a]] << 14, pkd[e] = word of gap a+e
        int D[kN], pkd[kN];
        D[1] = f1;
        D[kN - 1] = fm;
#pragma unroll
        for (int e = 1; e <= kN - 2; ++e) {
            pk = from_next_lane(pk);
            pkd[e] = pk;
            if (e >= 2) D[e] = *(const int32_t*)(mbytes + (((int)pk & 0xff) | rowofs));
        }
        // ---- running minima
        int acc[5] = {kIntMax, kIntMax, kIntMax, kIntMax, kIntMax};
        int acc2 = kIntMax;
        int x1_prev = 0, x2_prev = 0, x2_prev2 = 0;           // D_{e-1}[a+1], D_{e-1}[a+2], D_{e-2}[a+2]
#pragma unroll
        for (int e = 1; e <= kN - 2; ++e) {
            const int x1 = from_next_lane(D[e]);               // D_e[a+1]
            const int x2 = from_next_lane(x1);                 // D_e[a+2]
            const int w = pkd[e];
            acc[0] = min(acc[0], add3(D[e], D[e + 1], w));
            if (e >= 2) {
                acc[1] = min(acc[1], add3(D[e], x1, w));
                acc[2] = min(acc[2], add3(x1_prev, D[e + 1], w));
            }
            if (e >= 3) {
                acc[3] = min(acc[3], add3(D[e], x2_prev, w));
                acc[4] = min(acc[4], add3(x2_prev2, D[e + 1], w));
            }
            if (WITH_2OPT && e + 1 <= kN / 2) {                // 2-opt diagonal d = e + 1 uses the word of gap a+d-1
                const int d = e + 1;
                acc2 = min(acc2, D[d] + from_prev_lane(D[d]) + w);
            }
            x2_prev2 = x2_prev;
            x1_prev = x1;
            x2_prev = x2;
        }
        // ---- candidates of this lane, in id order
        int best_d = kIntMax, best_id = kIntMax;
        if (WITH_2OPT) {
            const int k = acc2 - fm;                           // + (-f[a])
            const int r = (k >> 8) & (kN - 1);
            best_d = k >> kSh;
            best_id = r < rank_a ? (r << 6) + kN + rank_a : lane * kN + r;
        }
        // cost of cutting the segment out: -f[a] - f[a+L] + c[t[a-1]][t[a+L]], the last term being D_{L+1}[a-1]
        int f_behind = f1;
#pragma unroll
        for (int v = 0; v < 5; ++v) {
            const int L = v == 0 ? 1 : (v + 3) / 2;
            if (v == 3) f_behind = from_next_lane(from_next_lane(f1));         // f[a+3]
            else if (v == 1) f_behind = from_next_lane(f1);                      // f[a+2]
            const bool has = lane >= 1 && lane + L <= kN;
            const int joined = from_prev_lane(D[L + 1]);      // every lane takes part in the rotate
            const int cut = has ? ((joined - fm - f_behind) >> kSh) : kNoSegment;
            const int dv = (acc[v] >> kSh) + cut;
            const int g = (acc[v] >> 8) & (kN - 1);
            const int id = kN * kN * (1 + v) + lane * kN + g;
            if (dv < best_d) {
                best_d = dv;
                best_id = id;
            }
        }
        const int dwin = wave_min(best_d);
        if (dwin >= 0) break;
        const int id = wave_min(best_d == dwin ? best_id : kIntMax);
        // ---- apply: new[p] = old[src(p)]
        const int src = move_source(lane, id, kN);
        t = __shfl(t, src, kWave);
        cur += (long long)dwin;
        ++applied;
    }
    cost = cur;
    applied_out = applied;
}

template <bool WITH_2OPT>
__global__ __launch_bounds__(256) void local_n64_kernel(const int32_t* __restrict__ c, int restarts,
                                                        int32_t* __restrict__ tours, int64_t* __restrict__ costs,
                                                        int32_t* __restrict__ moves,
                                                        const int32_t* __restrict__ flags) {
    if (flags[0] >= (1 << 16)) return;             // keys would not fit: the general kernel does the work
    __shared__ __attribute__((aligned(256))) int32_t m[kN * kN];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
#pragma unroll
    for (int k = 0; k < kN * kN / 256; ++k) m[tid + 256 * k] = clampi(c[tid + 256 * k], 0, (1 << 16) - 1) << kSh;
    __syncthreads();
    mirror_upper_triangle_64(m, tid);      // exact deltas for the matrix the search sees, whatever the buffer holds
    __syncthreads();
    const int64_t r = (int64_t)blockIdx.x * 4 + wv;
    if (r >= restarts) return;
    int t = clampi(tours[r * kN + lane], 0, kN - 1);
    long long cost;
    int applied;
    descend_local<WITH_2OPT>(m, lane, t, cost, applied);
    tours[r * kN + lane] = t;
    if (lane == 0) {
        costs[r] = cost;
        moves[r] = applied;
    }
}

}  // namespace

hipError_t launch_local_n64(const int32_t* c, bool with_2opt, int restarts, int32_t* tours, int64_t* costs,
                            int32_t* moves, const int32_t* flags, hipStream_t s) {
    const int grid = (restarts + 3) / 4;
    if (with_2opt)
        hipLaunchKernelGGL(local_n64_kernel<true>, dim3(grid), dim3(256), 0, s, c, restarts, tours, costs, moves, flags);
    else
        hipLaunchKernelGGL(local_n64_kernel<false>, dim3(grid), dim3(256), 0, s, c, restarts, tours, costs, moves, flags);
    return hipGetLastError();
}

}  // namespace cc
