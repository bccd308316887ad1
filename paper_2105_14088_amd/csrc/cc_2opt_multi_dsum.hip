// 2-opt descent for N = 128, 192 and 256 under the directed ring-sum objective (matrices with c[a][b] != c[b][a]): one
// wavefront per restart, K = N / 64 consecutive ranks per lane, the cost matrix staged once per workgroup in LDS as
// 16-bit entries, both triangles.
//
// The sweep of cc_2opt_n64_dsum.hip on the register layout of cc_2opt_multi.hip.  Exchanging ring edges a and
// b = a + d cuts the ring into S1 = ranks a .. b-1 and S2 = ranks b .. a-1; the result can be walked two ways:
//   A: S2 as it is, S1 backwards:  new hops GT(a-1,b-1) + GT(a,b);  S2's inner hops cost f, S1's inner hops b
//   B: the opposite direction:     new hops G(a-1,b-1) + G(a,b);    S2's inner hops cost b, S1's inner hops f
// with G(p,q) = c[t[p]][t[q]], GT(p,q) = c[t[q]][t[p]], f[p] = c[t[p]][t[p-1]] (hop p as walked now) and
// b[p] = c[t[p-1]][t[p]] (the same edge the other way).  With F = sum of f (the current cost), Bt = sum of b and
// q = sum over S1's inner hops a+1 .. b-1 of (b - f), which grows by one hop per diagonal,
//   value A - F = GT(a-1,b-1) + GT(a,b) - f[a] - f[b] + q
//   value B - F = G(a-1,b-1) + G(a,b) - b[a] - b[b] - q + (Bt - F).
// Rank a gathers G(a,b) and GT(a,b) and takes the (a-1, b-1) entries from rank a-1 (the same lane's previous
// registers for K-1 ranks out of K, a wave rotate for the first); the partner's f, b, b - f, rank and matrix offsets
// sit in windows of 2K registers that slide by one rank per diagonal and are refilled by K wave rotates every K
// diagonals.  Per rank two running minima over (partial delta) << 8 | rank(b); the rank's own terms are added after
// the sweep, both become (delta, move id) with the ids of cc.h, and the wave takes the lexicographic minimum.
//
// The 32-bit keys hold partial deltas below 2^23 in magnitude: the kernel runs when max(c) * (N + 2) < 2^22 (which also
// means max(c) < 2^16 for the 16-bit matrix), else the general kernel does the work (decided on the device from the
// matrix maximum, see the launch code).
#include "cc_device.h"
#include "cc_internal.h"

namespace cc {
using namespace ccd;

namespace {

constexpr int kDppWaveRol1 = 0x134;     // lane p <- lane p+1 (cyclic over 64 lanes)
constexpr int kDppWaveRor1 = 0x13C;     // lane p <- lane p-1 (cyclic over 64 lanes)
__device__ __forceinline__ int from_next_lane(int v) {
    return __builtin_amdgcn_update_dpp(v, v, kDppWaveRol1, 0xf, 0xf, true);
}
__device__ __forceinline__ int from_prev_lane(int v) {
    return __builtin_amdgcn_update_dpp(v, v, kDppWaveRor1, 0xf, 0xf, true);
}
__device__ __forceinline__ int wave_min_all(int v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v = min(v, __shfl_xor(v, m, kWave));
    return v;
}
constexpr int kRankBits = 8;
// restarts per workgroup at most: they share one LDS copy of the matrix
constexpr int max_waves(int) { return 12; }

template <int K>
__global__ __launch_bounds__(64 * max_waves(K)) void twoopt_dsum_multi_kernel(
    const int32_t* __restrict__ c, int restarts, int with_flip, int32_t* __restrict__ tours,
    int64_t* __restrict__ costs, int32_t* __restrict__ moves, const int32_t* __restrict__ flags) {
    constexpr int N = 64 * K;
    constexpr int H = N / 2;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    if (flags[0] >= dsum_multi_limit(N)) return;      // keys would not fit: the general kernel does the work
    uint16_t* mat = (uint16_t*)smem;                                   // [N][N]
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    int32_t* scratch = (int32_t*)(smem + (size_t)N * N * 2) + (size_t)wv * N;     // the wave's order while a move is applied
    for (int e = tid; e < N * N / 2; e += blockDim.x) {
        const int lo = clampi(c[2 * e], 0, 0xffff), hi = clampi(c[2 * e + 1], 0, 0xffff);
        ((uint32_t*)mat)[e] = (uint32_t)lo | ((uint32_t)hi << 16);
    }
    __syncthreads();
    const int64_t r = (int64_t)blockIdx.x * (blockDim.x >> 6) + wv;
    if (r >= restarts) return;
    const unsigned char* mbytes = (const unsigned char*)mat;

    int t[K];
#pragma unroll
    for (int m = 0; m < K; ++m) t[m] = clampi(tours[r * N + K * lane + m], 0, N - 1);

    int cur = 0, applied = 0;
    bool first = true;
    for (;;) {
        // hops into the lane's K ranks, both directions; Bt - F; row and column offsets
        int f[K], bw[K], rowofs[K], colofs[K];
        int turn;
        {
            const int tlast = from_prev_lane(t[K - 1]);
            int sf = 0, sd = 0;
#pragma unroll
            for (int m = 0; m < K; ++m) {
                const int tp = m ? t[m - 1] : tlast;
                rowofs[m] = t[m] * (2 * N);
                colofs[m] = 2 * t[m];
                f[m] = *(const uint16_t*)(mbytes + rowofs[m] + 2 * tp);
                bw[m] = *(const uint16_t*)(mbytes + tp * (2 * N) + colofs[m]);
                sf += f[m];
                sd += bw[m] - f[m];
            }
            turn = wave_sum(sd);
            if (first) {
                cur = wave_sum(sf);
                first = false;
            }
        }
        // partner windows: entries 0..K-1 belong to this lane's block of ranks, K..2K-1 to the next lane's
        int tr[2 * K], tc[2 * K], fw[2 * K], bww[2 * K], dw[2 * K], kw[2 * K];
#pragma unroll
        for (int m = 0; m < K; ++m) {
            const int a = K * lane + m;
            tr[m] = rowofs[m];
            tc[m] = colofs[m];
            fw[m] = f[m];
            bww[m] = bw[m];
            dw[m] = bw[m] - f[m];
            kw[m] = a ? a - 1 : N - 1;
        }
#pragma unroll
        for (int m = 0; m < K; ++m) {
            tr[K + m] = from_next_lane(tr[m]);
            tc[K + m] = from_next_lane(tc[m]);
            fw[K + m] = from_next_lane(fw[m]);
            bww[K + m] = from_next_lane(bww[m]);
            dw[K + m] = from_next_lane(dw[m]);
            kw[K + m] = from_next_lane(kw[m]);
            // keeps each rotate an instruction of its own: folded into a subtraction it would become
            // v_subrev_u32_dpp, which on this chip rotates the other operand
            asm("" : "+v"(fw[K + m]), "+v"(bww[K + m]), "+v"(dw[K + m]));
        }
        int q[K], bestA[K], bestB[K];
#pragma unroll
        for (int m = 0; m < K; ++m) {
            q[m] = dw[m + 1];                   // hop a+1: S1's only inner hop at d = 2
            bestA[m] = bestB[m] = 0x7fffffff;
        }

        auto diagonal = [&](int rr) {                    // partner of slot m sits at window index m + rr
            int G[K], GT[K];
#pragma unroll
            for (int m = 0; m < K; ++m) {
                G[m] = *(const uint16_t*)(mbytes + rowofs[m] + tc[m + rr]);        // c[t[a]][t[b]]
                GT[m] = *(const uint16_t*)(mbytes + tr[m + rr] + colofs[m]);       // c[t[b]][t[a]]
            }
            int Glast = from_prev_lane(G[K - 1]), GTlast = from_prev_lane(GT[K - 1]);
            asm("" : "+v"(Glast), "+v"(GTlast));
#pragma unroll
            for (int m = 0; m < K; ++m) {
                const int EG = m ? G[m - 1] : Glast, EGT = m ? GT[m - 1] : GTlast;
                const int dA = add3(EGT, GT[m], q[m] - fw[m + rr]);
                const int dB = EG + G[m] - (q[m] + bww[m + rr]);
                bestA[m] = min(bestA[m], (int)(((unsigned)dA << kRankBits) | (unsigned)kw[m + rr]));
                bestB[m] = min(bestB[m], (int)(((unsigned)dB << kRankBits) | (unsigned)kw[m + rr]));
                q[m] += dw[m + rr];             // the partner's hop is an inner hop of S1 from the next diagonal on
            }
        };
        auto slide = [&]() {
#pragma unroll
            for (int m = 0; m < K; ++m) {
                tr[m] = tr[K + m];
                tc[m] = tc[K + m];
                fw[m] = fw[K + m];
                bww[m] = bww[K + m];
                dw[m] = dw[K + m];
                kw[m] = kw[K + m];
            }
#pragma unroll
            for (int m = 0; m < K; ++m) {
                tr[K + m] = from_next_lane(tr[m]);
                tc[K + m] = from_next_lane(tc[m]);
                fw[K + m] = from_next_lane(fw[m]);
                bww[K + m] = from_next_lane(bww[m]);
                dw[K + m] = from_next_lane(dw[m]);
                kw[K + m] = from_next_lane(kw[m]);
                asm("" : "+v"(fw[K + m]), "+v"(bww[K + m]), "+v"(dw[K + m]));
            }
        };
        // d = K*q + rr.  q = 0: only rr >= 2 (K = 2: nothing); q = 1 .. H/K - 1: all rr; q = H/K: rr = 0 (d = N/2)
#pragma unroll
        for (int rr = 2; rr < K; ++rr) diagonal(rr);
        slide();
        int blocks_end = H / K;
        asm("" : "+s"(blocks_end));            // an opaque trip count: unrolled twice, never completely (register pressure)
#pragma unroll 2
        for (int qq = 1; qq < blocks_end; ++qq) {
#pragma unroll
            for (int rr = 0; rr < K; ++rr) diagonal(rr);
            slide();
        }
        diagonal(0);

        // per rank and direction: best partner -> (delta, move id); then the lexicographic minimum over the wave
        int bv = 0x7fffffff, bid = 0x7fffffff;
#pragma unroll
        for (int m = 0; m < K; ++m) {
            const int a = K * lane + m;
            const int rank_a = a ? a - 1 : N - 1;
#pragma unroll
            for (int which = 0; which < 2; ++which) {
                const int key = which ? bestB[m] : bestA[m];
                const int kv = (key >> kRankBits) + (which ? turn - bw[m] : -f[m]);
                const int rk = key & ((1 << kRankBits) - 1);
                const bool wrapped = rk < rank_a;         // b lies before a: the reversed piece is S2, not S1
                const int ij = wrapped ? (rk + 1) * N + rank_a : a * N + rk;
                const int id = ij * 2 + (which ^ (wrapped ? 1 : 0));
                const bool better = kv < bv || (kv == bv && id < bid);
                bv = better ? kv : bv;
                bid = better ? id : bid;
            }
        }
        if (with_flip && lane == 0) {                   // the orientation flip: every hop walked the other way
            const int idf = (N + N - 1) * 2;
            const bool better = turn < bv || (turn == bv && idf < bid);
            bv = better ? turn : bv;
            bid = better ? idf : bid;
        }
        const int dwin = wave_min_all(bv);
        if (dwin >= 0) break;
        const int idwin = wave_min_all(bv == dwin ? bid : 0x7fffffff);
        const int o = idwin & 1, ij = idwin >> 1, mi = ij / N, mj = ij % N;
        // new[p] = old[src(p)] through the wave's LDS slice
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int m = 0; m < K; ++m) scratch[K * lane + m] = t[m];
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int m = 0; m < K; ++m) {
            const int a = K * lane + m;
            const int p0 = o ? (a ? N - a : 0) : a;
            const int src = (p0 >= mi && p0 <= mj) ? mi + mj - p0 : p0;
            t[m] = scratch[src];
        }
        __builtin_amdgcn_wave_barrier();
        cur += dwin;
        ++applied;
    }
#pragma unroll
    for (int m = 0; m < K; ++m) tours[r * N + K * lane + m] = t[m];
    if (lane == 0) {
        costs[r] = (int64_t)cur;
        moves[r] = applied;
    }
}

template <int K>
hipError_t launch_k(const int32_t* c, int restarts, bool with_flip, int32_t* tours, int64_t* costs, int32_t* moves,
                    const int32_t* flags, hipStream_t s) {
    constexpr int N = 64 * K;
    // restarts per workgroup: as many as share one LDS copy of the matrix, but no more than keeps all compute units busy
    int waves = (restarts + 255) / 256;
    waves = waves < 1 ? 1 : (waves > max_waves(K) ? max_waves(K) : waves);
    const size_t lds = (size_t)N * N * 2 + (size_t)waves * N * sizeof(int32_t);
    hipError_t e = hipFuncSetAttribute((const void*)twoopt_dsum_multi_kernel<K>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int grid = (restarts + waves - 1) / waves;
    hipLaunchKernelGGL((twoopt_dsum_multi_kernel<K>), dim3(grid), dim3(64 * waves), lds, s, c, restarts,
                       with_flip ? 1 : 0, tours, costs, moves, flags);
    return hipGetLastError();
}

}  // namespace

// N = 128, 192 or 256.  Tours must already hold the initial orders; flags[0] must hold the matrix maximum
// (launch_matrix_max): the kernel returns at once if it is dsum_multi_limit(N) or more.
hipError_t launch_2opt_dsum_multi(const int32_t* c, int N, int restarts, bool with_flip, int32_t* tours, int64_t* costs,
                                  int32_t* moves, const int32_t* flags, hipStream_t s) {
    if (N == 128) return launch_k<2>(c, restarts, with_flip, tours, costs, moves, flags, s);
    if (N == 192) return launch_k<3>(c, restarts, with_flip, tours, costs, moves, flags, s);
    return launch_k<4>(c, restarts, with_flip, tours, costs, moves, flags, s);
}

}  // namespace cc
