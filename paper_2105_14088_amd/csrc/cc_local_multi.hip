// Ring search over segment insertions (Or-opt), alone or together with the 2-opt moves, for N = 128, 192 and 256,
// ring-sum objective on a symmetric matrix with entries below 2^16: one wavefront per restart, K = N / 64
// consecutive ranks per lane, the matrix staged once per workgroup in LDS as 16-bit entries.  Move set, ids and
// tie-breaks as in cc.h (cc_local_search).
//
// Same formulation as the N = 64 kernel (cc_local_n64.hip) on the layout of the 2-opt kernel for these sizes
// (cc_2opt_multi.hip).  Rank a gathers the cyclic diagonals D_e[a] = c[t[a+e]][t[a]], e = 1 .. N-1, one LDS gather
// each.  With the segment starting at rank a and the gap between ranks g = a+e and g+1 the five variants add the edges
//     length 1           D_e[a] + D_{e+1}[a]
//     length 2, kept     D_e[a] + D_e[a+1]            reversed   D_{e-1}[a+1] + D_{e+1}[a]
//     length 3, kept     D_e[a] + D_{e-1}[a+2]        reversed   D_{e-2}[a+2] + D_{e+1}[a]
// where the values of ranks a+1 and a+2 are the same lane's neighbouring registers except at the end of the lane's
// block (two DPP wave rotates per diagonal).  The gaps that touch the segment are e = -1 .. L-1 for every rank alike,
// so no move is masked.  The word of a gap, -f[g+1] << 8 | g, and its first node travel in a window of 2K registers
// that slides by one rank per diagonal and is refilled by K wave rotates every K diagonals; a 2-opt move between
// edges a and a+d is D_d[a] + D_d[a-1] plus the word of gap a+d-1, so the 2-opt sweep (d = 2 .. N/2) rides on the
// same gathers.  One running minimum per variant and rank; the cost of cutting the segment out is added after the
// sweep; every rank's best candidate goes into a lexicographic (delta, id) minimum over the wave.
#include "cc_device.h"
#include "cc_internal.h"
#include "cc_wave64.h"

namespace cc {
using namespace ccd;

namespace {

using w64::from_next_lane;
using w64::from_prev_lane;
constexpr int kRankBits = 8;
constexpr int kIntMax = 0x7fffffff;
constexpr int kNoSegment = 1 << 28;

__device__ __forceinline__ int wave_min_all(int v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v = min(v, __shfl_xor(v, m, kWave));
    return v;
}

template <int K, bool WITH_2OPT>
__global__ __launch_bounds__(K == 4 ? 768 : 1024) void local_multi_kernel(const int32_t* __restrict__ c, int restarts,
                                                           int32_t* __restrict__ tours, int64_t* __restrict__ costs,
                                                           int32_t* __restrict__ moves,
                                                           const int32_t* __restrict__ flags) {
    constexpr int N = 64 * K;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    if (flags[0] >= (1 << 16)) return;            // 16-bit staging impossible: the general kernel handles it
    uint16_t* mat = (uint16_t*)smem;                                   // [N][N]
    int32_t* slices = (int32_t*)(smem + (size_t)N * N * 2);            // per wave: order T[N], hops F[N]
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    // 16-bit entries, two per store; the matrix is read through its upper triangle (exact deltas whatever it holds)
    for (int e = tid; e < N * N / 2; e += blockDim.x) {
        const int lo = clampi(c[upper_index(2 * e, N)], 0, 0xffff), hi = clampi(c[upper_index(2 * e + 1, N)], 0, 0xffff);
        ((uint32_t*)mat)[e] = (uint32_t)lo | ((uint32_t)hi << 16);
    }
    __syncthreads();
    const int64_t r = (int64_t)blockIdx.x * (blockDim.x >> 6) + wv;
    if (r >= restarts) return;
    int32_t* T = slices + wv * 2 * N;
    int32_t* F = T + N;
    const unsigned char* mbytes = (const unsigned char*)mat;
    auto entry = [&](int rowofs, int node) { return (int)*(const uint16_t*)(mbytes + rowofs + 2 * node); };

    int t[K];
#pragma unroll
    for (int m = 0; m < K; ++m) t[m] = clampi(tours[r * N + K * lane + m], 0, N - 1);

    long long cur = 0;
    int applied = 0;
    bool first = true;
    for (;;) {
        // ---- hops into the lane's K ranks, row offsets, gap words
        int f[K], rowofs[K], gw[K];
        {
            const int tlast = from_prev_lane(t[K - 1]);
#pragma unroll
            for (int m = 0; m < K; ++m) {
                rowofs[m] = t[m] * (2 * N);
                f[m] = entry(rowofs[m], m ? t[m - 1] : tlast);
            }
            const int f_next_lane = from_next_lane(f[0]);
#pragma unroll
            for (int m = 0; m < K; ++m) {
                const int opened = m + 1 < K ? f[m + 1] : f_next_lane;         // f[a+1]: the edge gap a opens
                gw[m] = (int)(0u - ((unsigned)opened << kRankBits)) + (K * lane + m);
            }
        }
        if (first) {
            int s = 0;
#pragma unroll
            for (int m = 0; m < K; ++m) s += f[m];
            cur = wave_sum(s);
            first = false;
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int m = 0; m < K; ++m) {
            T[K * lane + m] = t[m];
            F[K * lane + m] = f[m];
        }
        __builtin_amdgcn_wave_barrier();

        // ---- windows: entries 0..K-1 belong to this lane's block of ranks, K..2K-1 to the next lane's
        int tw[2 * K], kw[2 * K];
#pragma unroll
        for (int m = 0; m < K; ++m) {
            tw[m] = t[m];
            kw[m] = gw[m];
            tw[K + m] = from_next_lane(t[m]);
            kw[K + m] = from_next_lane(gw[m]);
        }
        auto slide = [&]() {
#pragma unroll
            for (int m = 0; m < K; ++m) {
                tw[m] = tw[K + m];
                kw[m] = kw[K + m];
            }
#pragma unroll
            for (int m = 0; m < K; ++m) {
                tw[K + m] = from_next_lane(tw[m]);
                kw[K + m] = from_next_lane(kw[m]);
            }
        };
        int acc[5][K], acc2[K];
        int Dc[K], x1p[K], x2p[K], x2pp[K];
#pragma unroll
        for (int m = 0; m < K; ++m) {
#pragma unroll
            for (int v = 0; v < 5; ++v) acc[v][m] = kIntMax;
            acc2[m] = kIntMax;
            Dc[m] = entry(rowofs[m], tw[m + 1]) << kRankBits;          // D_1, kept shifted into key position
            x1p[m] = x2p[m] = x2pp[m] = 0;
        }
        // One diagonal e = K q + rr (the gap's window index is m + rr).  score1 / score2 / score3: e admits segments of
        // length 1 / 2 / 3; two_opt: diagonal e + 1 is a 2-opt diagonal.  The gathers of diagonal e + 1 go out first.
        auto step = [&](int rr, bool score1, bool score2, bool score3, bool two_opt) {
            int Dn[K];
#pragma unroll
            for (int m = 0; m < K; ++m) Dn[m] = entry(rowofs[m], tw[m + rr + 1]) << kRankBits;
            const int nx0 = from_next_lane(Dc[0]);
            const int nx1 = K >= 2 ? from_next_lane(Dc[K >= 2 ? 1 : 0]) : nx0;
            const int pv = two_opt ? from_prev_lane(Dn[K - 1]) : 0;
#pragma unroll
            for (int m = 0; m < K; ++m) {
                const int x1 = m + 1 < K ? Dc[m + 1 < K ? m + 1 : 0] : nx0;                        // D_e[a+1]
                const int x2 = m + 2 < K ? Dc[m + 2 < K ? m + 2 : 0] : (m + 2 == K ? nx0 : nx1);   // D_e[a+2]
                const int w = kw[m + rr];
                if (score1) acc[0][m] = min(acc[0][m], add3(Dc[m], Dn[m], w));
                if (score2) {
                    acc[1][m] = min(acc[1][m], add3(Dc[m], x1, w));
                    acc[2][m] = min(acc[2][m], add3(x1p[m], Dn[m], w));
                }
                if (score3) {
                    acc[3][m] = min(acc[3][m], add3(Dc[m], x2p[m], w));
                    acc[4][m] = min(acc[4][m], add3(x2pp[m], Dn[m], w));
                }
                if (two_opt) acc2[m] = min(acc2[m], add3(Dn[m], m ? Dn[m ? m - 1 : 0] : pv, w));
                x2pp[m] = x2p[m];
                x1p[m] = x1;
                x2p[m] = x2;
            }
#pragma unroll
            for (int m = 0; m < K; ++m) Dc[m] = Dn[m];
        };
        // q = 0: e = 1 .. K-1 (K = 2: q = 1 still lacks e >= 3 at its first diagonal)
#pragma unroll
        for (int rr = 1; rr < K; ++rr) step(rr, true, rr >= 2, rr >= 3, WITH_2OPT);
        slide();
        if (K == 2) {
            step(0, true, true, false, WITH_2OPT);
            step(1, true, true, true, WITH_2OPT);
            slide();
        }
        // 2-opt diagonals d = e + 1 <= N / 2, i.e. q <= 31
#pragma unroll 1
        for (int q = (K == 2 ? 2 : 1); q < 32; ++q) {
#pragma unroll
            for (int rr = 0; rr < K; ++rr) step(rr, true, true, true, WITH_2OPT);
            slide();
        }
#pragma unroll 1
        for (int q = 32; q < 63; ++q) {
#pragma unroll
            for (int rr = 0; rr < K; ++rr) step(rr, true, true, true, false);
            slide();
        }
        // q = 63: e = N-K .. N-2 are the last gaps; diagonal N-1 only served as D_{e+1} of e = N-2
#pragma unroll
        for (int rr = 0; rr + 1 < K; ++rr) step(rr, true, true, true, false);

        // ---- per rank: best candidate in id order; then the lexicographic minimum of (delta, id) over the wave
        int bd = kIntMax, bid = kIntMax;
#pragma unroll
        for (int m = 0; m < K; ++m) {
            const int a = K * lane + m;
            if (WITH_2OPT) {
                const int key = (int)((unsigned)acc2[m] - ((unsigned)f[m] << kRankBits));
                const int delta = key >> kRankBits;
                const int rank_b = key & ((1 << kRankBits) - 1);
                const int b = rank_b + 1 == N ? 0 : rank_b + 1;
                const int lo = min(a, b), hi = max(a, b);
                const int id = lo ? lo * N + hi - 1 : hi * N + N - 1;
                if (delta < bd || (delta == bd && id < bid)) { bd = delta; bid = id; }
            }
            const int before = T[a ? a - 1 : N - 1];
#pragma unroll
            for (int L = 1; L <= 3; ++L) {
                // cutting the segment out: -f[a] - f[a+L] + c[t[a-1]][t[a+L]]
                const int behind = a + L >= N ? a + L - N : a + L;
                const bool has = a >= 1 && a + L <= N;
                const int cut = has ? entry(before * (2 * N), T[behind]) - f[m] - F[behind] : kNoSegment;
#pragma unroll
                for (int o = 0; o < (L == 1 ? 1 : 2); ++o) {
                    const int v = L == 1 ? 0 : 2 * L - 3 + o;
                    const int delta = (acc[v][m] >> kRankBits) + cut;
                    const int g = acc[v][m] & ((1 << kRankBits) - 1);
                    const int id = N * N * (1 + v) + a * N + g;
                    if (delta < bd || (delta == bd && id < bid)) { bd = delta; bid = id; }
                }
            }
        }
        const int dwin = wave_min_all(bd);
        if (dwin >= 0) break;
        const int id = wave_min_all(bd == dwin ? bid : kIntMax);
        // ---- apply through the wave's copy of the order: new[p] = old[src(p)]
#pragma unroll
        for (int m = 0; m < K; ++m) t[m] = T[move_source(K * lane + m, id, N)];
        cur += dwin;
        ++applied;
    }
#pragma unroll
    for (int m = 0; m < K; ++m) tours[r * N + K * lane + m] = t[m];
    if (lane == 0) {
        costs[r] = cur;
        moves[r] = applied;
    }
}

template <int K, bool WITH_2OPT>
hipError_t launch_k(const int32_t* c, int restarts, int32_t* tours, int64_t* costs, int32_t* moves,
                    const int32_t* flags, hipStream_t s) {
    constexpr int N = 64 * K;
    // up to 16 (N = 256: 12) restarts share a workgroup's copy of the matrix, but no more than keeps all 256
    // compute units busy
    const int most = K == 4 ? 12 : 16;
    int waves = (restarts + 255) / 256;
    waves = waves < 1 ? 1 : (waves > most ? most : waves);
    const size_t lds = (size_t)N * N * 2 + (size_t)waves * 2 * N * 4;
    hipError_t e = hipFuncSetAttribute((const void*)local_multi_kernel<K, WITH_2OPT>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int grid = (restarts + waves - 1) / waves;
    hipLaunchKernelGGL((local_multi_kernel<K, WITH_2OPT>), dim3(grid), dim3(64 * waves), lds, s, c, restarts, tours, costs,
                       moves, flags);
    return hipGetLastError();
}

}  // namespace

// N = 128, 192 or 256.  `tours` must hold the initial tours, flags[0] the matrix maximum (launch_matrix_max).
hipError_t launch_local_multi(const int32_t* c, int N, bool with_2opt, int restarts, int32_t* tours, int64_t* costs,
                              int32_t* moves, const int32_t* flags, hipStream_t s) {
    if (N == 128)
        return with_2opt ? launch_k<2, true>(c, restarts, tours, costs, moves, flags, s)
                         : launch_k<2, false>(c, restarts, tours, costs, moves, flags, s);
    if (N == 192)
        return with_2opt ? launch_k<3, true>(c, restarts, tours, costs, moves, flags, s)
                         : launch_k<3, false>(c, restarts, tours, costs, moves, flags, s);
    return with_2opt ? launch_k<4, true>(c, restarts, tours, costs, moves, flags, s)
                     : launch_k<4, false>(c, restarts, tours, costs, moves, flags, s);
}

}  // namespace cc
