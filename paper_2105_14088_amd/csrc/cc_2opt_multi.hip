// 2-opt descent for N = 128, 192 and 256, ring-sum objective on a symmetric matrix: one wavefront per
// restart, K = N / 64 consecutive ranks per lane, the whole cost matrix staged once per workgroup in
// LDS as 16-bit entries (128 KiB at N = 256, shared by the 16 restarts of a 1024-thread workgroup).
//
// Same cyclic-diagonal sweep as the N = 64 kernel (cc_2opt_n64.hip): exchanging ring edges a and
// b = a + d costs  G(a-1, b-1) + G(a, b) - f[a] - f[b]  with G(p, q) = c[t[p]][t[q]], so rank a gathers
// one entry per move and takes the other from rank a-1 - here the same lane's previous register for
// three ranks out of four, a DPP wave rotate for the fourth.  Diagonals d = 2 .. N/2 cover all
// N(N-3)/2 moves with every lane busy.  The partner data (node id and (-f[b] << 8 | rank(b))) of the
// K ranks of a lane is a window of 2K registers that slides by one rank per diagonal and is refilled
// by K wave rotates every K diagonals.  rank(b) = (b-1) mod N orders the partners of one rank as
// their move ids are ordered; after the sweep each rank converts its best partner to the move id and
// (delta, id) is min-reduced lexicographically over the wave.
// Keys are delta << 8 | rank in 32 bits (|delta| < 2^22 always fits); the 16-bit matrix needs
// max(c) < 2^16, otherwise the general kernel runs instead (decided on the device, see launch code).
#include "cc_device.h"
#include "cc_internal.h"

namespace cc {
using namespace ccd;

namespace {

constexpr int kRankBits = 8;
constexpr int kWavesPerGroup = 16;
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

// flags[0] = largest entry of the matrix (entries clamped to the contract range first).  One workgroup,
// plain stores: nothing to clear beforehand.
__global__ __launch_bounds__(1024) void matrix_max_kernel(const int32_t* __restrict__ c, int n2,
                                                          int32_t* __restrict__ flags) {
    __shared__ int part[16];
    const int4* c4 = (const int4*)c;           // N is a multiple of 64 here, so n2 is a multiple of 4
    const int n4 = n2 / 4;
    int mx = 0;
    if ((uintptr_t)c & 15u) {                  // matrix not 16-byte aligned: scalar loads
        for (int e = threadIdx.x; e < n2; e += 1024) mx = max(mx, clampi(c[e], 0, (1 << 21) - 1));
    } else
    for (int e = threadIdx.x; e < n4; e += 8 * 1024) {
        int4 v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = (e + k * 1024 < n4) ? c4[e + k * 1024] : make_int4(0, 0, 0, 0);
#pragma unroll
        for (int k = 0; k < 8; ++k)
            mx = max(max(mx, clampi(v[k].x, 0, (1 << 21) - 1)),
                     max(max(clampi(v[k].y, 0, (1 << 21) - 1), clampi(v[k].z, 0, (1 << 21) - 1)),
                         clampi(v[k].w, 0, (1 << 21) - 1)));
    }
    mx = wave_max(mx);
    if (lane_id() == 0) part[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int k = 1; k < 16; ++k) mx = max(mx, part[k]);
        flags[0] = mx;
    }
}

template <int K>
__global__ __launch_bounds__(64 * kWavesPerGroup) void twoopt_sum_multi_kernel(
    const int32_t* __restrict__ c, int restarts, int32_t* __restrict__ tours, int64_t* __restrict__ costs,
    int32_t* __restrict__ moves, const int32_t* __restrict__ flags) {
    constexpr int N = 64 * K;
    constexpr int H = N / 2;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    if (flags[0] >= (1 << 16)) return;            // 16-bit staging impossible: the general kernel handles it
    uint16_t* mat = (uint16_t*)smem;                                   // [N][N]
    int32_t* scratch_all = (int32_t*)(smem + (size_t)N * N * 2);       // kWavesPerGroup x N
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    // stage the matrix as 16-bit entries, two per 32-bit store
    for (int e = tid; e < N * N / 2; e += 64 * kWavesPerGroup) {
        const int lo = clampi(c[2 * e], 0, 0xffff), hi = clampi(c[2 * e + 1], 0, 0xffff);
        ((uint32_t*)mat)[e] = (uint32_t)lo | ((uint32_t)hi << 16);
    }
    __syncthreads();
    const int64_t r = (int64_t)blockIdx.x * kWavesPerGroup + wv;
    if (r >= restarts) return;
    int32_t* scratch = scratch_all + wv * N;
    const unsigned char* mbytes = (const unsigned char*)mat;

    int t[K];
#pragma unroll
    for (int m = 0; m < K; ++m) t[m] = clampi(tours[r * N + K * lane + m], 0, N - 1);

    long long cur = 0;
    int applied = 0;
    bool first = true;
    for (;;) {
        // hops into the lane's K ranks; partner words; row offsets
        int f[K], kp[K], rowofs[K];
        {
            const int tlast = from_prev_lane(t[K - 1]);
#pragma unroll
            for (int m = 0; m < K; ++m) {
                const int tp = m ? t[m - 1] : tlast;
                rowofs[m] = t[m] * (2 * N);
                f[m] = *(const uint16_t*)(mbytes + rowofs[m] + 2 * tp);
                const int a = K * lane + m;
                kp[m] = (int)(0u - ((unsigned)f[m] << kRankBits)) + (a ? a - 1 : N - 1);
            }
        }
        if (first) {
            int s = 0;
#pragma unroll
            for (int m = 0; m < K; ++m) s += f[m];
            cur = wave_sum(s);
            first = false;
        }
        // partner windows: entries 0..K-1 belong to this lane's block of ranks, K..2K-1 to the next lane's
        int tw[2 * K], kw[2 * K];
#pragma unroll
        for (int m = 0; m < K; ++m) {
            tw[m] = t[m];
            kw[m] = kp[m];
            tw[K + m] = from_next_lane(t[m]);
            kw[K + m] = from_next_lane(kp[m]);
        }
        int best[K];
#pragma unroll
        for (int m = 0; m < K; ++m) best[m] = 0x7fffffff;

        auto diagonal = [&](int rr) {          // partner of slot m sits at window index m + rr
            int D[K];
#pragma unroll
            for (int m = 0; m < K; ++m) D[m] = *(const uint16_t*)(mbytes + rowofs[m] + 2 * tw[m + rr]);
            const int Dlast = from_prev_lane(D[K - 1]);
#pragma unroll
            for (int m = 0; m < K; ++m) {
                const int E = m ? D[m - 1] : Dlast;
                const int key = (int)(((unsigned)(E + D[m]) << kRankBits) + (unsigned)kw[m + rr]);
                best[m] = min(best[m], key);
            }
        };
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
        // d = K*q + rr.  q = 0: only rr >= 2 (K = 2: nothing); q = 1 .. H/K - 1: all rr; q = H/K: rr = 0 (d = N/2)
#pragma unroll
        for (int rr = 2; rr < K; ++rr) diagonal(rr);
        slide();
#pragma unroll 1
        for (int q = 1; q < H / K; ++q) {
#pragma unroll
            for (int rr = 0; rr < K; ++rr) diagonal(rr);
            slide();
        }
        diagonal(0);

        // per rank: best partner -> move id; then the lexicographic minimum of (delta, id) over the wave
        int bd = 0x7fffffff, bid = 0x7fffffff;
#pragma unroll
        for (int m = 0; m < K; ++m) {
            const int key = (int)((unsigned)best[m] - ((unsigned)f[m] << kRankBits));
            const int delta = key >> kRankBits;
            const int rank_b = key & ((1 << kRankBits) - 1);
            const int b = rank_b + 1 == N ? 0 : rank_b + 1;
            const int a = K * lane + m;
            const int lo = min(a, b), hi = max(a, b);
            const int id = lo ? lo * N + hi - 1 : hi * N + N - 1;
            if (delta < bd || (delta == bd && id < bid)) { bd = delta; bid = id; }
        }
        const int dwin = wave_min_all(bd);
        if (dwin >= 0) break;
        const int id = wave_min_all(bd == dwin ? bid : 0x7fffffff);
        const int mi = id / N, mj = id % N;
        // reverse ranks mi..mj through the wave's LDS slice
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int m = 0; m < K; ++m) scratch[K * lane + m] = t[m];
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int m = 0; m < K; ++m) {
            const int a = K * lane + m;
            const int src = (a >= mi && a <= mj) ? mi + mj - a : a;
            t[m] = scratch[src];
        }
        __builtin_amdgcn_wave_barrier();
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

}  // namespace

hipError_t launch_matrix_max(const int32_t* c, int N, int32_t* flags, hipStream_t s) {
    hipLaunchKernelGGL(matrix_max_kernel, dim3(1), dim3(1024), 0, s, c, N * N, flags);
    return hipGetLastError();
}

template <int K>
static hipError_t launch_multi(const int32_t* c, int restarts, int32_t* tours, int64_t* costs, int32_t* moves,
                               const int32_t* flags, hipStream_t s) {
    constexpr int N = 64 * K;
    const size_t lds = (size_t)N * N * 2 + (size_t)kWavesPerGroup * N * 4;
    hipError_t e = hipFuncSetAttribute((const void*)twoopt_sum_multi_kernel<K>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int grid = (restarts + kWavesPerGroup - 1) / kWavesPerGroup;
    hipLaunchKernelGGL((twoopt_sum_multi_kernel<K>), dim3(grid), dim3(64 * kWavesPerGroup), lds, s, c, restarts, tours,
                       costs, moves, flags);
    return hipGetLastError();
}

// Tours must already hold the initial orders.  flags[0] must hold the matrix maximum (launch_matrix_max).
hipError_t launch_2opt_sum_multi(const int32_t* c, int N, int restarts, int32_t* tours, int64_t* costs,
                                 int32_t* moves, const int32_t* flags, hipStream_t s) {
    if (N == 128) return launch_multi<2>(c, restarts, tours, costs, moves, flags, s);
    if (N == 192) return launch_multi<3>(c, restarts, tours, costs, moves, flags, s);
    return launch_multi<4>(c, restarts, tours, costs, moves, flags, s);
}

}  // namespace cc
