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
constexpr int kWavesPerGroup = 16;      // at most; fewer when the restarts would otherwise leave compute units idle

// Restarts per workgroup: up to 16 share one LDS copy of the matrix, but no more than keeps all 256 compute units busy.
inline int waves_per_group(int restarts, int most) {
    int w = (restarts + 255) / 256;
    w = w < 1 ? 1 : w;
    return w > most ? most : w;
}
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
    const int4* c4 = (const int4*)c;
    const int n4 = n2 / 4;
    int mx = 0;
    if ((uintptr_t)c & 15u) {                  // matrix not 16-byte aligned: scalar loads
        for (int e = threadIdx.x; e < n2; e += 1024) mx = max(mx, clampi(c[e], 0, (1 << 21) - 1));
    } else {
        for (int e = 4 * n4 + threadIdx.x; e < n2; e += 1024) mx = max(mx, clampi(c[e], 0, (1 << 21) - 1));   // odd N
    }
    if (!((uintptr_t)c & 15u))
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
    for (int e = tid; e < N * N / 2; e += blockDim.x) {
        const int lo = clampi(c[upper_index(2 * e, N)], 0, 0xffff), hi = clampi(c[upper_index(2 * e + 1, N)], 0, 0xffff);
        ((uint32_t*)mat)[e] = (uint32_t)lo | ((uint32_t)hi << 16);
    }
    __syncthreads();
    const int64_t r = (int64_t)blockIdx.x * (blockDim.x >> 6) + wv;
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

// ------------------------------------------------------------------------------------ any N <= 256
// Ring-sum descent for the sizes the kernels above do not cover (N not a multiple of 64).  One wavefront per
// restart, rank a = lane + 64 m in slot m (slots past N idle), 16-bit matrix in LDS.  Without N = 64 K the partner
// data cannot travel round the wave by lane rotates, so it sits in LDS: the wave's slice holds the order T[N] and,
// twice over so that a + d never wraps, the pairs P[x] = (column byte offset of t[x mod N],
// -f[x mod N] << 8 | rank(x mod N)).  A move (a, b = a + d) costs one 8-byte read of P[a + d] and two gathers,
// G(a, b) and G(a-1, b-1); the column of b-1 is the previous diagonal's column of b.  Diagonals d = 2 .. N/2
// (rounded down) cover every pair of non-adjacent ring edges.  Keys, move ids and reductions as above.
__host__ __device__ inline size_t flex_slice_bytes(int N) { return (size_t)N * 16 + (((size_t)N * 4 + 15) & ~(size_t)15); }

template <int K>
__global__ void twoopt_sum_flex_kernel(const int32_t* __restrict__ c, int N, int restarts, int32_t* __restrict__ tours,
                                       int64_t* __restrict__ costs, int32_t* __restrict__ moves,
                                       const int32_t* __restrict__ flags) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    if (flags[0] >= (1 << 16)) return;            // 16-bit staging impossible: the general kernel handles it
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, waves = blockDim.x >> 6;
    uint16_t* mat = (uint16_t*)smem;                                           // [N][N]
    const size_t slice_bytes = flex_slice_bytes(N);                            // P: 16 N, then T: 4 N (padded)
    unsigned char* slice = smem + (((size_t)N * N * 2 + 15) & ~(size_t)15) + (size_t)wv * slice_bytes;
    int2* P = (int2*)slice;
    int32_t* T = (int32_t*)(slice + (size_t)N * 16);
    for (int e = tid; e < N * N; e += blockDim.x) mat[e] = (uint16_t)clampi(c[upper_index(e, N)], 0, 0xffff);
    __syncthreads();
    const int64_t r = (int64_t)blockIdx.x * waves + wv;
    if (r >= restarts) return;
    const unsigned char* mbytes = (const unsigned char*)mat;
    const int row_bytes = 2 * N, D = N / 2;

    int t[K];
    bool live[K];
#pragma unroll
    for (int m = 0; m < K; ++m) {
        const int a = lane + 64 * m;
        live[m] = a < N;
        t[m] = live[m] ? clampi(tours[r * N + a], 0, N - 1) : 0;
    }
    long long cur = 0;
    int applied = 0;
    bool first = true;
    for (;;) {
#pragma unroll
        for (int m = 0; m < K; ++m)
            if (live[m]) T[lane + 64 * m] = t[m];
        __builtin_amdgcn_wave_barrier();
        int f[K], rowA[K], rowP[K];
        int fsum = 0;
#pragma unroll
        for (int m = 0; m < K; ++m) {
            const int a = lane + 64 * m;
            f[m] = rowA[m] = rowP[m] = 0;
            if (live[m]) {
                const int tp = T[a ? a - 1 : N - 1];
                rowA[m] = t[m] * row_bytes;
                rowP[m] = tp * row_bytes;
                f[m] = *(const uint16_t*)(mbytes + rowA[m] + 2 * tp);
                const int2 pw = make_int2(2 * t[m], (int)(0u - ((unsigned)f[m] << kRankBits)) + (a ? a - 1 : N - 1));
                P[a] = pw;
                P[a + N] = pw;
                fsum += f[m];
            }
        }
        if (first) {
            cur = wave_sum(fsum);
            first = false;
        }
        __builtin_amdgcn_wave_barrier();
        // idle slots score rank 0's moves again (in bounds, no divergence in the loop) and are discarded afterwards
        int best[K], colprev[K], abase[K];
#pragma unroll
        for (int m = 0; m < K; ++m) {
            best[m] = 0x7fffffff;
            abase[m] = live[m] ? lane + 64 * m : 0;
            colprev[m] = P[abase[m] + 1].x;                        // column of rank a + 1 = b - 1 at d = 2
        }
#pragma unroll 4
        for (int d = 2; d <= D; ++d) {
#pragma unroll
            for (int m = 0; m < K; ++m) {
                const int2 pw = P[abase[m] + d];
                const int g1 = *(const uint16_t*)(mbytes + rowA[m] + pw.x);
                const int g2 = *(const uint16_t*)(mbytes + rowP[m] + colprev[m]);
                best[m] = min(best[m], (int)(((unsigned)(g1 + g2) << kRankBits) + (unsigned)pw.y));
                colprev[m] = pw.x;
            }
        }
#pragma unroll
        for (int m = 0; m < K; ++m)
            if (!live[m]) best[m] = 0x7fffffff;
        // per rank: best partner -> move id; then the lexicographic minimum of (delta, id) over the wave
        int bd = 0x7fffffff, bid = 0x7fffffff;
#pragma unroll
        for (int m = 0; m < K; ++m) {
            if (live[m] && best[m] != 0x7fffffff) {
                const int key = (int)((unsigned)best[m] - ((unsigned)f[m] << kRankBits));
                const int delta = key >> kRankBits;
                const int rank_b = key & ((1 << kRankBits) - 1);
                const int b = rank_b + 1 == N ? 0 : rank_b + 1;
                const int a = lane + 64 * m;
                const int lo = min(a, b), hi = max(a, b);
                const int id = lo ? lo * N + hi - 1 : hi * N + N - 1;
                if (delta < bd || (delta == bd && id < bid)) { bd = delta; bid = id; }
            }
        }
        const int dwin = wave_min(bd);
        if (dwin >= 0) break;
        const int id = wave_min(bd == dwin ? bid : 0x7fffffff);
        const int mi = id / N, mj = id % N;
        // reverse ranks mi..mj: T still holds the order
#pragma unroll
        for (int m = 0; m < K; ++m) {
            const int a = lane + 64 * m;
            if (live[m]) t[m] = T[(a >= mi && a <= mj) ? mi + mj - a : a];
        }
        __builtin_amdgcn_wave_barrier();
        cur += dwin;
        ++applied;
    }
#pragma unroll
    for (int m = 0; m < K; ++m)
        if (live[m]) tours[r * N + lane + 64 * m] = t[m];
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
    const int waves = waves_per_group(restarts, kWavesPerGroup);
    const size_t lds = (size_t)N * N * 2 + (size_t)waves * N * 4;
    hipError_t e = hipFuncSetAttribute((const void*)twoopt_sum_multi_kernel<K>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int grid = (restarts + waves - 1) / waves;
    hipLaunchKernelGGL((twoopt_sum_multi_kernel<K>), dim3(grid), dim3(64 * waves), lds, s, c, restarts, tours,
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

template <int K>
static hipError_t launch_flex_k(const int32_t* c, int N, int restarts, int32_t* tours, int64_t* costs, int32_t* moves,
                                const int32_t* flags, hipStream_t s) {
    const size_t mat_bytes = ((size_t)N * N * 2 + 15) & ~(size_t)15;
    const size_t slice = flex_slice_bytes(N);
    const int fit = (int)((160 * 1024 - 512 - mat_bytes) / slice);
    if (fit < 1) return hipErrorInvalidValue;
    const int waves = waves_per_group(restarts, fit < kWavesPerGroup ? fit : kWavesPerGroup);
    const size_t lds = mat_bytes + (size_t)waves * slice;
    hipError_t e = hipFuncSetAttribute((const void*)twoopt_sum_flex_kernel<K>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int grid = (restarts + waves - 1) / waves;
    hipLaunchKernelGGL((twoopt_sum_flex_kernel<K>), dim3(grid), dim3(64 * waves), lds, s, c, N, restarts, tours, costs,
                       moves, flags);
    return hipGetLastError();
}

// Any 4 <= N <= 256.  Tours must already hold the initial orders, flags[0] the matrix maximum.
hipError_t launch_2opt_sum_flex(const int32_t* c, int N, int restarts, int32_t* tours, int64_t* costs, int32_t* moves,
                                const int32_t* flags, hipStream_t s) {
    if (N <= 64) return launch_flex_k<1>(c, N, restarts, tours, costs, moves, flags, s);
    if (N <= 128) return launch_flex_k<2>(c, N, restarts, tours, costs, moves, flags, s);
    if (N <= 192) return launch_flex_k<3>(c, N, restarts, tours, costs, moves, flags, s);
    return launch_flex_k<4>(c, N, restarts, tours, costs, moves, flags, s);
}

}  // namespace cc
