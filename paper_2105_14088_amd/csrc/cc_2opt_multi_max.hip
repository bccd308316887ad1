// 2-opt descent for N = 128, 192 and 256 under the bottleneck (max-hop) objective, directed or undirected: one
// wavefront per restart, K = N / 64 consecutive ranks per lane, the cost matrix staged once per workgroup in LDS as
// 16-bit entries (both triangles: the matrix need not be symmetric).
//
// The sweep is the cyclic-diagonal sweep of cc_2opt_n64_max.hip on the register layout of cc_2opt_multi.hip.
// Exchanging ring edges a and b = a + d (edge p joins ranks p-1 and p) cuts the ring into S1 = ranks a .. b-1 and
// S2 = ranks b .. a-1 and rejoins them with one piece reversed; as a directed ring the result can be walked two ways:
//   A: S2 as it is, S1 backwards:  new hops c[t[b-1]][t[a-1]], c[t[b]][t[a]];  S2's inner hops f, S1's b
//   B: the opposite direction:     new hops c[t[a-1]][t[b-1]], c[t[a]][t[b]];  S2's inner hops b, S1's f
// (f[p] = c[t[p]][t[p-1]] is hop p as walked now, b[p] = c[t[p-1]][t[p]] the same edge the other way).  Every word
// below carries both directions as two 16-bit halves and every maximum is a v_pk_max_u16: rank a gathers
// G = c[t[a]][t[b]] and GT = c[t[b]][t[a]] into P = G | GT << 16 and takes the (a-1, b-1) pair from rank a-1 (the
// same lane's previous register for K-1 ranks out of K, a wave rotate for the first);
//   S1's inner hops a+1 .. b-1 grow by one per diagonal: a running maximum over the hop words h = f | b << 16;
//   S2's inner hops b+1 .. a-1 are a cyclic window of N-d-1 hops: the maximum of two windows of 2^k hops,
//   [b+1, b+2^k] and [a-2^k, a-1], from a doubling table over the swapped hop words b | f << 16 that the wave builds
//   once per sweep in its LDS slice; k is the largest level with 2^k <= N-d-1 (the top level for most diagonals,
//   one below for the last ones).
// Values: lower half = B, upper half = A.  Per rank two running minima over value << 16 | rank(b); after the sweep
// they become (value, move id) with the ids of cc.h (orientation bit included) and the wave takes the
// lexicographic minimum.  On a symmetric matrix A = B and orientation 0 has the lower id, which is the undirected
// trajectory, so the kernel also serves the undirected max-hop objective.
// The undirected objective has a form of its own (DIRECTED = false): one direction only, so one gather per move, plain
// 32-bit maxima, one running minimum per rank; on the symmetric matrix that objective requires it takes the same
// decisions as the directed form.
// Needs max(c) < 2^16, else the general kernel runs instead (decided on the device, see launch code).
#include "cc_device.h"
#include "cc_internal.h"

namespace cc {
using namespace ccd;

namespace {

constexpr int kDppWaveRol1 = 0x134;     // lane p <- lane p+1 (cyclic over 64 lanes)
constexpr int kDppWaveRor1 = 0x13C;     // lane p <- lane p-1 (cyclic over 64 lanes)
__device__ __forceinline__ unsigned from_next_lane(unsigned v) {
    return (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, kDppWaveRol1, 0xf, 0xf, true);
}
__device__ __forceinline__ unsigned from_prev_lane(unsigned v) {
    return (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, kDppWaveRor1, 0xf, 0xf, true);
}
typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pk_max(unsigned a, unsigned b) {
    return __builtin_bit_cast(unsigned, __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, a),
                                                                  __builtin_bit_cast(ushort2_t, b)));
}
__device__ __forceinline__ int wave_min_all(int v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v = min(v, __shfl_xor(v, m, kWave));
    return v;
}
constexpr int floor_log2(int x) { return x <= 1 ? 0 : 1 + floor_log2(x >> 1); }
// Restarts per workgroup at most: they share one LDS copy of the matrix; the directed form needs more registers.
constexpr int max_waves(bool directed) { return directed ? 8 : 12; }

template <int K, bool DIRECTED>
__global__ __launch_bounds__(64 * max_waves(DIRECTED)) void twoopt_max_multi_kernel(
    const int32_t* __restrict__ c, int restarts, int with_flip, int32_t* __restrict__ tours,
    int64_t* __restrict__ costs, int32_t* __restrict__ moves, const int32_t* __restrict__ flags) {
    constexpr int N = 64 * K;
    constexpr int H = N / 2;
    constexpr int kTop = floor_log2(N - 3);           // level of the windows used by most diagonals
    constexpr int L1 = 1 << kTop, L0 = L1 >> 1;
    constexpr int kSwitch = N - L1;                   // from this diagonal on the windows are one level shorter
    static_assert(L0 <= H - 1 && 2 * L0 >= N - kSwitch - 1 && 2 * L1 >= N - 3, "two windows must cover S2's inner hops");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    if (flags[0] >= (1 << 16)) return;            // 16-bit staging impossible: the general kernel handles it
    uint16_t* mat = (uint16_t*)smem;                                   // [N][N]
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    // the wave's slice: the table under construction (N words) and the table one level below the top (N words), whose
    // place the order takes while a move is applied (by then the sweep holds everything it needs in registers)
    uint32_t* slice = (uint32_t*)(smem + (size_t)N * N * 2) + (size_t)wv * 2 * N;
    uint32_t* tk = slice;
    uint32_t* keep = slice + N;
    uint32_t* hs = keep;
    auto wmax = [](unsigned a, unsigned b) { return DIRECTED ? pk_max(a, b) : max(a, b); };
    for (int e = tid; e < N * N / 2; e += blockDim.x) {
        const int lo = clampi(c[2 * e], 0, 0xffff), hi = clampi(c[2 * e + 1], 0, 0xffff);
        ((uint32_t*)mat)[e] = (uint32_t)lo | ((uint32_t)hi << 16);
    }
    __syncthreads();
    const int64_t r = (int64_t)blockIdx.x * (blockDim.x >> 6) + wv;
    if (r >= restarts) return;
    const unsigned char* mbytes = (const unsigned char*)mat;
    auto wrap = [](int p) { return p >= N ? p - N : p; };          // p in [0, 2N)

    int t[K];
#pragma unroll
    for (int m = 0; m < K; ++m) t[m] = clampi(tours[r * N + K * lane + m], 0, N - 1);

    int cur = 0, applied = 0;
    bool first = true;
    for (;;) {
        // hop words of the lane's K ranks, both directions
        unsigned h[K];
        int rowofs[K], colofs[K];
        {
            const int tlast = (int)from_prev_lane((unsigned)t[K - 1]);
            int fmax = 0;
#pragma unroll
            for (int m = 0; m < K; ++m) {
                const int tp = m ? t[m - 1] : tlast;
                rowofs[m] = t[m] * (2 * N);
                colofs[m] = 2 * t[m];
                const unsigned f = *(const uint16_t*)(mbytes + rowofs[m] + 2 * tp);
                h[m] = f;
                if (DIRECTED) h[m] |= (unsigned)*(const uint16_t*)(mbytes + tp * (2 * N) + colofs[m]) << 16;
                fmax = max(fmax, (int)f);
            }
            if (first) {
                cur = wave_max(fmax);
                first = false;
            }
        }
        // doubling table over the swapped hop words: after level j, tk[p] = max over hops p .. p + 2^j - 1 (cyclic)
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int m = 0; m < K; ++m) tk[K * lane + m] = DIRECTED ? __builtin_amdgcn_alignbit(h[m], h[m], 16) : h[m];
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < kTop; ++j) {
            unsigned x[K], y[K];
#pragma unroll
            for (int m = 0; m < K; ++m) {
                x[m] = tk[K * lane + m];
                y[m] = tk[wrap(K * lane + m + ((1 << j) % N))];
            }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int m = 0; m < K; ++m) {
                if (j == kTop - 1) keep[K * lane + m] = x[m];
                tk[K * lane + m] = wmax(x[m], y[m]);
            }
            __builtin_amdgcn_wave_barrier();
        }
        // the window that ends at rank a-1, at both levels; the largest backward hop for the orientation flip
        unsigned far1[K], far0[K];
#pragma unroll
        for (int m = 0; m < K; ++m) {
            far1[m] = tk[wrap(K * lane + m + N - L1)];
            far0[m] = keep[wrap(K * lane + m + N - L0)];
        }
        unsigned flip_value = 0;
        if (DIRECTED && with_flip) {
            unsigned x = h[0];
#pragma unroll
            for (int m = 1; m < K; ++m) x = pk_max(x, h[m]);
            flip_value = (unsigned)wave_max((int)(x >> 16));
        }
        // partner windows: entries 0..K-1 belong to this lane's block of ranks, K..2K-1 to the next lane's
        unsigned tr[2 * K], tc[2 * K], hw[2 * K], kw[2 * K], wl[2 * K];
#pragma unroll
        for (int m = 0; m < K; ++m) {
            const int a = K * lane + m;
            tr[m] = (unsigned)rowofs[m];
            tc[m] = (unsigned)colofs[m];
            hw[m] = h[m];
            kw[m] = (unsigned)(a ? a - 1 : N - 1);
            wl[m] = tk[wrap(a + 1)];
        }
#pragma unroll
        for (int m = 0; m < K; ++m) {
            tr[K + m] = from_next_lane(tr[m]);
            tc[K + m] = from_next_lane(tc[m]);
            hw[K + m] = from_next_lane(hw[m]);
            kw[K + m] = from_next_lane(kw[m]);
            wl[K + m] = from_next_lane(wl[m]);
        }
        // N = 128, 256: the windows keep their length up to the last diagonal (kSwitch == H), and a move's value is the
        // maximum over both pieces anyway, so the fixed window that ends at a-1 starts the running maximum of S1 and
        // costs nothing per diagonal; the last diagonal, with its shorter windows, takes S1's inner hops from the table.
        constexpr bool kFold = kSwitch == H;
        unsigned s1[K], bestA[K], bestB[K], far[K];
#pragma unroll
        for (int m = 0; m < K; ++m) {
            s1[m] = hw[m + 1];                  // hop a+1: S1's only inner hop at d = 2
            bestA[m] = bestB[m] = 0xffffffffu;
            far[m] = far1[m];
            if (kFold) s1[m] = wmax(s1[m], far1[m]);
        }

        auto diagonal = [&](int rr, bool folded) {       // partner of slot m sits at window index m + rr
            unsigned P[K];
#pragma unroll
            for (int m = 0; m < K; ++m) {
                P[m] = *(const uint16_t*)(mbytes + rowofs[m] + tc[m + rr]);                                   // G
                if (DIRECTED) P[m] |= (unsigned)*(const uint16_t*)(mbytes + tr[m + rr] + colofs[m]) << 16;    // GT
            }
            const unsigned Plast = from_prev_lane(P[K - 1]);
#pragma unroll
            for (int m = 0; m < K; ++m) {
                const unsigned EP = m ? P[m - 1] : Plast;
                const unsigned s2 = folded ? wl[m + rr] : wmax(wl[m + rr], far[m]);
                const unsigned val = wmax(wmax(P[m], EP), wmax(s1[m], s2));
                if (DIRECTED) {
                    bestA[m] = min(bestA[m], (val & 0xffff0000u) | kw[m + rr]);
                    bestB[m] = min(bestB[m], (val << 16) | kw[m + rr]);
                } else {
                    bestA[m] = min(bestA[m], (val << 16) | kw[m + rr]);
                }
                s1[m] = wmax(s1[m], hw[m + rr]);        // the partner's hop is an inner hop of S1 from the next diagonal on
            }
        };
        auto slide = [&]() {
#pragma unroll
            for (int m = 0; m < K; ++m) {
                tr[m] = tr[K + m];
                tc[m] = tc[K + m];
                hw[m] = hw[K + m];
                kw[m] = kw[K + m];
                wl[m] = wl[K + m];
            }
#pragma unroll
            for (int m = 0; m < K; ++m) {
                tr[K + m] = from_next_lane(tr[m]);
                tc[K + m] = from_next_lane(tc[m]);
                hw[K + m] = from_next_lane(hw[m]);
                kw[K + m] = from_next_lane(kw[m]);
                wl[K + m] = from_next_lane(wl[m]);
            }
        };
        // from diagonal kSwitch on S2's inner hops are fewer than 2^kTop: both windows come from the table one level down
        auto shorter_windows = [&](int q) {              // window index j holds partner rank K * lane + K * q + j
#pragma unroll
            for (int j = 0; j < 2 * K; ++j) {
                int p = K * lane + K * q + j + 1;
                p = p >= N ? p - N : p;
                wl[j] = keep[p >= N ? p - N : p];
            }
#pragma unroll
            for (int m = 0; m < K; ++m) far[m] = far0[m];
        };
        // d = K*q + rr.  q = 0: only rr >= 2 (K = 2: nothing); q = 1 .. H/K - 1: all rr; q = H/K: rr = 0 (d = N/2)
#pragma unroll
        for (int rr = 2; rr < K; ++rr) diagonal(rr, kFold);
        slide();
        constexpr int kSwitchQ = kSwitch / K, kSwitchR = kSwitch % K;       // the block of diagonals that holds the switch
        auto blocks = [&](int q0, int q1) {
            asm("" : "+s"(q1));                // an opaque trip count: unrolled twice, never completely (register pressure)
#pragma unroll 2
            for (int q = q0; q < q1; ++q) {
#pragma unroll
                for (int rr = 0; rr < K; ++rr) diagonal(rr, kFold);
                slide();
            }
        };
        if (kSwitch < H) {
            blocks(1, kSwitchQ);
#pragma unroll
            for (int rr = 0; rr < K; ++rr) {
                if (rr == kSwitchR) shorter_windows(kSwitchQ);
                diagonal(rr, false);
            }
            slide();
            blocks(kSwitchQ + 1, H / K);
        } else {
            blocks(1, H / K);
        }
        if (kSwitch == H) {
            shorter_windows(H / K);
            // S1's inner hops a+1 .. a+H-1 without the fixed window: two windows of L0 = H / 2 hops from the table one level
            // down, whose words carry the two directions the other way round
#pragma unroll
            for (int m = 0; m < K; ++m) {
                const int a = K * lane + m;
                const unsigned x = wmax(keep[wrap(a + 1)], keep[wrap(a + H - L0)]);
                s1[m] = DIRECTED ? __builtin_amdgcn_alignbit(x, x, 16) : x;
            }
        }
        diagonal(0, false);

        // per rank and direction: best partner -> move id; then the lexicographic minimum of (value, id) over the wave
        int bv = 0x7fffffff, bid = 0x7fffffff;
#pragma unroll
        for (int m = 0; m < K; ++m) {
            const int a = K * lane + m;
            const int rank_a = a ? a - 1 : N - 1;
#pragma unroll
            for (int which = 0; which < (DIRECTED ? 2 : 1); ++which) {
                const unsigned key = which ? bestB[m] : bestA[m];
                const int kv = (int)(key >> 16), rk = (int)(key & 0xffffu);
                const bool wrapped = rk < rank_a;         // b lies before a: the reversed piece is S2, not S1
                const int ij = wrapped ? (rk + 1) * N + rank_a : a * N + rk;
                const int id = ij * 2 + (DIRECTED ? which ^ (wrapped ? 1 : 0) : 0);
                const bool better = kv < bv || (kv == bv && id < bid);
                bv = better ? kv : bv;
                bid = better ? id : bid;
            }
        }
        if (DIRECTED && with_flip && lane == 0) {       // the orientation flip: every hop walked the other way
            const int vf = (int)flip_value, idf = (N + N - 1) * 2;
            const bool better = vf < bv || (vf == bv && idf < bid);
            bv = better ? vf : bv;
            bid = better ? idf : bid;
        }
        const int vwin = wave_min_all(bv);
        if (vwin >= cur) break;
        const int idwin = wave_min_all(bv == vwin ? bid : 0x7fffffff);
        const int o = idwin & 1, ij = idwin >> 1, mi = ij / N, mj = ij % N;
        // new[p] = old[src(p)] through the wave's LDS slice
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int m = 0; m < K; ++m) hs[K * lane + m] = (uint32_t)t[m];
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int m = 0; m < K; ++m) {
            const int a = K * lane + m;
            const int p0 = o ? (a ? N - a : 0) : a;
            const int src = (p0 >= mi && p0 <= mj) ? mi + mj - p0 : p0;
            t[m] = (int)hs[src];
        }
        __builtin_amdgcn_wave_barrier();
        cur = vwin;
        ++applied;
    }
#pragma unroll
    for (int m = 0; m < K; ++m) tours[r * N + K * lane + m] = t[m];
    if (lane == 0) {
        costs[r] = (int64_t)cur;
        moves[r] = applied;
    }
}

template <int K, bool DIRECTED>
hipError_t launch_k(const int32_t* c, int restarts, bool with_flip, int32_t* tours, int64_t* costs, int32_t* moves,
                    const int32_t* flags, hipStream_t s) {
    constexpr int N = 64 * K;
    // restarts per workgroup: as many as share one LDS copy of the matrix, but no more than keeps all compute units busy
    int waves = (restarts + 255) / 256;
    waves = waves < 1 ? 1 : (waves > max_waves(DIRECTED) ? max_waves(DIRECTED) : waves);
    const size_t lds = (size_t)N * N * 2 + (size_t)waves * 2 * N * sizeof(uint32_t);
    hipError_t e = hipFuncSetAttribute((const void*)twoopt_max_multi_kernel<K, DIRECTED>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int grid = (restarts + waves - 1) / waves;
    hipLaunchKernelGGL((twoopt_max_multi_kernel<K, DIRECTED>), dim3(grid), dim3(64 * waves), lds, s, c, restarts,
                       with_flip ? 1 : 0, tours, costs, moves, flags);
    return hipGetLastError();
}

}  // namespace

// N = 128, 192 or 256.  Tours must already hold the initial orders; flags[0] must hold the matrix maximum
// (launch_matrix_max): the kernel returns at once if it is 2^16 or more.
hipError_t launch_2opt_max_multi(const int32_t* c, int N, bool directed, int restarts, bool with_flip, int32_t* tours,
                                 int64_t* costs, int32_t* moves, const int32_t* flags, hipStream_t s) {
    if (directed) {
        if (N == 128) return launch_k<2, true>(c, restarts, with_flip, tours, costs, moves, flags, s);
        if (N == 192) return launch_k<3, true>(c, restarts, with_flip, tours, costs, moves, flags, s);
        return launch_k<4, true>(c, restarts, with_flip, tours, costs, moves, flags, s);
    }
    if (N == 128) return launch_k<2, false>(c, restarts, false, tours, costs, moves, flags, s);
    if (N == 192) return launch_k<3, false>(c, restarts, false, tours, costs, moves, flags, s);
    return launch_k<4, false>(c, restarts, false, tours, costs, moves, flags, s);
}

}  // namespace cc
