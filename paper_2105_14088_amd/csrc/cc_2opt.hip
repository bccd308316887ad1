// Multi-start best-improvement 2-opt over the ring (Section 4.3 neighbour search; move set, value
// and tie-break rules as stated in cc.h).
//
// General kernel: one workgroup per restart, one thread per rank.  Tour, hop arrays and the prefix /
// suffix tables live in LDS; thread j scores the moves (i, j) for i = j-1 down to 1 so that the
// "inside the reversed span" aggregate grows by one hop per step; keys (value << 32 | move id) are
// min-reduced over the workgroup, which makes the lowest-id tie-break independent of the order in
// which moves are visited.  Handles every objective and every N <= 1024; the matrix sits in LDS for
// N <= 96 and is gathered through L2 above.
#include <cstdlib>
#include <cstring>

#include "cc_device.h"
#include "cc_internal.h"

namespace cc {
using namespace ccd;

namespace {

constexpr unsigned long long kNoMove = ~0ull;
// Up to this N the general kernel keeps the matrix in LDS: 7 N + N^2 int32 words are then at most 40 KiB, so four
// workgroups still share a compute unit (measured at 1024 restarts: N = 96 1.75x faster than through L2, N = 100,
// where only three fit, no faster).
constexpr int kGeneralLdsMatrixMaxN = 96;

template <bool IS_MAX>
__device__ __forceinline__ int comb(int a, int b) { return IS_MAX ? max(a, b) : a + b; }

// In-place inclusive scan over arr[0..N) (forward: arr[p] = op(arr[0..p]); backward: op(arr[p..N-1])).
// Every thread of the workgroup must call it; blockDim.x >= N.
template <bool IS_MAX, bool BACKWARD>
__device__ void block_scan(int32_t* arr, int N) {
    const int p = threadIdx.x;
    for (int off = 1; off < N; off <<= 1) {
        int v = 0, w = 0;
        bool has = false;
        if (p < N) {
            v = arr[p];
            const int src = BACKWARD ? p + off : p - off;
            has = BACKWARD ? (src < N) : (src >= 0);
            if (has) w = arr[src];
        }
        __syncthreads();
        if (p < N && has) arr[p] = comb<IS_MAX>(v, w);
        __syncthreads();
    }
}

// LDS_MATRIX: the matrix is staged once per workgroup in LDS behind the seven rank arrays (small N).
template <int OBJ, bool LDS_MATRIX>
__global__ void twoopt_general_kernel(const int32_t* __restrict__ c, int N, int32_t* __restrict__ tours,
                                      int64_t* __restrict__ costs, int32_t* __restrict__ moves,
                                      const int32_t* __restrict__ skip_if_small, int with_flip, int small_limit) {
    // when a fast path is launched beside this kernel, flags[0] = max(c) decides which of the two runs: the fast one
    // takes the matrices whose largest entry is below small_limit
    if (skip_if_small && skip_if_small[0] < small_limit) return;
    constexpr bool IS_MAX = (OBJ & 1) != 0;
    constexpr bool DIRECTED = (OBJ & 2) != 0;
    extern __shared__ int32_t sm[];
    int32_t* t = sm;           // tour
    int32_t* f = t + N;        // f[p] = c[t[p]][t[p-1]]
    int32_t* b = f + N;        // b[p] = c[t[p-1]][t[p]]
    int32_t* pf = b + N;       // SUM: inclusive prefix sum of f;  MAX: max f over ranks 1..p (0 at p = 0)
    int32_t* pb = pf + N;      // same for b
    int32_t* sf = pb + N;      // MAX: max f over ranks p..N-1
    int32_t* sb = sf + N;      // same for b
    __shared__ unsigned long long red[16];
    __shared__ unsigned long long winner;
    __shared__ int red_cost[16];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6, nwv = blockDim.x >> 6;
    const int64_t r = blockIdx.x;
    // entries are clamped to the contract range: all int32 arithmetic below is then exact, every applied
    // move lowers the true cost, and the descent terminates whatever the buffer holds
    int32_t* m = sb + N;
    // the ring-sum objective reads the matrix through its upper triangle (exact deltas, hence a descent that ends,
    // whatever the caller's matrix holds); the other objectives score true values of the orders they produce
    constexpr bool UPPER = OBJ == 0;
    if (LDS_MATRIX)
        for (int e = tid; e < N * N; e += blockDim.x) m[e] = clampi(c[UPPER ? upper_index(e, N) : e], 0, (1 << 21) - 1);
    auto C = [&](int a, int b2) {
        if (LDS_MATRIX) return m[a * N + b2];
        return clampi(UPPER ? c[min(a, b2) * N + max(a, b2)] : c[a * N + b2], 0, (1 << 21) - 1);
    };
    if (tid < N) t[tid] = clampi(tours[r * N + tid], 0, N - 1);
    __syncthreads();

    int cur = 0;
    int applied = 0;
    bool first = true;
    for (;;) {
        // ---- hop arrays and tables for the current tour
        int myf = 0;
        if (tid < N) {
            const int a = t[tid], pr = t[tid ? tid - 1 : N - 1];
            myf = C(a, pr);
            f[tid] = myf;
            if (DIRECTED) b[tid] = C(pr, a);
            if (DIRECTED || IS_MAX) {
                pf[tid] = (IS_MAX && tid == 0) ? 0 : myf;
                if (IS_MAX) sf[tid] = myf;
            }
        }
        __syncthreads();
        if (DIRECTED && tid < N) {
            pb[tid] = (IS_MAX && tid == 0) ? 0 : b[tid];
            if (IS_MAX) sb[tid] = b[tid];
        }
        if (DIRECTED || IS_MAX) {
            __syncthreads();
            block_scan<IS_MAX, false>(pf, N);
            if (DIRECTED) block_scan<IS_MAX, false>(pb, N);
            if (IS_MAX) {
                block_scan<true, true>(sf, N);
                if (DIRECTED) block_scan<true, true>(sb, N);
            }
        }
        if (first) {   // cost of the initial tour (afterwards the winning move's value is the cost)
            int v = IS_MAX ? wave_max(myf) : wave_sum(myf);
            if (lane == 0) red_cost[wv] = v;
            __syncthreads();
            v = 0;
            for (int k = 0; k < nwv; ++k) v = comb<IS_MAX>(v, red_cost[k]);
            cur = v;
            first = false;
        }

        // ---- score column j = tid of the neighbourhood
        unsigned long long best = kNoMove;
        const int j = tid;
        if (j >= 2 && j < N) {
            const int q = (j + 1 == N) ? 0 : j + 1;
            const int tj = t[j], tq = t[q];
            const int fq = f[q];
            const int bq = DIRECTED ? b[q] : 0;
            const int tot_f = (!IS_MAX && DIRECTED) ? pf[N - 1] : 0;
            const int tot_b = (!IS_MAX && DIRECTED) ? pb[N - 1] : 0;
            const int pfj = (!IS_MAX && DIRECTED) ? pf[j] : 0;
            const int pbj = (!IS_MAX && DIRECTED) ? pb[j] : 0;
            // MAX: hops outside the span on the far side (ranks j+2..N-1) and rank 0 unless it is q
            int far_f = 0, far_b = 0;
            if (IS_MAX && q != 0) {
                far_f = f[0];
                if (j + 2 <= N - 1) far_f = max(far_f, sf[j + 2]);
                if (DIRECTED) {
                    far_b = b[0];
                    if (j + 2 <= N - 1) far_b = max(far_b, sb[j + 2]);
                }
            }
            int in_f = 0, in_b = 0;
            for (int i = j - 1; i >= 1; --i) {
                if (IS_MAX) {                       // inside = ranks i+1..j
                    in_f = max(in_f, f[i + 1]);
                    if (DIRECTED) in_b = max(in_b, b[i + 1]);
                }
                if (i == 1 && j == N - 1) continue;
                const int ti = t[i], tim = t[i - 1];
                const int x0 = C(tj, tim), y0 = C(tq, ti);
                int v0, v1 = 0;
                if (!IS_MAX && !DIRECTED) {
                    v0 = cur + x0 + y0 - f[i] - fq;
                } else if (!IS_MAX) {
                    const int x1 = C(tim, tj), y1 = C(ti, tq);
                    const int inf = pfj - pf[i], inb = pbj - pb[i];
                    const int outf = tot_f - f[i] - fq - inf, outb = tot_b - b[i] - bq - inb;
                    v0 = x0 + y0 + outf + inb;
                    v1 = x1 + y1 + outb + inf;
                } else if (!DIRECTED) {
                    const int outf = max(far_f, pf[i - 1]);
                    v0 = max(max(x0, y0), max(outf, in_f));
                } else {
                    const int x1 = C(tim, tj), y1 = C(ti, tq);
                    const int outf = max(far_f, pf[i - 1]), outb = max(far_b, pb[i - 1]);
                    v0 = max(max(x0, y0), max(outf, in_b));
                    v1 = max(max(x1, y1), max(outb, in_f));
                }
                const unsigned id = (unsigned)(i * N + j);
                if (DIRECTED) {
                    const unsigned long long k0 = ((unsigned long long)(unsigned)v0 << 32) | (id * 2u);
                    const unsigned long long k1 = ((unsigned long long)(unsigned)v1 << 32) | (id * 2u + 1u);
                    best = min(best, min(k0, k1));
                } else {
                    best = min(best, ((unsigned long long)(unsigned)v0 << 32) | id);
                }
            }
        }
        // the orientation flip, the pair (1, N-1) that the move set leaves out: every hop walked the other way
        if (DIRECTED && with_flip && tid == 0 && N >= 3) {
            const int v = IS_MAX ? max(pb[N - 1], b[0]) : pb[N - 1];
            best = ((unsigned long long)(unsigned)v << 32) | ((unsigned)(N + N - 1) * 2u);
        }
        best = wave_min_u64(best);
        if (lane == 0) red[wv] = best;
        __syncthreads();
        if (tid == 0) {
            unsigned long long m = red[0];
            for (int k = 1; k < nwv; ++k) m = min(m, red[k]);
            winner = m;
        }
        __syncthreads();
        const unsigned long long win = winner;
        if (win == kNoMove || (long long)(win >> 32) >= (long long)cur) break;

        // ---- apply the winning move: new[p] = old[src(p)]
        unsigned id = (unsigned)(win & 0xffffffffu);
        const int o = DIRECTED ? (int)(id & 1u) : 0;
        if (DIRECTED) id >>= 1;
        const int mi = (int)(id / (unsigned)N), mj = (int)(id % (unsigned)N);
        int val = 0;
        if (tid < N) {
            const int p0 = o ? (tid == 0 ? 0 : N - tid) : tid;
            const int src = (p0 >= mi && p0 <= mj) ? mi + mj - p0 : p0;
            val = t[src];
        }
        __syncthreads();
        if (tid < N) t[tid] = val;
        __syncthreads();
        cur = (int)(win >> 32);
        ++applied;
    }
    if (tid < N) tours[r * N + tid] = t[tid];
    if (tid == 0) {
        costs[r] = (int64_t)cur;
        moves[r] = applied;
    }
}

// Lexicographic minimum of (cost, restart) over all restarts; copies the winner's tour.  One workgroup of 256 or
// (many restarts) 1024 threads: strided loads, a shuffle reduction inside each wave, the waves' results through LDS.
__global__ __launch_bounds__(1024) void best_restart_kernel(const int64_t* __restrict__ costs,
                                                            const int32_t* __restrict__ tours, int N, int restarts,
                                                            int32_t* __restrict__ best_perm,
                                                            int64_t* __restrict__ best_cost,
                                                            int32_t* __restrict__ best_restart) {
    __shared__ long long sc[16];
    __shared__ int sr[16];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, nwv = blockDim.x >> 6, stride = blockDim.x;
    long long bc = 0x7fffffffffffffffll;
    int br = 0x7fffffff;
    auto take = [&](long long v, int r) {
        if (v < bc || (v == bc && r < br)) { bc = v; br = r; }
    };
    int r = tid;
    for (; r + 3 * stride < restarts; r += 4 * stride) {      // four loads in flight
        const long long v0 = costs[r], v1 = costs[r + stride], v2 = costs[r + 2 * stride], v3 = costs[r + 3 * stride];
        take(v0, r);
        take(v1, r + stride);
        take(v2, r + 2 * stride);
        take(v3, r + 3 * stride);
    }
    for (; r < restarts; r += stride) take(costs[r], r);
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        const long long v = __shfl_xor(bc, m, kWave);
        const int rr = __shfl_xor(br, m, kWave);
        take(v, rr);
    }
    if (lane == 0) {
        sc[wv] = bc;
        sr[wv] = br;
    }
    __syncthreads();
    bc = sc[0];
    br = sr[0];
    for (int k = 1; k < nwv; ++k) take(sc[k], sr[k]);
    const int win = br;
    for (int p = tid; p < N; p += stride) best_perm[p] = tours[(int64_t)win * N + p];
    if (tid == 0) {
        best_cost[0] = bc;
        if (best_restart) best_restart[0] = win;
    }
}

template <int OBJ>
hipError_t launch_general(const int32_t* c, int N, int restarts, int32_t* tours, int64_t* costs, int32_t* moves,
                          const int32_t* skip_if_small, int with_flip, int small_limit, hipStream_t s) {
    const int threads = ((N + 63) / 64) * 64;
    if (N <= kGeneralLdsMatrixMaxN) {
        const size_t lds = sizeof(int32_t) * (7 * (size_t)N + (size_t)N * N);
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute((const void*)twoopt_general_kernel<OBJ, true>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL((twoopt_general_kernel<OBJ, true>), dim3(restarts), dim3(threads), lds, s, c, N, tours, costs,
                           moves, skip_if_small, with_flip, small_limit);
    } else {
        const size_t lds = sizeof(int32_t) * 7 * (size_t)N;
        hipLaunchKernelGGL((twoopt_general_kernel<OBJ, false>), dim3(restarts), dim3(threads), lds, s, c, N, tours, costs,
                           moves, skip_if_small, with_flip, small_limit);
    }
    return hipGetLastError();
}

hipError_t launch_general_objective(const int32_t* c, int N, int objective, int restarts, int32_t* tours,
                                    int64_t* costs, int32_t* moves, const int32_t* skip_if_small, bool with_flip,
                                    hipStream_t s, int small_limit = 1 << 16) {
    const int flip = with_flip ? 1 : 0;
    switch (objective) {
        case 0: return launch_general<0>(c, N, restarts, tours, costs, moves, skip_if_small, 0, small_limit, s);
        case 1: return launch_general<1>(c, N, restarts, tours, costs, moves, skip_if_small, 0, small_limit, s);
        case 2: return launch_general<2>(c, N, restarts, tours, costs, moves, skip_if_small, flip, small_limit, s);
        default: return launch_general<3>(c, N, restarts, tours, costs, moves, skip_if_small, flip, small_limit, s);
    }
}

}  // namespace

bool force_general_path() {
    const char* v = getenv("CC_FORCE_PATH");
    return v && strcmp(v, "general") == 0;
}

hipError_t launch_best_restart(const int64_t* costs, const int32_t* tours, int N, int restarts, int32_t* best_perm,
                               int64_t* best_cost, int32_t* best_restart, hipStream_t s) {
    hipLaunchKernelGGL(best_restart_kernel, dim3(1), dim3(restarts > 1024 ? 1024 : 256), 0, s, costs, tours, N, restarts,
                       best_perm, best_cost, best_restart);
    return hipGetLastError();
}

hipError_t launch_2opt(const int32_t* c, int N, int objective, int classes, int restarts, uint64_t seed,
                       bool tours_hold_init, int32_t* tours, int64_t* costs, int32_t* moves, int32_t* flags,
                       uint16_t* mat16, int32_t* best_perm, int64_t* best_cost, int32_t* best_restart, hipStream_t s) {
    hipError_t e;
    const bool flip = classes == (kMoves2opt | kMovesFlip);      // only defined with the directed objectives
    if (force_general_path() && !(classes & kMovesOropt)) {
        if (!tours_hold_init) {
            e = launch_init_tours(N, 0, restarts, seed, tours, s);
            if (e != hipSuccess) return e;
        }
        e = launch_general_objective(c, N, objective, restarts, tours, costs, moves, nullptr, flip, s);
    } else if (flip && N == 64 && objective == 3) {
        e = launch_2opt_max_n64(c, restarts, seed, !tours_hold_init, true, tours, costs, moves, s);
    } else if ((flip || classes == kMoves2opt) && N == 64 && objective == 2) {
        // directed sum: wavefront kernel with 32-bit keys when max(c) < 2^16, else the general kernel (both enqueued,
        // the matrix maximum computed on the device decides)
        if (!tours_hold_init) {
            e = launch_init_tours(N, 0, restarts, seed, tours, s);
            if (e != hipSuccess) return e;
        }
        e = launch_matrix_max(c, N, flags, s);
        if (e != hipSuccess) return e;
        e = launch_2opt_dsum_n64(c, restarts, seed, false, flip, tours, costs, moves, flags, s);
        if (e != hipSuccess) return e;
        e = launch_general_objective(c, N, objective, restarts, tours, costs, moves, flags, flip, s);
    } else if ((flip || classes == kMoves2opt) && (objective & 1) && (N == 128 || N == 192 || N == 256)) {
        // max-hop at 128 / 192 / 256: several ranks per lane with a 16-bit LDS matrix when max(c) < 2^16, else the
        // general kernel (both enqueued, the matrix maximum computed on the device decides)
        if (!tours_hold_init) {
            e = launch_init_tours(N, 0, restarts, seed, tours, s);
            if (e != hipSuccess) return e;
        }
        e = launch_matrix_max(c, N, flags, s);
        if (e != hipSuccess) return e;
        e = launch_2opt_max_multi(c, N, (objective & 2) != 0, restarts, flip, tours, costs, moves, flags, s);
        if (e != hipSuccess) return e;
        e = launch_general_objective(c, N, objective, restarts, tours, costs, moves, flags, flip, s);
    } else if ((flip || classes == kMoves2opt) && objective == 2 && (N == 128 || N == 192 || N == 256)) {
        // directed sum at 128 / 192 / 256: several ranks per lane with a 16-bit LDS matrix when its 32-bit keys hold
        // every partial delta, else the general kernel (both enqueued, the matrix maximum decides)
        if (!tours_hold_init) {
            e = launch_init_tours(N, 0, restarts, seed, tours, s);
            if (e != hipSuccess) return e;
        }
        e = launch_matrix_max(c, N, flags, s);
        if (e != hipSuccess) return e;
        e = launch_2opt_dsum_multi(c, N, restarts, flip, tours, costs, moves, flags, s);
        if (e != hipSuccess) return e;
        e = launch_general_objective(c, N, objective, restarts, tours, costs, moves, flags, flip, s, dsum_multi_limit(N));
    } else if (classes != kMoves2opt) {
        // wider move sets: the segment-insertion kernel (ring sum) or the general kernel with the orientation flip
        if (!tours_hold_init) {
            e = launch_init_tours(N, 0, restarts, seed, tours, s);
            if (e != hipSuccess) return e;
        }
        if (classes & kMovesOropt)
            e = launch_insertion_search(c, N, (classes & kMoves2opt) != 0, restarts, tours, costs, moves, flags, s);
        else
            e = launch_general_objective(c, N, objective, restarts, tours, costs, moves, nullptr, true, s);
    } else if (N == 64 && objective == 0) {
        e = launch_2opt_sum_n64(c, restarts, seed, !tours_hold_init, tours, costs, moves, s);
    } else if (N == 64 && (objective & 1)) {
        e = launch_2opt_max_n64(c, restarts, seed, !tours_hold_init, false, tours, costs, moves, s);
    } else {
        if (!tours_hold_init) {
            e = launch_init_tours(N, 0, restarts, seed, tours, s);
            if (e != hipSuccess) return e;
        }
        if (objective == 0 && (N == 128 || N == 192 || N == 256)) {
            // 16-bit LDS matrix path when max(c) < 2^16, else the general kernel: both are enqueued and the
            // matrix maximum, computed on the device, decides which one does the work (no host round trip)
            e = launch_matrix_max(c, N, flags, s);
            if (e != hipSuccess) return e;
            e = launch_2opt_sum_multi(c, N, restarts, tours, costs, moves, flags, s);
            if (e != hipSuccess) return e;
            e = launch_general_objective(c, N, objective, restarts, tours, costs, moves, flags, false, s);
        } else if (objective == 0 && N >= 4 && N <= 256) {
            e = launch_matrix_max(c, N, flags, s);
            if (e != hipSuccess) return e;
            e = launch_2opt_sum_flex(c, N, restarts, tours, costs, moves, flags, s);
            if (e != hipSuccess) return e;
            e = launch_general_objective(c, N, objective, restarts, tours, costs, moves, flags, false, s);
        } else if (objective == 0 && (N == 512 || N == 1024)) {
            e = launch_matrix_max(c, N, flags, s);
            if (e != hipSuccess) return e;
            e = launch_2opt_sum_n1024(c, N, mat16, restarts, tours, costs, moves, flags, s);
            if (e != hipSuccess) return e;
            e = launch_general_objective(c, N, objective, restarts, tours, costs, moves, flags, false, s);
        } else {
            e = launch_general_objective(c, N, objective, restarts, tours, costs, moves, nullptr, false, s);
        }
    }
    if (e != hipSuccess) return e;
    if (!best_perm) return hipSuccess;       // per-restart results only
    return launch_best_restart(costs, tours, N, restarts, best_perm, best_cost, best_restart, s);
}

}  // namespace cc
