// Best-improvement descent over segment insertions (Or-opt), alone or together with the 2-opt moves, for the
// ring-sum objective on a symmetric matrix (Section 4.3: neighbour search "alongside standard heuristics"; move
// set, ids, values and tie-breaks as stated in cc.h, cc_local_search).
//
// One workgroup per restart, one thread per rank.  Thread s owns the segments that start at rank s (lengths 1, 2, 3)
// and walks the gaps g = 0 .. N-1 once: per gap it gathers the three entries c[t[g+1]][t[s+k]], k = 0, 1, 2, keeps
// the previous gap's three as c[t[g]][t[s+k]], and scores the five variants (length 1; lengths 2 and 3 kept or
// reversed) with adds only.  The node and hop of a gap are the same for all threads (LDS broadcast reads), the three
// gathers of a gap lie in one matrix row.  Thread j also scores the 2-opt moves (i, j) when they are enabled.  Keys
// (value << 32 | id) are min-reduced over the workgroup, so the result is the lexicographic minimum whatever the
// visiting order.  The matrix sits in LDS for N <= 96 and is gathered through L2 above.
#include "cc_device.h"
#include "cc_internal.h"

namespace cc {
using namespace ccd;

namespace {

constexpr unsigned long long kNoMove = ~0ull;
constexpr int kLdsMatrixMaxN = 96;
constexpr int kCostMax = (1 << 21) - 1;

__device__ __forceinline__ unsigned long long key_of(int value, unsigned id) {
    return ((unsigned long long)(unsigned)value << 32) | id;
}

template <bool WITH_2OPT, bool LDS_MATRIX>
__global__ void insertion_search_kernel(const int32_t* __restrict__ c, int N, int32_t* __restrict__ tours,
                                        int64_t* __restrict__ costs, int32_t* __restrict__ moves,
                                        const int32_t* __restrict__ skip_if_small) {
    // when the 16-bit fast path is launched beside this kernel, skip_if_small[0] = max(c) decides which one runs
    if (skip_if_small && skip_if_small[0] < (1 << 16)) return;
    extern __shared__ int32_t sm[];
    int32_t* t = sm;            // tour
    int32_t* f = t + N;         // f[p] = c[t[p]][t[p-1]]
    int32_t* m = f + N;         // matrix (LDS_MATRIX only)
    __shared__ unsigned long long red[16];
    __shared__ unsigned long long winner;
    __shared__ int red_cost[16];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6, nwv = blockDim.x >> 6;
    const int64_t r = blockIdx.x;
    // entries are clamped to the contract range: all int32 arithmetic is then exact, every applied move lowers
    // the true cost, and the descent ends whatever the buffer holds
    // and the matrix is read through its upper triangle, so the deltas are exact for the matrix the kernel sees
    if (LDS_MATRIX)
        for (int e = tid; e < N * N; e += blockDim.x) m[e] = clampi(c[upper_index(e, N)], 0, kCostMax);
    auto C = [&](int a, int b) {
        return LDS_MATRIX ? m[a * N + b] : clampi(c[min(a, b) * N + max(a, b)], 0, kCostMax);
    };
    if (tid < N) t[tid] = clampi(tours[r * N + tid], 0, N - 1);
    __syncthreads();

    const int max_len = min(3, N - 3);      // longest segment
    const unsigned nn = (unsigned)N * (unsigned)N;
    int cur = 0, applied = 0;
    bool first = true;
    for (;;) {
        int myf = 0;
        if (tid < N) {
            myf = C(t[tid], t[tid ? tid - 1 : N - 1]);
            f[tid] = myf;
        }
        __syncthreads();
        if (first) {
            const int v = wave_sum(myf);
            if (lane == 0) red_cost[wv] = v;
            __syncthreads();
            cur = 0;
            for (int k = 0; k < nwv; ++k) cur += red_cost[k];
            first = false;
        }

        unsigned long long best = kNoMove;
        // ---- 2-opt moves (i, j), j = tid: reverse ranks i .. j
        if (WITH_2OPT && tid >= 2 && tid < N) {
            const int j = tid, q = (j + 1 == N) ? 0 : j + 1;
            const int tj = t[j], tq = t[q];
            const int base = cur - f[q];
            for (int i = j - 1; i >= 1; --i) {
                if (i == 1 && j == N - 1) continue;
                const int v = base + C(tj, t[i - 1]) + C(tq, t[i]) - f[i];
                best = min(best, key_of(v, (unsigned)(i * N + j)));
            }
        }
        // ---- segment insertions, segment start s = tid
        if (tid >= 1 && tid < N && max_len >= 1) {
            const int s = tid;
            const int len = min(max_len, N - s);           // segments must end at rank N-1 at the latest
            const int a = t[s - 1];
            const int s0 = t[s], s1 = t[min(s + 1, N - 1)], s2 = t[min(s + 2, N - 1)];
            // cost of the ring once the segment of length L is cut out and its neighbours are joined
            int without[3];
#pragma unroll
            for (int L = 1; L <= 3; ++L) {
                const int behind = (s + L >= N) ? s + L - N : s + L;      // only read when L <= len (then <= N-1 or 0)
                without[L - 1] = L <= len ? cur - f[s] - f[behind] + C(a, t[behind]) : 0;
            }
            const unsigned id_s = nn + (unsigned)s * (unsigned)N;
            int p0 = C(t[0], s0), p1 = C(t[0], s1), p2 = C(t[0], s2);      // entries of the gap's first node
            for (int g = 0; g < N; ++g) {
                const int gq = (g + 1 == N) ? 0 : g + 1;
                const int row = t[gq];
                const int q0 = C(row, s0), q1 = C(row, s1), q2 = C(row, s2);
                const int open = f[gq];                    // the edge the gap opens
                const int d = g - (s - 1);                 // gaps s-1 .. s+L-1 touch the segment: d in 0 .. L
                if (d < 0 || d > 1)
                    best = min(best, key_of(without[0] - open + p0 + q0, id_s + (unsigned)g));
                if (len >= 2 && (d < 0 || d > 2)) {
                    best = min(best, key_of(without[1] - open + p0 + q1, id_s + 1u * nn + (unsigned)g));
                    best = min(best, key_of(without[1] - open + p1 + q0, id_s + 2u * nn + (unsigned)g));
                }
                if (len >= 3 && (d < 0 || d > 3)) {
                    best = min(best, key_of(without[2] - open + p0 + q2, id_s + 3u * nn + (unsigned)g));
                    best = min(best, key_of(without[2] - open + p2 + q0, id_s + 4u * nn + (unsigned)g));
                }
                p0 = q0;
                p1 = q1;
                p2 = q2;
            }
        }
        best = wave_min_u64(best);
        if (lane == 0) red[wv] = best;
        __syncthreads();
        if (tid == 0) {
            unsigned long long w = red[0];
            for (int k = 1; k < nwv; ++k) w = min(w, red[k]);
            winner = w;
        }
        __syncthreads();
        const unsigned long long win = winner;
        if (win == kNoMove || (long long)(win >> 32) >= (long long)cur) break;

        // ---- apply: new[p] = old[src(p)]
        const int id = (int)(win & 0xffffffffu);
        const int val = tid < N ? t[move_source(tid, id, N)] : 0;
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

template <bool WITH_2OPT>
hipError_t launch_insertion(const int32_t* c, int N, int restarts, int32_t* tours, int64_t* costs, int32_t* moves,
                            const int32_t* skip_if_small, hipStream_t s) {
    const int threads = ((N + 63) / 64) * 64;
    if (N <= kLdsMatrixMaxN) {
        const size_t lds = sizeof(int32_t) * (2 * (size_t)N + (size_t)N * N);
        hipLaunchKernelGGL((insertion_search_kernel<WITH_2OPT, true>), dim3(restarts), dim3(threads), lds, s, c, N, tours,
                           costs, moves, skip_if_small);
    } else {
        const size_t lds = sizeof(int32_t) * 2 * (size_t)N;
        hipLaunchKernelGGL((insertion_search_kernel<WITH_2OPT, false>), dim3(restarts), dim3(threads), lds, s, c, N,
                           tours, costs, moves, skip_if_small);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_insertion_search(const int32_t* c, int N, bool with_2opt, int restarts, int32_t* tours,
                                   int64_t* costs, int32_t* moves, int32_t* flags, hipStream_t s) {
    const int32_t* skip = nullptr;
    if (force_general_path()) {
        // pinned: the kernel below for every size
    } else if (N == 64) {
        // one wavefront per restart with 32-bit keys when max(c) < 2^16, else the kernel above: both are enqueued
        // and the matrix maximum, computed on the device, decides which of them does the work
        hipError_t e = launch_matrix_max(c, N, flags, s);
        if (e != hipSuccess) return e;
        e = launch_local_n64(c, with_2opt, restarts, tours, costs, moves, flags, s);
        if (e != hipSuccess) return e;
        skip = flags;
    } else if (N == 128 || N == 192 || N == 256) {
        hipError_t e = launch_matrix_max(c, N, flags, s);
        if (e != hipSuccess) return e;
        e = launch_local_multi(c, N, with_2opt, restarts, tours, costs, moves, flags, s);
        if (e != hipSuccess) return e;
        skip = flags;
    }
    return with_2opt ? launch_insertion<true>(c, N, restarts, tours, costs, moves, skip, s)
                     : launch_insertion<false>(c, N, restarts, tours, costs, moves, skip, s);
}

}  // namespace cc
