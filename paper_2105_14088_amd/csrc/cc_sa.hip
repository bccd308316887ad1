// Simulated annealing over the ring (Section 4.3: stochastic search by simulated annealing, neighbours
// obtained by reversing a random sub-array).  Proposal, temperature schedule and the integer acceptance
// rule are stated in cc.h, cc_sa_search.
//
// One wavefront per chain; the order lives in LDS.  A chain is sequential, but a rejected proposal
// leaves the order untouched, so the 64 lanes evaluate the proposals of the next 64 steps against the
// current order at once; the wave then commits the FIRST accepted one (ballot + find-first-set), and
// the steps after it are proposed again in the next round against the new order.  The result is the
// sequential chain bit for bit; a round advances 1 .. 64 steps, most of them when the chain is cold.
// Each lane draws its step's random word itself (counter-based generator), gathers four ranks of the
// order and four matrix entries (LDS for N <= 128, else through L2), and tests acceptance in 64-bit
// integer arithmetic.  The committed reversal is done by the whole wave, one pair of ranks per lane.
#include "cc_device.h"
#include "cc_internal.h"

namespace cc {
using namespace ccd;

namespace {

constexpr int kCostMax = (1 << 21) - 1;
constexpr int kDrawBase = 1024;       // low counter words below this belong to the initial shuffles

// all LDS traffic of the wave issued so far is complete and visible to every lane, and the compiler keeps
// LDS accesses on their side of this point
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <bool LDS_MATRIX>
__global__ __launch_bounds__(256) void sa_ring_kernel(const int32_t* __restrict__ c, int N, int chains,
                                                      long long steps, int t_start, int t_end, uint64_t seed,
                                                      int32_t* __restrict__ tours, int64_t* __restrict__ costs,
                                                      int32_t* __restrict__ accepted) {
    extern __shared__ int32_t sm[];
    const int lane = lane_id(), wv = threadIdx.x >> 6;
    int32_t* t = sm + wv * 2 * N;     // current order
    int32_t* bt = t + N;              // best order so far
    const int32_t* mat = c;
    if (LDS_MATRIX) {
        int32_t* m = sm + 8 * N;
        for (int e = threadIdx.x; e < N * N; e += 256) m[e] = clampi(c[e], 0, kCostMax);
        __syncthreads();
        mat = m;
    }
    const int64_t r = (int64_t)blockIdx.x * 4 + wv;
    if (r >= chains) return;
    auto M = [&](int x, int y) { return LDS_MATRIX ? mat[x * N + y] : clampi(mat[x * N + y], 0, kCostMax); };

    for (int p = lane; p < N; p += kWave) {
        const int v = clampi(tours[r * N + p], 0, N - 1);
        t[p] = v;
        bt[p] = v;
    }
    wave_lds_sync();
    long long cur = 0;
    for (int p = lane; p < N; p += kWave) cur += M(t[p], t[p ? p - 1 : N - 1]);
    cur = wave_sum64(cur);
    long long best = cur;
    int acc = 0;

    if (N >= 4) {
        const uint64_t chain_hi = (uint64_t)(uint32_t)r << 32;
        long long s = 0;
        while (s < steps) {
            const long long step = s + lane;
            const bool active = step < steps;
            const uint64_t w = splitmix64_at(seed, (chain_hi | (uint32_t)(kDrawBase + (uint32_t)step)) + 1u);
            const int a = (int)(((uint32_t)(w >> 43) * (uint32_t)N) >> 21);
            const int d = 2 + (int)((((uint32_t)(w >> 22) & 0x1FFFFFu) * (uint32_t)(N - 3)) >> 21);
            int b = a + d;
            b = b >= N ? b - N : b;
            const int u = (int)((uint32_t)w & 0x3FFFFFu) + 1;
            const int ap = a ? a - 1 : N - 1, bp = b ? b - 1 : N - 1;
            const int ta = t[a], tap = t[ap], tb = t[b], tbp = t[bp];
            const int delta = M(tap, tbp) + M(ta, tb) - M(ta, tap) - M(tb, tbp);
            bool accept = active;
            if (delta > 0) {
                const int e = 31 - __clz(u);
                const int mant = u - (1 << e);
                const int frac = e >= 12 ? (mant >> (e - 12)) : (mant << (12 - e));
                const long long E = 22 * 4096 - (e * 4096 + frac);
                const long long num = (long long)t_start * (steps - step) + (long long)t_end * step;
                accept = active && ((long long)delta * 4096 * steps <= num * E);
            }
            const unsigned long long mask = __ballot(accept);
            if (mask == 0ull) {
                s += kWave;
                continue;
            }
            const int k = __ffsll((long long)mask) - 1;
            const int ak = __shfl(a, k, kWave), bk = __shfl(b, k, kWave), dk = __shfl(delta, k, kWave);
            const int lo = min(ak, bk), hi = max(ak, bk);
            const int i = lo ? lo : hi, j = lo ? hi - 1 : N - 1;
            wave_lds_sync();                       // every lane has read the order before it changes
            const int half = (j - i + 1) >> 1;
            for (int x = lane; x < half; x += kWave) {
                const int p = i + x, q = j - x;
                const int vp = t[p], vq = t[q];
                t[p] = vq;
                t[q] = vp;
            }
            wave_lds_sync();
            cur += dk;
            ++acc;
            if (cur < best) {
                best = cur;
                for (int p = lane; p < N; p += kWave) bt[p] = t[p];
            }
            s += k + 1;
        }
    }
    wave_lds_sync();
    for (int p = lane; p < N; p += kWave) tours[r * N + p] = bt[p];
    if (lane == 0) {
        costs[r] = best;
        accepted[r] = acc;
    }
}

// ---------------------------------------------------------- halving-doubling model, pair neighbour (cc_sa_rd_search)
// Same round structure: 64 proposals against the current order, commit the first accepted one.  A proposal
// exchanges ranks p and q; per round only the links of p and q change, so the new round cost is
// max(link of p re-evaluated, link of q re-evaluated, largest link among the others), the last term being one of
// the round's three largest links.  Those three (value and lower rank of the link) are wave-uniform state,
// recomputed for every round after a commit: each lane evaluates its share of the N/2 links of the round and three
// wave-wide max-reductions over (value << 9 | link index) pick them (any choice among equal values is valid).
template <int LOGN>
__global__ __launch_bounds__(256) void sa_rd_kernel(const int32_t* __restrict__ c, int chains, long long steps,
                                                    int t_start, int t_end, uint64_t seed,
                                                    int32_t* __restrict__ tours, int64_t* __restrict__ costs,
                                                    int32_t* __restrict__ accepted) {
    constexpr int N = 1 << LOGN;
    constexpr bool LDS_MATRIX = LOGN <= 7;
    constexpr int LINKS = N / 2;
    constexpr int U = LINKS > 64 ? LINKS / 64 : 1;      // links per lane and round
    extern __shared__ int32_t sm[];
    const int lane = lane_id(), wv = threadIdx.x >> 6;
    int32_t* t = sm + wv * 2 * N;
    int32_t* bt = t + N;
    const int32_t* mat = c;
    if (LDS_MATRIX) {
        int32_t* m = sm + 8 * N;
        for (int e = threadIdx.x; e < N * N; e += 256) m[e] = clampi(c[e], 0, kCostMax);
        __syncthreads();
        mat = m;
    }
    const int64_t r = (int64_t)blockIdx.x * 4 + wv;
    if (r >= chains) return;
    auto M = [&](int x, int y) { return LDS_MATRIX ? mat[x * N + y] : clampi(mat[x * N + y], 0, kCostMax); };

    for (int p = lane; p < N; p += kWave) {
        const int v = clampi(tours[r * N + p], 0, N - 1);
        t[p] = v;
        bt[p] = v;
    }
    wave_lds_sync();

    int tv[LOGN][3], tj[LOGN][3];                       // the three largest links of every round: value, lower rank
    auto refresh = [&]() {                              // from the order in LDS; returns the cost
        int cost = 0;
#pragma unroll
        for (int k = 0; k < LOGN; ++k) {
            const int bit = 1 << k;
            int key[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = lane + 64 * u;            // link index
                const int j = ((i >> k) << (k + 1)) | (i & (bit - 1));
                key[u] = -1;
                if (i < LINKS) {
                    const int a = t[j], b = t[j | bit];
                    key[u] = (max(M(a, b), M(b, a)) << 9) | i;
                }
            }
            int taken0 = -2, taken1 = -2;
#pragma unroll
            for (int pass = 0; pass < 3; ++pass) {
                int best = -1;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int i = lane + 64 * u;
                    best = max(best, (i == taken0 || i == taken1) ? -1 : key[u]);
                }
                best = wave_max(best);
                const int i = best & 511;
                tv[k][pass] = best >> 9;                // -1 when the round has fewer links
                tj[k][pass] = best < 0 ? -1 : (((i >> k) << (k + 1)) | (i & (bit - 1)));
                if (pass == 0) taken0 = best < 0 ? -2 : i;
                else taken1 = best < 0 ? -2 : i;
            }
            cost += tv[k][0];
        }
        return cost;
    };

    int cur = refresh();
    int best = cur;
    int acc = 0;
    const uint64_t chain_hi = (uint64_t)(uint32_t)r << 32;
    long long s = 0;
    while (s < steps) {
        const long long step = s + lane;
        const bool active = step < steps;
        const uint64_t w = splitmix64_at(seed, (chain_hi | (uint32_t)(kDrawBase + (uint32_t)step)) + 1u);
        const int p = (int)(((uint32_t)(w >> 43) * (uint32_t)N) >> 21);
        const int d = 1 + (int)((((uint32_t)(w >> 22) & 0x1FFFFFu) * (uint32_t)(N - 1)) >> 21);
        const int q = (p + d) & (N - 1);
        const int u = (int)((uint32_t)w & 0x3FFFFFu) + 1;
        const int tp = t[p], tq = t[q];
        int total = 0;
#pragma unroll
        for (int k = 0; k < LOGN; ++k) {
            const int bit = 1 << k;
            const int pb = t[p ^ bit], qb = t[q ^ bit];
            const int link_p = max(M(tq, pb), M(pb, tq));           // rank p now holds t[q]
            const int link_q = max(M(tp, qb), M(qb, tp));           // rank q now holds t[p]
            const int lp = p & ~bit, lq = q & ~bit;
            const bool f0 = tj[k][0] != lp && tj[k][0] != lq, f1 = tj[k][1] != lp && tj[k][1] != lq;
            const int others = f0 ? tv[k][0] : (f1 ? tv[k][1] : tv[k][2]);
            const int stage = max(others, max(link_p, link_q));
            total += (q == (p ^ bit)) ? tv[k][0] : stage;
        }
        const int delta = total - cur;
        bool accept = active;
        if (delta > 0) {
            const int e = 31 - __clz(u);
            const int mant = u - (1 << e);
            const int frac = e >= 12 ? (mant >> (e - 12)) : (mant << (12 - e));
            const long long E = 22 * 4096 - (e * 4096 + frac);
            const long long num = (long long)t_start * (steps - step) + (long long)t_end * step;
            accept = active && ((long long)delta * 4096 * steps <= num * E);
        }
        const unsigned long long mask = __ballot(accept);
        if (mask == 0ull) {
            s += kWave;
            continue;
        }
        const int kk = __ffsll((long long)mask) - 1;
        const int sp = __shfl(p, kk, kWave), sq = __shfl(q, kk, kWave), dk = __shfl(delta, kk, kWave);
        wave_lds_sync();                               // every lane has read the order before it changes
        if (lane == 0) {
            const int a = t[sp], b = t[sq];
            t[sp] = b;
            t[sq] = a;
        }
        wave_lds_sync();
        cur += dk;
        ++acc;
        refresh();
        if (cur < best) {
            best = cur;
            for (int x = lane; x < N; x += kWave) bt[x] = t[x];
        }
        s += kk + 1;
    }
    wave_lds_sync();
    for (int x = lane; x < N; x += kWave) tours[r * N + x] = bt[x];
    if (lane == 0) {
        costs[r] = (int64_t)best;
        accepted[r] = acc;
    }
}

template <int LOGN>
static hipError_t sa_rd_launch(const int32_t* c, int chains, long long steps, int t_start, int t_end, uint64_t seed,
                               int32_t* tours, int64_t* costs, int32_t* accepted, hipStream_t s) {
    constexpr int N = 1 << LOGN;
    const size_t lds = sizeof(int32_t) * ((size_t)8 * N + (LOGN <= 7 ? (size_t)N * N : 0));
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)sa_rd_kernel<LOGN>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(sa_rd_kernel<LOGN>, dim3((chains + 3) / 4), dim3(256), lds, s, c, chains, steps, t_start, t_end,
                       seed, tours, costs, accepted);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_sa_ring(const int32_t* c, int N, int chains, long long steps, int t_start, int t_end, uint64_t seed,
                          bool generate, int32_t* tours, int64_t* costs, int32_t* accepted, hipStream_t s) {
    if (generate) {
        hipError_t e = launch_init_tours(N, 0, chains, seed, tours, s);
        if (e != hipSuccess) return e;
    }
    const int grid = (chains + 3) / 4;
    if (N <= 128) {
        const size_t lds = sizeof(int32_t) * ((size_t)8 * N + (size_t)N * N);
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute((const void*)sa_ring_kernel<true>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL((sa_ring_kernel<true>), dim3(grid), dim3(256), lds, s, c, N, chains, steps, t_start, t_end,
                           seed, tours, costs, accepted);
    } else {
        const size_t lds = sizeof(int32_t) * (size_t)8 * N;
        hipLaunchKernelGGL((sa_ring_kernel<false>), dim3(grid), dim3(256), lds, s, c, N, chains, steps, t_start, t_end,
                           seed, tours, costs, accepted);
    }
    return hipGetLastError();
}

// N is a power of two in [2, 1024] (checked by the caller)
hipError_t launch_sa_rd(const int32_t* c, int N, int chains, long long steps, int t_start, int t_end, uint64_t seed,
                        bool generate, int32_t* tours, int64_t* costs, int32_t* accepted, hipStream_t s) {
    if (generate) {
        hipError_t e = launch_init_tours(N, 0, chains, seed, tours, s);
        if (e != hipSuccess) return e;
    }
    switch (N) {
        case 2: return sa_rd_launch<1>(c, chains, steps, t_start, t_end, seed, tours, costs, accepted, s);
        case 4: return sa_rd_launch<2>(c, chains, steps, t_start, t_end, seed, tours, costs, accepted, s);
        case 8: return sa_rd_launch<3>(c, chains, steps, t_start, t_end, seed, tours, costs, accepted, s);
        case 16: return sa_rd_launch<4>(c, chains, steps, t_start, t_end, seed, tours, costs, accepted, s);
        case 32: return sa_rd_launch<5>(c, chains, steps, t_start, t_end, seed, tours, costs, accepted, s);
        case 64: return sa_rd_launch<6>(c, chains, steps, t_start, t_end, seed, tours, costs, accepted, s);
        case 128: return sa_rd_launch<7>(c, chains, steps, t_start, t_end, seed, tours, costs, accepted, s);
        case 256: return sa_rd_launch<8>(c, chains, steps, t_start, t_end, seed, tours, costs, accepted, s);
        case 512: return sa_rd_launch<9>(c, chains, steps, t_start, t_end, seed, tours, costs, accepted, s);
        default: return sa_rd_launch<10>(c, chains, steps, t_start, t_end, seed, tours, costs, accepted, s);
    }
}

}  // namespace cc
