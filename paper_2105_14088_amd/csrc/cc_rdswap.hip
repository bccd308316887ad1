// Multi-start pair-swap local search under the halving-doubling cost model (Section 4.1 equation
// C_hd with the pairing of Section 2.2; neighbour "permute a pair" of Section 4.3; move set, value and
// tie-break rules as stated in cc.h, cc_rd_swap_search).
//
// In round k ranks i and i xor 2^k form a LINK whose value is the larger of its two directed costs; a
// round costs its largest link.  Swapping ranks p and q touches, per round, only the links of p and of q
// (one link, with unchanged value, when q = p xor 2^k).  The new round cost is therefore
//     max( link of p re-evaluated, link of q re-evaluated, largest link among all the others ),
// and "largest among the others" is one of the round's three largest links, found once per sweep.
//
// General kernel: one workgroup per restart, one thread per rank p scanning q = p+1 .. N-1; matrix
// gathered through L2; 64-bit keys (value << 32 | move id) min-reduced over the workgroup.
// N = 64 kernel: one wavefront per restart, matrix in LDS, lane p scans partners q = p xor x; two rank
// differences x with the same top bit share a step (lanes with that bit clear take one, the others the
// other), so every pair is scored once, in 32 steps; the top-3 links of a round come from three
// wave-wide max-reductions over (value << 5 | link index).
#include "cc_device.h"
#include "cc_internal.h"
#include "cc_wave64.h"

namespace cc {
using namespace ccd;

namespace {

constexpr int kCostMax = (1 << 21) - 1;
constexpr int kMaxStages = 10;
constexpr unsigned long long kNoMove = ~0ull;

// ------------------------------------------------------------------------------------- general kernel
__global__ void rdswap_general_kernel(const int32_t* __restrict__ c, int N, int32_t* __restrict__ tours,
                                      int64_t* __restrict__ costs, int32_t* __restrict__ moves,
                                      const int32_t* __restrict__ skip_if_small) {
    // when the 16-bit workgroup kernel is launched beside this one, flags[0] = max(c) decides which of the two runs
    if (skip_if_small && skip_if_small[0] < (1 << 16)) return;
    extern __shared__ int32_t sm[];
    int32_t* t = sm;                 // [N]
    int32_t* w = sm + N;             // [N] directed cost of each rank in the round being prepared
    __shared__ int top_v[kMaxStages][3], top_l[kMaxStages][3], top_n[kMaxStages];
    __shared__ unsigned long long red[16];
    __shared__ unsigned long long winner;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, nwv = blockDim.x >> 6;
    const int64_t r = blockIdx.x;
    auto C = [&](int a, int b) { return clampi(c[a * N + b], 0, kCostMax); };
    if (tid < N) t[tid] = clampi(tours[r * N + tid], 0, N - 1);
    __syncthreads();

    auto block_max_u64 = [&](unsigned long long key) {   // every thread gets the maximum
        unsigned long long v = key;
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) {
            const unsigned long long o = __shfl_xor(v, m, kWave);
            v = o > v ? o : v;
        }
        __syncthreads();
        if (lane == 0) red[wv] = v;
        __syncthreads();
        v = red[0];
        for (int k = 1; k < nwv; ++k) v = red[k] > v ? red[k] : v;
        return v;
    };

    int applied = 0;
    long long cur = 0;
    for (;;) {
        // ---- per round: link values and the three largest links
        int stages = 0;
        cur = 0;
        for (int bit = 1; bit < N; bit <<= 1, ++stages) {
            if (tid < N) w[tid] = C(t[tid], t[tid ^ bit]);
            __syncthreads();
            int lv = -1;
            if (tid < N && !(tid & bit)) lv = max(w[tid], w[tid | bit]);
            int taken[3] = {-1, -1, -1};
            int n = 0;
            for (int round = 0; round < 3; ++round) {
                const bool mine = lv >= 0 && tid != taken[0] && tid != taken[1];
                // key: value, then a preference for the lower link id (any choice among equal values is valid)
                const unsigned long long key = mine ? (((unsigned long long)(unsigned)lv << 32) | (unsigned)(N - tid)) : 0ull;
                const unsigned long long best = block_max_u64(key);
                if (best == 0ull) break;
                taken[round] = N - (int)(best & 0xffffffffu);
                if (tid == 0) {
                    top_v[stages][round] = (int)(best >> 32);
                    top_l[stages][round] = taken[round];
                }
                ++n;
            }
            if (tid == 0) top_n[stages] = n;
            __syncthreads();
            cur += top_v[stages][0];
        }
        // ---- score swaps (p, q), q > p, for p = tid
        unsigned long long best = kNoMove;
        const int p = tid;
        if (p < N - 1) {
            const int tp = t[p];
            for (int q = p + 1; q < N; ++q) {
                const int tq = t[q];
                int total = 0;
                int k = 0;
                for (int bit = 1; bit < N; bit <<= 1, ++k) {
                    if (q == (p ^ bit)) { total += top_v[k][0]; continue; }
                    const int lp = p & ~bit, lq = q & ~bit;
                    int others = 0;
                    for (int m = 0; m < top_n[k]; ++m)
                        if (top_l[k][m] != lp && top_l[k][m] != lq) { others = top_v[k][m]; break; }
                    const int pb = t[p ^ bit], qb = t[q ^ bit];
                    const int link_p = max(C(tq, pb), C(pb, tq));      // rank p now holds t[q]
                    const int link_q = max(C(tp, qb), C(qb, tp));      // rank q now holds t[p]
                    total += max(others, max(link_p, link_q));
                }
                best = min(best, ((unsigned long long)(unsigned)total << 32) | (unsigned)(p * N + q));
            }
        }
        best = wave_min_u64(best);
        __syncthreads();
        if (lane == 0) red[wv] = best;
        __syncthreads();
        if (tid == 0) {
            unsigned long long m = red[0];
            for (int k = 1; k < nwv; ++k) m = min(m, red[k]);
            winner = m;
        }
        __syncthreads();
        const unsigned long long win = winner;
        if (win == kNoMove || (long long)(win >> 32) >= cur) break;
        const unsigned id = (unsigned)(win & 0xffffffffu);
        const int sp = (int)(id / (unsigned)N), sq = (int)(id % (unsigned)N);
        if (tid == 0) {
            const int a = t[sp];
            t[sp] = t[sq];
            t[sq] = a;
        }
        __syncthreads();
        ++applied;
    }
    if (tid < N) tours[r * N + tid] = t[tid];
    if (tid == 0) {
        costs[r] = cur;
        moves[r] = applied;
    }
}

// ----------------------------------------------------------------------------------------- N = 64
using namespace w64;

__device__ __forceinline__ int wave_max_all(int v) { return wave_max(v); }

__global__ __launch_bounds__(256) void rdswap_n64_kernel(const int32_t* __restrict__ c, int restarts, uint64_t seed,
                                                         int generate, int32_t* __restrict__ tours,
                                                         int64_t* __restrict__ costs, int32_t* __restrict__ moves) {
    __shared__ __attribute__((aligned(256))) int32_t m[kN * kN];
    __shared__ int32_t tl_all[4][kN];            // each wave's tour, for "node at rank p xor x" look-ups
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    int v[kN * kN / 256];
#pragma unroll
    for (int k = 0; k < kN * kN / 256; ++k) v[k] = c[tid + 256 * k];
    const int64_t r = (int64_t)blockIdx.x * 4 + wv;
    int t = 0;
    if (r < restarts)
        t = generate ? init_tour_in_wave(seed, (uint32_t)r, lane) : clampi(tours[r * kN + lane], 0, kN - 1);
#pragma unroll
    for (int k = 0; k < kN * kN / 256; ++k) m[tid + 256 * k] = clampi(v[k], 0, kCostMax);
    __syncthreads();
    // a link costs the larger of its two directed entries: fold the two into both places once, so that a link is one
    // gather
    for_each_pair_64(tid, [&](int lo, int hi) {
        const int both = max(m[lo * kN + hi], m[hi * kN + lo]);
        m[lo * kN + hi] = both;
        m[hi * kN + lo] = both;
    });
    __syncthreads();
    if (r >= restarts) return;
    const char* mbytes = (const char*)m;
    int32_t* tl = tl_all[wv];
    const char* tlbytes = (const char*)tl;
    auto entry = [&](int row8, int col2) { return *(const int32_t*)(mbytes + (row8 | col2)); };   // row << 8 | col << 2

    int applied = 0, cur = 0;
    for (;;) {
        tl[lane] = t;
        __builtin_amdgcn_wave_barrier();
        const int t8 = t << 8;
        // per round: partner, link value, and the best / second-best link value among links other than this lane's
        int pb2[6], x1v[6], x2v[6], zk[6], round_cost[6], own_addr[6];
        cur = 0;
#pragma unroll
        for (int k = 0; k < 6; ++k) {
            const int bit = 1 << k;
            const int pb = tl[lane ^ bit];
            pb2[k] = pb << 2;
            own_addr[k] = (lane ^ bit) << 2;                       // byte offset of rank p xor 2^k in tl
            const int lv = entry(t8, pb2[k]);
            const int li = ((lane >> (k + 1)) << k) | (lane & (bit - 1));          // link index, 5 bits
            int key = (lv << 5) | li;
            const int k1 = wave_max_all(key);
            const int k2 = wave_max_all((li == (k1 & 31)) ? -1 : key);
            const int k3 = wave_max_all((li == (k1 & 31) || li == (k2 & 31)) ? -1 : key);
            // k2, k3 are -1 when fewer links exist (never at N = 64: 32 links per round)
            const int l1 = k1 & 31, l2 = k2 & 31;
            const int a1 = (li == l1) ? k2 : k1;                   // best link that is not mine
            const int a2 = (li == l1 || li == l2) ? k3 : k2;       // second best that is not mine
            x1v[k] = a1 >> 5;
            x2v[k] = a2 >> 5;
            zk[k] = li ^ (a1 & 31);                                // partner's link == that best link  <=>  li(m) == zk
            round_cost[k] = k1 >> 5;
            cur += round_cost[k];
        }
        // Partners by rank difference x = p xor q.  Every pair would be seen from both of its ends; instead two
        // differences with the same top bit h, x = 2j and 2j + 1, share a step: the lanes whose rank has bit h clear
        // take the first, the others the second, so the 64 lanes score 64 distinct pairs.  x = 1 has no mate: its
        // step scores each of its 32 pairs twice (same value, same id).
        unsigned long long best = kNoMove;
#pragma unroll 1
        for (int j = 0; j < kN / 2; ++j) {
            const int x0 = j ? 2 * j : 1, x1 = j ? 2 * j + 1 : 1;                           // wave-uniform
            const int top = 31 - __builtin_clz(x0);
            const bool second = (lane >> top) & 1;
            const int mm = second ? x1 : x0;
            const int q = lane ^ mm;
            const int tq = *(const int32_t*)(tlbytes + (q << 2));
            const int tq8 = tq << 8;
            int total = 0;
#pragma unroll
            for (int k = 0; k < 6; ++k) {
                const int bit = 1 << k;
                const int qb = *(const int32_t*)(tlbytes + (own_addr[k] ^ (mm << 2)));      // node at rank q xor 2^k
                const int link_p = entry(tq8, pb2[k]);             // rank p now holds t[q]
                const int link_q = entry(t8, qb << 2);             // rank q now holds t[p]
                // link index offset of the partner, for either difference (wave-uniform), then this lane's
                const int lim0 = ((x0 >> (k + 1)) << k) | (x0 & (bit - 1));
                const int lim1 = ((x1 >> (k + 1)) << k) | (x1 & (bit - 1));
                const int lim = second ? lim1 : lim0;
                const int others = (zk[k] == lim) ? x2v[k] : x1v[k];
                const int stage = max(others, max(link_p, link_q));
                total += (mm == bit) ? round_cost[k] : stage;
            }
            const int lo = min(lane, q), hi = max(lane, q);
            best = min(best, ((unsigned long long)(unsigned)total << 12) | (unsigned)(lo * kN + hi));
        }
        const unsigned long long win = wave_min_u64(best);
        const int total_win = (int)(win >> 12);
        if (total_win >= cur) break;
        const int id = __builtin_amdgcn_readfirstlane((int)(win & 0xfff)), sp = id >> 6, sq = id & 63;
        const int a = __builtin_amdgcn_readlane(t, sp), b = __builtin_amdgcn_readlane(t, sq);
        t = lane == sp ? b : (lane == sq ? a : t);
        ++applied;
        __builtin_amdgcn_wave_barrier();
    }
    tours[r * kN + lane] = t;
    if (lane == 0) {
        costs[r] = (int64_t)cur;
        moves[r] = applied;
    }
}

// 16-bit matrix with both directed entries of a pair folded into both places, max(c[x][y], c[y][x]): a link is then
// one gather.  For the sizes whose matrix does not fit LDS; skipped when an entry needs more than 16 bits.
__global__ __launch_bounds__(256) void fold_to_u16_kernel(const int32_t* __restrict__ c, int n,
                                                          uint16_t* __restrict__ c16,
                                                          const int32_t* __restrict__ flags) {
    if (flags[0] >= (1 << 16)) return;
    for (int e = blockIdx.x * 256 + threadIdx.x; e < n * n; e += gridDim.x * 256) {
        const int x = e / n, y = e - x * n;
        c16[e] = (uint16_t)max(clampi(c[e], 0, 0xffff), clampi(c[y * n + x], 0, 0xffff));
    }
}

// ------------------------------------------------------------------------- N = 128 .. 1024: one workgroup per restart
// The N = 64 scheme with one thread per rank: N threads, the order in LDS, the three largest links of a round from
// workgroup-wide max-reductions, two rank differences per step so that the N threads score N distinct pairs.  The
// matrix is read as folded 16-bit entries: staged and folded in LDS for N = 128, 256 (32 / 128 KiB), gathered through
// L2 from the folded copy in the workspace for N = 512, 1024 (IN_LDS false).  Needs max(c) < 2^16, otherwise the
// general kernel runs instead, decided on the device.  Keys: value << 2 log2 N | move id (value < 2^20).
template <int LOGN, bool IN_LDS>
__global__ __launch_bounds__(1 << LOGN) void rdswap_block_kernel(const int32_t* __restrict__ c,
                                                                 const uint16_t* __restrict__ folded,
                                                                 int32_t* __restrict__ tours,
                                                                 int64_t* __restrict__ costs,
                                                                 int32_t* __restrict__ moves,
                                                                 const int32_t* __restrict__ flags) {
    constexpr int N = 1 << LOGN, NW = N / 64, LB = LOGN - 1;   // LB: bits of a link index
    constexpr int kIdBits = 2 * LOGN;
    if (flags[0] >= (1 << 16)) return;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint16_t* m16 = (uint16_t*)smem;                           // [N * N] (IN_LDS)
    int32_t* tl = (int32_t*)(smem + (IN_LDS ? sizeof(uint16_t) * N * N : 0)); // [N] the order
    __shared__ int red_i[2][NW];
    __shared__ unsigned long long red_k[NW];
    const int p = threadIdx.x, lane = p & 63, wv = p >> 6;
    const int64_t r = blockIdx.x;
    if (IN_LDS)
        for (int e = p; e < N * N; e += N) m16[e] = (uint16_t)clampi(c[e], 0, 0xffff);
    int t = clampi(tours[r * N + p], 0, N - 1);
    tl[p] = t;
    __syncthreads();
    if (IN_LDS) {
        // a link costs the larger of its two directed entries: fold the two into both places once (thread p takes
        // the pairs {p, p + j}, j = 1 .. N/2; every unordered pair exactly once), so that a link is one gather
        for (int j = 1; j <= N / 2; ++j) {
            const int b = (p + j) & (N - 1);
            if (j < N / 2 || p < N / 2) {
                const uint16_t both = max(m16[p * N + b], m16[b * N + p]);
                m16[p * N + b] = both;
                m16[b * N + p] = both;
            }
        }
        __syncthreads();
    }
    auto entry = [&](int a, int b) { return IN_LDS ? (int)m16[a * N + b] : (int)folded[a * N + b]; };
    int parity = 0;
    auto block_max = [&](int v) {                              // every thread gets the maximum; one barrier per call
        v = wave_max(v);
        if (lane == 0) red_i[parity][wv] = v;
        __syncthreads();
        int o = red_i[parity][0];
#pragma unroll
        for (int k = 1; k < NW; ++k) o = max(o, red_i[parity][k]);
        parity ^= 1;
        return o;
    };

    int applied = 0, cur = 0;
    for (;;) {
        int pb[LOGN], x1v[LOGN], x2v[LOGN], zk[LOGN], round_cost[LOGN];
        cur = 0;
#pragma unroll
        for (int k = 0; k < LOGN; ++k) {
            const int bit = 1 << k;
            pb[k] = tl[p ^ bit];
            const int lv = entry(t, pb[k]);
            const int li = ((p >> (k + 1)) << k) | (p & (bit - 1));
            const int key = (lv << LB) | li;
            const int k1 = block_max(key);
            const int k2 = block_max((li == (k1 & (N / 2 - 1))) ? -1 : key);
            const int k3 = block_max((li == (k1 & (N / 2 - 1)) || li == (k2 & (N / 2 - 1))) ? -1 : key);
            const int l1 = k1 & (N / 2 - 1), l2 = k2 & (N / 2 - 1);
            const int a1 = (li == l1) ? k2 : k1;               // best link that is not this rank's
            const int a2 = (li == l1 || li == l2) ? k3 : k2;   // second best that is not this rank's
            x1v[k] = a1 >> LB;
            x2v[k] = a2 >> LB;
            zk[k] = li ^ (a1 & (N / 2 - 1));                   // partner's link is that best link  <=>  li(x) == zk
            round_cost[k] = k1 >> LB;
            cur += round_cost[k];
        }
        unsigned long long best = kNoMove;
#pragma unroll 1
        for (int j = 0; j < N / 2; ++j) {
            const int x0 = j ? 2 * j : 1, x1 = j ? 2 * j + 1 : 1;
            const int top = 31 - __builtin_clz(x0);
            const bool second = (p >> top) & 1;
            const int mm = second ? x1 : x0;
            const int q = p ^ mm;
            const int tq = tl[q];
            int total = 0;
#pragma unroll
            for (int k = 0; k < LOGN; ++k) {
                const int bit = 1 << k;
                const int qb = tl[q ^ bit];
                const int link_p = entry(tq, pb[k]);
                const int link_q = entry(t, qb);
                const int lim0 = ((x0 >> (k + 1)) << k) | (x0 & (bit - 1));
                const int lim1 = ((x1 >> (k + 1)) << k) | (x1 & (bit - 1));
                const int lim = second ? lim1 : lim0;
                const int others = (zk[k] == lim) ? x2v[k] : x1v[k];
                const int stage = max(others, max(link_p, link_q));
                total += (mm == bit) ? round_cost[k] : stage;
            }
            const int lo = min(p, q), hi = max(p, q);
            best = min(best, ((unsigned long long)(unsigned)total << kIdBits) | (unsigned)(lo * N + hi));
        }
        best = wave_min_u64(best);
        if (lane == 0) red_k[wv] = best;
        __syncthreads();
        unsigned long long win = red_k[0];
#pragma unroll
        for (int k = 1; k < NW; ++k) win = min(win, red_k[k]);
        if ((int)(win >> kIdBits) >= cur) break;
        const int id = (int)(win & ((1u << kIdBits) - 1u)), sp = id >> LOGN, sq = id & (N - 1);
        const int a = tl[sp], b = tl[sq];
        __syncthreads();                                       // everyone has read red_k and the two ranks
        if (p == sp) { t = b; tl[p] = b; }
        if (p == sq) { t = a; tl[p] = a; }
        ++applied;
        __syncthreads();
    }
    tours[r * N + p] = t;
    if (p == 0) {
        costs[r] = (int64_t)cur;
        moves[r] = applied;
    }
}

template <int LOGN>
static hipError_t rdswap_block_launch(const int32_t* c, uint16_t* folded, int restarts, int32_t* tours, int64_t* costs,
                                      int32_t* moves, const int32_t* flags, hipStream_t s) {
    constexpr int N = 1 << LOGN;
    constexpr bool kInLds = LOGN <= 8;
    if (!kInLds) {
        hipLaunchKernelGGL(fold_to_u16_kernel, dim3(512), dim3(256), 0, s, c, N, folded, flags);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const size_t lds = (kInLds ? sizeof(uint16_t) * N * N : 0) + sizeof(int32_t) * N;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)rdswap_block_kernel<LOGN, kInLds>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((rdswap_block_kernel<LOGN, kInLds>), dim3(restarts), dim3(N), lds, s, c, folded, tours, costs,
                       moves, flags);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_rdswap(const int32_t* c, int N, int restarts, uint64_t seed, bool tours_hold_init, int32_t* tours,
                         int64_t* costs, int32_t* moves, int32_t* flags, uint16_t* mat16, hipStream_t s) {
    if (N == 64) {
        hipLaunchKernelGGL(rdswap_n64_kernel, dim3((restarts + 3) / 4), dim3(256), 0, s, c, restarts, seed,
                           tours_hold_init ? 0 : 1, tours, costs, moves);
        return hipGetLastError();
    }
    if (!tours_hold_init) {
        hipError_t e = launch_init_tours(N, 0, restarts, seed, tours, s);
        if (e != hipSuccess) return e;
    }
    const int32_t* skip = nullptr;
    if (N == 128 || N == 256 || N == 512 || N == 1024) {
        // 16-bit workgroup kernel when max(c) < 2^16, else the general kernel: both are enqueued and the matrix
        // maximum, computed on the device, decides which one does the work (no host round trip)
        hipError_t e = launch_matrix_max(c, N, flags, s);
        if (e != hipSuccess) return e;
        e = N == 128   ? rdswap_block_launch<7>(c, mat16, restarts, tours, costs, moves, flags, s)
            : N == 256 ? rdswap_block_launch<8>(c, mat16, restarts, tours, costs, moves, flags, s)
            : N == 512 ? rdswap_block_launch<9>(c, mat16, restarts, tours, costs, moves, flags, s)
                       : rdswap_block_launch<10>(c, mat16, restarts, tours, costs, moves, flags, s);
        if (e != hipSuccess) return e;
        skip = flags;
    }
    const int threads = ((N + 63) / 64) * 64;
    hipLaunchKernelGGL(rdswap_general_kernel, dim3(restarts), dim3(threads), sizeof(int32_t) * 2 * (size_t)N, s, c, N,
                       tours, costs, moves, skip);
    return hipGetLastError();
}

}  // namespace cc
