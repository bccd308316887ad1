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
// N = 64 kernel: one wavefront per restart, matrix in LDS (both directed entries of a pair folded into one value),
// lane p scans partners q = p xor x; two rank differences x with the same top bit share a step (lanes with that bit
// clear take one, the others the other), so every pair is scored once, in 32 steps.  The node at rank p xor y is
// fetched once per sweep for all 64 y (ds_swizzle) and the step loop is fully unrolled, so the partner and the round
// mates of both ends are register selects; the top-3 links of a round come from wave-wide max-reductions over
// (value << 5 | link index), three rounds at a time.
#include <type_traits>
#include <utility>

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

// lane p <- lane p xor Y for Y < 32 (ds_swizzle in bit mode: no LDS access, no address arithmetic)
template <int Y>
__device__ __forceinline__ int from_lane_xor(int v) {
    if constexpr (Y == 0) return v;
    else return __builtin_amdgcn_ds_swizzle(v, (Y << 10) | 0x1f);
}
// out[y] = the value lane p xor y holds, for every y: own (lower 32 differences) and far (the value of lane p xor 32)
template <int... Y>
__device__ __forceinline__ void from_every_lane(int (&out)[kN], int own, int far, std::integer_sequence<int, Y...>) {
    ((out[Y] = from_lane_xor<(Y & 31)>((Y & 32) ? far : own)), ...);
}

// Keeps "cond ? a[i] : a[j]" a select between two registers: without it the compiler selects the index instead and
// the array leaves the register file.
__device__ __forceinline__ int in_register(int v) {
    asm("" : "+v"(v));
    return v;
}

// One descent.  m: the folded matrix in LDS.  WIDE: totals that need more than 19 bits (entries from 2^16 up), keys
// of 64 bits.
template <bool WIDE>
__device__ __forceinline__ void descend_swaps(const int32_t* m, int lane, int& t, int& cost, int& applied_out) {
    using K = typename std::conditional<WIDE, unsigned long long, int>::type;
    const char* mbytes = (const char*)m;
    auto entry = [&](int byte_offset) { return *(const int32_t*)(mbytes + byte_offset); };   // row << 8 | col << 2
    const int pair_base = lane * (kN + 1);       // id of the pair {lane, lane xor x}: pair_base ^ x or ^ (x << 6)
    int applied = 0, cur = 0;
    for (;;) {
        // node at rank p xor y, as a column byte offset, for every y: the partners q = p xor x of this sweep and the
        // round mates of both ends all come from here, by register index
        const int t2 = t << 2, t8 = t << 8;
        int tl[kN];
        from_every_lane(tl, t2, __shfl_xor(t2, 32, kWave), std::make_integer_sequence<int, kN>{});
        // per round: the best / second-best link value among links other than this lane's, and where the best one is
        int x1v[6], x2v[6], zk[6], zk_second[6], round_cost[6];
        int li[6], key[6], k1[6], k2[6], k3[6];
#pragma unroll
        for (int k = 0; k < 6; ++k) {
            const int bit = 1 << k;
            li[k] = ((lane >> (k + 1)) << k) | (lane & (bit - 1));                 // link index, 5 bits
            key[k] = (entry(t8 | tl[bit]) << 5) | li[k];
            k1[k] = key[k];
        }
        // the three largest links of every round: the rounds are independent, so their reductions run three at a time
        wave_max3(k1[0], k1[1], k1[2]);
        wave_max3(k1[3], k1[4], k1[5]);
#pragma unroll
        for (int k = 0; k < 6; ++k) k2[k] = (li[k] == (k1[k] & 31)) ? -1 : key[k];
        wave_max3(k2[0], k2[1], k2[2]);
        wave_max3(k2[3], k2[4], k2[5]);
#pragma unroll
        for (int k = 0; k < 6; ++k) k3[k] = (li[k] == (k1[k] & 31) || li[k] == (k2[k] & 31)) ? -1 : key[k];
        wave_max3(k3[0], k3[1], k3[2]);
        wave_max3(k3[3], k3[4], k3[5]);
        cur = 0;
#pragma unroll
        for (int k = 0; k < 6; ++k) {
            const int l1 = k1[k] & 31, l2 = k2[k] & 31;
            const int a1 = (li[k] == l1) ? k2[k] : k1[k];                          // best link that is not mine
            const int a2 = (li[k] == l1 || li[k] == l2) ? k3[k] : k2[k];           // second best that is not mine
            x1v[k] = a1 >> 5;
            x2v[k] = a2 >> 5;
            zk[k] = li[k] ^ (a1 & 31);                             // partner's link == that best link  <=>  li(x) == zk
            zk_second[k] = zk[k] ^ (k ? 1 : 0);                    // the same test for the odd difference of a step
            round_cost[k] = k1[k] >> 5;
            cur += round_cost[k];
        }
        // Partners by rank difference x = p xor q.  Every pair would be seen from both of its ends; instead two
        // differences with the same top bit h, x0 = 2j and x1 = 2j + 1, share a step: the lanes whose rank has bit h
        // clear take x0, the others x1, so the 64 lanes score 64 distinct pairs.  x = 1 has no mate: its step scores
        // each of its 32 pairs twice (same value, same id).  The loop is unrolled, so every index below is a constant.
        K best = WIDE ? (K)~0ull : (K)0x7fffffff;
#pragma unroll
        for (int j = 0; j < kN / 2; ++j) {
            const int x0 = j ? 2 * j : 1, x1 = j ? 2 * j + 1 : 1;
            const int h = 31 - __builtin_clz(x0);
            const bool second = (lane >> h) & 1;
            const int tq_second = in_register(tl[x1]);
            const int tq2 = second ? tq_second : tl[x0];
            int total = 0;
#pragma unroll
            for (int k = 0; k < 6; ++k) {
                const int bit = 1 << k;
                if (x0 == bit && x1 == bit) {                      // x = 1 in round 0: every lane swaps with its mate
                    total += round_cost[k];
                    continue;
                }
                const int qb_second = in_register(tl[x1 ^ bit]);
                const int qb2 = second ? qb_second : tl[x0 ^ bit];                 // node at rank q xor 2^k
                const int link_p = entry((tq2 << 6) | tl[bit]);    // rank p now holds t[q]
                const int link_q = entry(t8 | qb2);                // rank q now holds t[p]
                // the partner's link index relative to this lane's: x without bit k; x1's differs from x0's in bit 0
                const int lim0 = ((x0 >> (k + 1)) << k) | (x0 & (bit - 1));
                const int z = (second && x1 != x0) ? zk_second[k] : zk[k];
                const int others = (z == lim0) ? x2v[k] : x1v[k];
                int stage = max(others, max(link_p, link_q));
                if (x0 == bit) stage = second ? stage : round_cost[k];             // x0 swaps the two ends of a link
                total += stage;
            }
            const int id = pair_base ^ (second ? (x1 << 6) : x0);                  // lower rank * 64 + higher rank
            const K key = WIDE ? (K)(((unsigned long long)(unsigned)total << 12) | (unsigned)id) : (K)((total << 12) | id);
            best = key < best ? key : best;
            // steps are scheduled four at a time: enough gathers in flight, and the live ranges stay within the
            // register file
            if ((j & 3) == 3) __builtin_amdgcn_sched_barrier(0);
        }
        int total_win, id;
        if constexpr (WIDE) {
            const unsigned long long win = wave_min_u64(best);
            total_win = (int)(win >> 12);
            id = __builtin_amdgcn_readfirstlane((int)(win & 0xfff));
        } else {
            const int win = wave_min(best);
            total_win = win >> 12;
            id = win & 0xfff;
        }
        if (total_win >= cur) break;
        const int sp = id >> 6, sq = id & 63;
        const int a = __builtin_amdgcn_readlane(t, sp), b = __builtin_amdgcn_readlane(t, sq);
        t = lane == sp ? b : (lane == sq ? a : t);
        ++applied;
    }
    cost = cur;
    applied_out = applied;
}

__global__ __launch_bounds__(256) void rdswap_n64_kernel(const int32_t* __restrict__ c, int restarts, uint64_t seed,
                                                         int generate, int32_t* __restrict__ tours,
                                                         int64_t* __restrict__ costs, int32_t* __restrict__ moves) {
    __shared__ __attribute__((aligned(256))) int32_t m[kN * kN];
    __shared__ int wave_max_entry[4];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    int v[kN * kN / 256];
#pragma unroll
    for (int k = 0; k < kN * kN / 256; ++k) v[k] = c[tid + 256 * k];
    const int64_t r = (int64_t)blockIdx.x * 4 + wv;
    int t = 0;
    if (r < restarts)
        t = generate ? init_tour_in_wave(seed, (uint32_t)r, lane) : clampi(tours[r * kN + lane], 0, kN - 1);
    int mx = 0;
#pragma unroll
    for (int k = 0; k < kN * kN / 256; ++k) {
        v[k] = clampi(v[k], 0, kCostMax);
        mx = max(mx, v[k]);
        m[tid + 256 * k] = v[k];
    }
    mx = wave_max(mx);
    if (lane == 0) wave_max_entry[wv] = mx;
    __syncthreads();
    mx = max(max(wave_max_entry[0], wave_max_entry[1]), max(wave_max_entry[2], wave_max_entry[3]));
    // a link costs the larger of its two directed entries: fold the two into both places once, so that a link is one
    // gather
    for_each_pair_64(tid, [&](int lo, int hi) {
        const int both = max(m[lo * kN + hi], m[hi * kN + lo]);
        m[lo * kN + hi] = both;
        m[hi * kN + lo] = both;
    });
    __syncthreads();
    if (r >= restarts) return;
    int cur, applied;
    if (mx >= (1 << 16)) descend_swaps<true>(m, lane, t, cur, applied);
    else descend_swaps<false>(m, lane, t, cur, applied);
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
// The N = 64 scheme with one thread per rank (SPLIT threads per rank, sharing the rank's steps, where the matrix is
// in LDS and a restart has a compute unit to itself: one wavefront per SIMD cannot overlap its gathers with its own
// arithmetic): the order in LDS, the three largest links of a round from workgroup-wide max-reductions, two rank
// differences per step so that N threads score N distinct pairs.  The matrix is read as folded 16-bit entries:
// staged and folded in LDS for N = 128, 256 (32 / 128 KiB), gathered through L2 from the folded copy in the
// workspace for N = 512, 1024 (IN_LDS false).  Needs max(c) < 2^16, otherwise the general kernel runs instead,
// decided on the device.  Per thread the running minimum is kept over total << log2 N | q (the move id grows with
// q); the workgroup reduces value << 2 log2 N | move id (value < 2^20).
template <int LOGN, bool IN_LDS, int SPLIT>
__global__ __launch_bounds__(SPLIT << LOGN) void rdswap_block_kernel(const int32_t* __restrict__ c,
                                                                     const uint16_t* __restrict__ folded,
                                                                     int32_t* __restrict__ tours,
                                                                     int64_t* __restrict__ costs,
                                                                     int32_t* __restrict__ moves,
                                                                     const int32_t* __restrict__ flags) {
    // SPLIT threads per rank share its steps: several wavefronts per SIMD, whose gathers and arithmetic overlap
    constexpr int N = 1 << LOGN, THREADS = SPLIT << LOGN, NW = THREADS / 64, LB = LOGN - 1;   // LB: bits of a link index
    constexpr int kIdBits = 2 * LOGN;
    constexpr int kStepUnroll = IN_LDS ? 2 : 1;                // two steps in flight where registers allow
    // 16 wavefronts: the workgroup-wide reductions finish with a wave reduction over the 16 partial results (read as
    // a chain into registers they cost spills under the 128-register limit of 1024 threads); 8 wavefronts keep the chain
    constexpr bool kTwoLevel = NW >= 16;
    if (flags[0] >= (1 << 16)) return;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    int32_t* tl = (int32_t*)smem;                              // [N] the order
    uint16_t* m16 = (uint16_t*)(smem + sizeof(int32_t) * N);   // [N * N] (IN_LDS)
    __shared__ int red_i[2][NW];
    __shared__ unsigned long long red_k[NW];
    const int tid = threadIdx.x, p = tid & (N - 1), part = tid >> LOGN, lane = tid & 63, wv = tid >> 6;
    const int64_t r = blockIdx.x;
    if (IN_LDS)
        for (int e = tid; e < N * N; e += THREADS) m16[e] = (uint16_t)clampi(c[e], 0, 0xffff);
    int t = clampi(tours[r * N + p], 0, N - 1);
    if (part == 0) tl[p] = t;
    __syncthreads();
    if (IN_LDS) {
        // a link costs the larger of its two directed entries: fold the two into both places once (the threads of
        // rank p take the pairs {p, p + j}, j = 1 .. N/2; every unordered pair exactly once), so that a link is one
        // gather
        for (int j = 1 + part; j <= N / 2; j += SPLIT) {
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
    auto entry_at = [&](unsigned byte_offset) {                // row << (LOGN + 1) | column << 1
        return (int)*(const uint16_t*)((IN_LDS ? (const char*)m16 : (const char*)folded) + byte_offset);
    };
    int parity = 0;
    auto block_max = [&](int v) {                              // every thread gets the maximum; one barrier per call
        v = wave_max(v);
        if (lane == 0) red_i[parity][wv] = v;
        __syncthreads();
        int o;
        if (kTwoLevel) {
            o = wave_max(red_i[parity][lane & (NW - 1)]);      // second level: one value per lane, no long chain
        } else {
            o = red_i[parity][0];
#pragma unroll
            for (int k = 1; k < NW; ++k) o = max(o, red_i[parity][k]);
        }
        parity ^= 1;
        return o;
    };

    int applied = 0, cur = 0;
    for (;;) {
        int pb2[LOGN], x1v[LOGN], x2v[LOGN], zk[LOGN], round_cost[LOGN];
        cur = 0;
#pragma unroll
        for (int k = 0; k < LOGN; ++k) {
            const int bit = 1 << k;
            const int pb = tl[p ^ bit];
            pb2[k] = pb << 1;                                  // the round mate's node as a column byte offset
            const int lv = entry(t, pb);
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
            round_cost[k] = __builtin_amdgcn_readfirstlane(k1 >> LB);
            cur += round_cost[k];
        }
        // Steps grouped by the top bit of the rank difference: within a group a thread keeps its side (x0 = 2j or
        // x1 = 2j + 1), so the side-dependent link-index test is prepared once per group.  The first step of a group
        // has x0 = 2^top: there the threads on the x0 side swap with their mate of round `top`, which leaves that
        // round as it is.  Per thread the move id grows with q, so the running minimum is kept over total << LOGN | q.
        const int trow = t << (LOGN + 1);
        int best32 = 0x7fffffff;
        auto score = [&](int x0, bool second, int secbit, int mate_round) {
            const int q = p ^ (x0 | secbit);
            const int q4 = q << 2;
            const int tqrow = *(const int32_t*)((const char*)tl + q4) << (LOGN + 1);
            int total = 0;
#pragma unroll
            for (int k = 0; k < LOGN; ++k) {
                const int bit = 1 << k;
                const int qb = *(const int32_t*)((const char*)tl + (q4 ^ (bit << 2)));     // node at rank q xor 2^k
                const int link_p = entry_at((unsigned)(tqrow | pb2[k]));           // rank p now holds t[q]
                const int link_q = entry_at((unsigned)(trow | (qb << 1)));         // rank q now holds t[p]
                const int lim0 = ((x0 >> (k + 1)) << k) | (x0 & (bit - 1));        // wave-uniform
                const int others = (zk[k] == lim0) ? x2v[k] : x1v[k];
                int stage = max(others, max(link_p, link_q));
                if (k == mate_round) stage = second ? stage : round_cost[k];
                total += stage;
            }
            best32 = min(best32, (total << LOGN) | q);
        };
        int side = 0;                                          // the side zk is prepared for
#pragma unroll 1
        for (int top = 0; top < LOGN; ++top) {
            const bool second = top && ((p >> top) & 1);
            const int secbit = second ? 1 : 0;
#pragma unroll
            for (int k = 1; k < LOGN; ++k) zk[k] ^= secbit ^ side;                 // x1's link index is x0's with bit 0 set
            side = secbit;
            const int x_first = 1 << top, x_end = 2 << top;
            if (part == top % SPLIT) score(x_first, second, secbit, top);
            if (top == 0) continue;                            // the difference 1 has no second step
#pragma unroll kStepUnroll
            for (int x0 = x_first + 2 + 2 * part; x0 < x_end; x0 += 2 * SPLIT) score(x0, second, secbit, -1);
        }
        unsigned long long best = kNoMove;
        {
            const int q = best32 & (N - 1), total = best32 >> LOGN;
            const int lo = min(p, q), hi = max(p, q);
            best = ((unsigned long long)(unsigned)total << kIdBits) | (unsigned)(lo * N + hi);
        }
        best = wave_min_u64(best);
        if (lane == 0) red_k[wv] = best;
        __syncthreads();
        unsigned long long win;
        if (kTwoLevel) {
            win = wave_min_u64(red_k[lane & (NW - 1)]);
        } else {
            win = red_k[0];
#pragma unroll
            for (int k = 1; k < NW; ++k) win = min(win, red_k[k]);
        }
        if ((int)(win >> kIdBits) >= cur) break;
        const int id = (int)(win & ((1u << kIdBits) - 1u)), sp = id >> LOGN, sq = id & (N - 1);
        const int a = tl[sp], b = tl[sq];
        __syncthreads();                                       // everyone has read red_k and the two ranks
        if (p == sp) { t = b; tl[p] = b; }
        if (p == sq) { t = a; tl[p] = a; }
        ++applied;
        __syncthreads();
    }
    if (part == 0) tours[r * N + p] = t;
    if (tid == 0) {
        costs[r] = (int64_t)cur;
        moves[r] = applied;
    }
}

// ------------------------------------------------------------------ N = 512, 1024: tiles of the folded matrix in LDS
// One workgroup per restart, one or two threads per rank p (two at N = 512: 1024 threads either way).  The folded
// 16-bit matrix F (512 KiB / 2 MiB, in the workspace)
// does not fit LDS, and gathered through L2 a sweep is bound by the misses one compute unit keeps in flight.  Here
// a sweep goes through the partner ranks q in blocks of QB consecutive ranks B; for a block the workgroup stages
//   CT[x][j]      = F[x][t[B + j]]                 every row x, the QB columns of the block's nodes
//   RT[h][j][y]   = F[t[(B + j) xor 2^k]][y]       k = log2 QB + h: the rows of the block's mates in the rounds whose
//                                                  mate lies outside the block, every column y
// and every link of every pair (p, q in B) is then an LDS gather: rank p holding t[q] costs, in round k,
// F[t[q]][t[p xor 2^k]] = CT[t[p xor 2^k]][j]; rank q holding t[p] costs F[t[p]][t[q xor 2^k]], which is
// CT[t[p]][j xor 2^k] when the mate of q lies in the block and RT[h][j][t[p]] otherwise (F is symmetric).
// Pairs are split so that every thread scores one pair per step: of two neighbouring partners q0, q0 + 1 a thread
// takes the one with its own parity when it lies below them and the other one when it lies above (every unordered
// pair is then scored exactly once, by the thread p for which p + q is even and p < q, or odd and p > q).  Pairs of
// round mates (q = p xor 2^k), whose round k keeps its cost, are scored apart from the folded copy through L2: 9 or
// 10 per thread.  Round maxima, keys, reduction and the swap as in the kernel above.
template <int LOGN, int LOGQ, int SPLIT>
__global__ __launch_bounds__(SPLIT << LOGN) void rdswap_tiled_kernel(const uint16_t* __restrict__ folded,
                                                                 int32_t* __restrict__ tours,
                                                                 int64_t* __restrict__ costs,
                                                                 int32_t* __restrict__ moves,
                                                                 const int32_t* __restrict__ flags) {
    constexpr int N = 1 << LOGN, QB = 1 << LOGQ, NH = LOGN - LOGQ, NT = SPLIT * N, NW = NT / 64, LB = LOGN - 1;
    static_assert(SPLIT == 1 || SPLIT == 2, "one or two threads per rank");
    constexpr int kIdBits = 2 * LOGN;
    constexpr int kInf = 0x7fffffff;
    // a row of CT takes QB / 2 + 1 words: with QB / 2 the rows of the 64 lanes of a gather would fall into four or
    // eight LDS banks only
    constexpr int kCtRowBytes = (QB / 2 + 1) * 4;
    if (flags[0] >= (1 << 16)) return;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    int32_t* tl = (int32_t*)smem;                                          // [N] the order
    uint16_t* rt = (uint16_t*)(smem + sizeof(int32_t) * N);                // [NH][QB][N]
    unsigned char* ct = (unsigned char*)(rt + (size_t)NH * QB * N);        // [N] rows of kCtRowBytes
    __shared__ int red_i[2][NW];
    __shared__ unsigned long long red_k[NW];
    // SPLIT threads per rank p share the rank's steps (part 0 takes the first half of every block of partners): with one
    // thread per rank at N = 512 a SIMD holds two wavefronts, too few to overlap one's LDS gathers with the other's
    // arithmetic
    const int tid = threadIdx.x, p = tid & (N - 1), part = tid >> LOGN, lane = tid & 63, wv = tid >> 6;
    const int64_t r = blockIdx.x;
    int t = clampi(tours[r * N + p], 0, N - 1);
    if (part == 0) tl[p] = t;
    __syncthreads();
    int parity = 0;
    auto block_max = [&](int v) {                              // every thread gets the maximum; one barrier per call
        v = wave_max(v);
        if (lane == 0) red_i[parity][wv] = v;
        __syncthreads();
        int o;
        if (NW >= 16) {
            o = wave_max(red_i[parity][lane & (NW - 1)]);
        } else {
            o = red_i[parity][0];
#pragma unroll
            for (int k = 1; k < NW; ++k) o = max(o, red_i[parity][k]);
        }
        parity ^= 1;
        return o;
    };

    int applied = 0, cur = 0;
    for (;;) {
        // per round: the mate's node, the largest and second largest link that is not this rank's, and the two ranks
        // (with the round's bit set) of that largest link
        int pbq[LOGN], x1v[LOGN], x2v[LOGN], a1r[LOGN], round_cost[LOGN];
        cur = 0;
#pragma unroll
        for (int k = 0; k < LOGN; ++k) {
            const int bit = 1 << k;
            const int pb = tl[p ^ bit];
            pbq[k] = pb * kCtRowBytes;                         // the mate's node as a row byte offset of CT
            const int lv = (int)folded[t * N + pb];
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
            const int al = a1 & (N / 2 - 1);
            a1r[k] = (((al >> k) << (k + 1)) | (al & (bit - 1))) | bit;    // link index -> its rank with bit k set
            round_cost[k] = __builtin_amdgcn_readfirstlane(k1 >> LB);
            cur += round_cost[k];
        }
        int best_below = kInf, best_above = kInf;              // over partners q < p and q > p: total << LOGN | q
        // pairs of round mates, scored by the thread whose bit is clear
#pragma unroll 1
        for (int km = 0; km < LOGN; ++km) {
            const int q = p ^ (1 << km);
            if (q < p || (km & (SPLIT - 1)) != part) continue;
            const int tq = tl[q];
            int total = 0;
#pragma unroll
            for (int k = 0; k < LOGN; ++k) {
                const int bit = 1 << k;
                const int link_p = (int)folded[tq * N + tl[p ^ bit]];
                const int link_q = (int)folded[t * N + tl[q ^ bit]];
                const int others = ((q | bit) == a1r[k]) ? x2v[k] : x1v[k];
                const int stage = max(others, max(link_p, link_q));
                total += (k == km) ? round_cost[k] : stage;
            }
            best_above = min(best_above, (total << LOGN) | q);
        }
        const int tq2 = t * kCtRowBytes, tc2 = t << 1;
#pragma unroll 1
        for (int b0 = 0; b0 < N; b0 += QB) {
            __syncthreads();                                   // the tiles of the previous block are free
            // all loads of the block first, then the stores: one L2 latency per block
            // RT: NH * QB rows of N entries, copied 16 bytes at a time; CT: row p, the block's QB columns
            constexpr int kChunksPerRow = N * 2 / 16, kChunks = NH * QB * kChunksPerRow, kPerThread = kChunks / NT;
            static_assert(kChunks % NT == 0, "every thread copies the same number of 16-byte pieces");
            int4 piece[kPerThread];
#pragma unroll
            for (int i = 0; i < kPerThread; ++i) {
                const int ch = tid + i * NT;
                const int rowi = ch / kChunksPerRow, off = ch % kChunksPerRow;
                const int h = rowi >> LOGQ, j = rowi & (QB - 1);
                const int node = tl[(b0 + j) ^ (QB << h)];
                piece[i] = ((const int4*)(folded + (size_t)node * N))[off];
            }
            {
                // F is symmetric: column t[B + j] is read as row t[B + j], which the threads of a wave read side by side
                const uint16_t* col = folded + p;
                constexpr int kWords = QB / 2 / SPLIT;             // words of row p that this thread stages
                const int j0 = part * kWords;
                uint32_t w[kWords];
#pragma unroll
                for (int j = 0; j < kWords; ++j)
                    w[j] = (uint32_t)col[(size_t)tl[b0 + 2 * (j0 + j)] * N] |
                           ((uint32_t)col[(size_t)tl[b0 + 2 * (j0 + j) + 1] * N] << 16);
#pragma unroll
                for (int j = 0; j < kWords; ++j) ((uint32_t*)(ct + p * kCtRowBytes))[j0 + j] = w[j];
            }
#pragma unroll
            for (int i = 0; i < kPerThread; ++i) ((int4*)rt)[tid + i * NT] = piece[i];
            __syncthreads();
            constexpr int kSteps = QB / 2 / SPLIT;
#pragma unroll 2
            for (int ii = 0; ii < kSteps; ++ii) {
                const int i = part * kSteps + ii;
                const int q0 = b0 + 2 * i;
                const bool above = p > q0;                     // p = q0 + 1 takes q0; p = q0 sits this step out
                const int q = q0 + (((p ^ q0) & 1) ^ (above ? 1 : 0));
                const int j = q - b0, j2 = j << 1;
                const int x = p ^ q;
                int total = 0;
#pragma unroll
                for (int k = 0; k < LOGN; ++k) {
                    const int bit = 1 << k;
                    const int link_p = (int)*(const uint16_t*)((const char*)ct + (pbq[k] + j2));
                    int link_q;
                    if (k < LOGQ) link_q = (int)*(const uint16_t*)((const char*)ct + (tq2 + (j2 ^ (bit << 1))));
                    else link_q = (int)*(const uint16_t*)((const char*)rt + ((((k - LOGQ) << LOGQ) + j) << (LOGN + 1)) + tc2);
                    const int others = ((q | bit) == a1r[k]) ? x2v[k] : x1v[k];
                    total += max(others, max(link_p, link_q));
                }
                const bool skip = (x & (x - 1)) == 0;          // itself (x = 0) or a round mate (scored above)
                const int key = skip ? kInf : ((total << LOGN) | q);
                best_below = min(best_below, above ? key : kInf);
                best_above = min(best_above, above ? kInf : key);
            }
        }
        unsigned long long best = kNoMove;
        if (best_below != kInf) {
            const int q = best_below & (N - 1), total = best_below >> LOGN;
            best = ((unsigned long long)(unsigned)total << kIdBits) | (unsigned)(q * N + p);
        }
        if (best_above != kInf) {
            const int q = best_above & (N - 1), total = best_above >> LOGN;
            best = min(best, ((unsigned long long)(unsigned)total << kIdBits) | (unsigned)(p * N + q));
        }
        best = wave_min_u64(best);
        if (lane == 0) red_k[wv] = best;
        __syncthreads();
        unsigned long long win;
        if (NW >= 16) {
            win = wave_min_u64(red_k[lane & (NW - 1)]);
        } else {
            win = red_k[0];
#pragma unroll
            for (int k = 1; k < NW; ++k) win = min(win, red_k[k]);
        }
        if ((int)(win >> kIdBits) >= cur) break;
        const int id = (int)(win & ((1u << kIdBits) - 1u)), sp = id >> LOGN, sq = id & (N - 1);
        const int a = tl[sp], b = tl[sq];
        __syncthreads();                                       // everyone has read red_k and the two ranks
        if (p == sp) { t = b; if (part == 0) tl[p] = b; }
        if (p == sq) { t = a; if (part == 0) tl[p] = a; }
        ++applied;
        __syncthreads();
    }
    if (part == 0) tours[r * N + p] = t;
    if (tid == 0) {
        costs[r] = (int64_t)cur;
        moves[r] = applied;
    }
}

template <int LOGN, int LOGQ, int SPLIT>
static hipError_t rdswap_tiled_launch(const int32_t* c, uint16_t* folded, int restarts, int32_t* tours, int64_t* costs,
                                      int32_t* moves, const int32_t* flags, hipStream_t s) {
    constexpr int N = 1 << LOGN, QB = 1 << LOGQ, NH = LOGN - LOGQ;
    hipError_t e = launch_fold_to_u16(c, N, folded, flags, s);
    if (e != hipSuccess) return e;
    const size_t lds = sizeof(int32_t) * N + sizeof(uint16_t) * (size_t)NH * QB * N + (size_t)N * (QB / 2 + 1) * 4;
    e = hipFuncSetAttribute((const void*)rdswap_tiled_kernel<LOGN, LOGQ, SPLIT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((rdswap_tiled_kernel<LOGN, LOGQ, SPLIT>), dim3(restarts), dim3(SPLIT * N), lds, s, folded, tours, costs, moves,
                       flags);
    return hipGetLastError();
}

template <int LOGN>
static hipError_t rdswap_block_launch(const int32_t* c, uint16_t* folded, int restarts, int32_t* tours, int64_t* costs,
                                      int32_t* moves, const int32_t* flags, hipStream_t s) {
    constexpr int N = 1 << LOGN;
    constexpr bool kInLds = LOGN <= 8;
    if (!kInLds) {
        hipError_t e = launch_fold_to_u16(c, N, folded, flags, s);
        if (e != hipSuccess) return e;
    }
    // matrix in LDS: a workgroup of 1024 threads whatever N (16 wavefronts on the restart's compute unit); through
    // L2 more wavefronts only queue up behind the same misses (N = 512: 0.57 s with two threads per rank, 0.47 s with one)
    constexpr int kSplit = kInLds ? 1024 / N : 1;
    const size_t lds = (kInLds ? sizeof(uint16_t) * N * N : 0) + sizeof(int32_t) * N;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)rdswap_block_kernel<LOGN, kInLds, kSplit>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((rdswap_block_kernel<LOGN, kInLds, kSplit>), dim3(restarts), dim3(N * kSplit), lds, s, c, folded,
                       tours, costs, moves, flags);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_fold_to_u16(const int32_t* c, int N, uint16_t* folded, const int32_t* flags, hipStream_t s) {
    hipLaunchKernelGGL(fold_to_u16_kernel, dim3(512), dim3(256), 0, s, c, N, folded, flags);
    return hipGetLastError();
}

hipError_t launch_rdswap(const int32_t* c, int N, int restarts, uint64_t seed, bool tours_hold_init, int32_t* tours,
                         int64_t* costs, int32_t* moves, int32_t* flags, uint16_t* mat16, hipStream_t s) {
    const bool pinned = force_general_path();
    if (N == 64 && !pinned) {
        hipLaunchKernelGGL(rdswap_n64_kernel, dim3((restarts + 3) / 4), dim3(256), 0, s, c, restarts, seed,
                           tours_hold_init ? 0 : 1, tours, costs, moves);
        return hipGetLastError();
    }
    if (!tours_hold_init) {
        hipError_t e = launch_init_tours(N, 0, restarts, seed, tours, s);
        if (e != hipSuccess) return e;
    }
    const int32_t* skip = nullptr;
    if (!pinned && (N == 128 || N == 256 || N == 512 || N == 1024)) {
        // 16-bit workgroup kernel when max(c) < 2^16, else the general kernel: both are enqueued and the matrix
        // maximum, computed on the device, decides which one does the work (no host round trip)
        hipError_t e = launch_matrix_max(c, N, flags, s);
        if (e != hipSuccess) return e;
        e = N == 128   ? rdswap_block_launch<7>(c, mat16, restarts, tours, costs, moves, flags, s)
            : N == 256 ? rdswap_block_launch<8>(c, mat16, restarts, tours, costs, moves, flags, s)
            : N == 512 ? rdswap_tiled_launch<9, 4, 2>(c, mat16, restarts, tours, costs, moves, flags, s)
                       : rdswap_tiled_launch<10, 3, 1>(c, mat16, restarts, tours, costs, moves, flags, s);
        if (e != hipSuccess) return e;
        skip = flags;
    }
    const int threads = ((N + 63) / 64) * 64;
    hipLaunchKernelGGL(rdswap_general_kernel, dim3(restarts), dim3(threads), sizeof(int32_t) * 2 * (size_t)N, s, c, N,
                       tours, costs, moves, skip);
    return hipGetLastError();
}

}  // namespace cc
