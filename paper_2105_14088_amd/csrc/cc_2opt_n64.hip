// 2-opt descent for N = 64, ring-sum objective on a symmetric matrix: one wavefront per restart, the
// tour in one VGPR (lane p holds t[p]), the cost matrix staged once per workgroup in LDS.
//
// Neighbourhood as cyclic diagonals.  A 2-opt move exchanges two non-adjacent ring edges.  Number the
// edges by their upper rank: edge p joins ranks p-1 and p (edge 0 joins 63 and 0).  Exchanging edges a
// and b replaces them by (t[a-1], t[b-1]) and (t[a], t[b]), so with G(p, q) = c[t[p]][t[q]]
//     delta(a, b) = G(a-1, b-1) + G(a, b) - f[a] - f[b],      f[p] = c[t[p]][t[p-1]].
// Both new hops sit on the same cyclic diagonal d = b - a of G, in adjacent lanes.  Lane a therefore
// needs ONE gather per move, D_d[a] = G(a, a+d), and takes G(a-1, a-1+d) from lane a-1 with a DPP
// wave rotate.  Diagonals d = 2 .. 32 cover every unordered pair of non-adjacent edges (d = 32 twice),
// i.e. all N(N-3)/2 = 1952 moves in 31 fully occupied wave steps; no lane is ever masked.
// In move terms: edges {a, b}, lo = min, hi = max, is the reversal of ranks lo .. hi-1, or, when
// lo = 0 (the edge into the anchor), of ranks hi .. 63; these are exactly the moves (i, j) of cc.h.
//
// Keys.  Per lane the running minimum is kept over   key = (delta' << 14) | rank(b) << 8 | 4*t[b]
// where delta' = G + G - f[b] (the lane's own -f[a] is added after the sweep), rank(b) = (b-1) mod 64
// orders the partners of one lane exactly as their move ids are ordered, and the low byte is the
// column byte-offset of node t[b], which makes the gather address a single v_and_or.  The value
// packed[b] = (-f[b] << 14) | rank(b) << 8 | 4*t[b] travels round the wave by one lane per diagonal
// (DPP wave rotate), and the matrix is stored pre-shifted (c << 14), so a key costs two adds.
// This needs |delta| < 2^17, i.e. max(c) < 2^16; larger matrices (up to 2^21 - 1) take the same
// sweep with 64-bit keys.  After the sweep each lane turns its best partner into the move id
// i*64 + j, and (delta << 12 | id) is min-reduced over the wave with DPP row operations: the result
// is the lexicographic minimum of (value, id) over the whole neighbourhood, whatever the visit order.
#include <type_traits>

#include "cc_device.h"
#include "cc_internal.h"
#include "cc_wave64.h"
#include "cc_2opt_n64_loop.inc"

namespace cc {
using namespace ccd;

namespace {

using namespace w64;
constexpr int kSh = 14;           // key = delta << 14 | rank << 8 | column byte offset
constexpr int kIdBits = 12;       // move id i*64 + j
constexpr int kCostMax = (1 << 21) - 1;

// One descent.  m: LDS matrix, entries c << 14 (narrow) or c (wide).  Returns the final tour in t.
template <bool WIDE>
__device__ __forceinline__ void descend(const int32_t* m, int lane, int& t, long long& cost, int& applied_out) {
    using K = typename std::conditional<WIDE, long long, int>::type;
    using UK = typename std::conditional<WIDE, unsigned long long, unsigned>::type;
    const int rank_a = (lane + kN - 1) & (kN - 1);
    const int rank_bits = rank_a << 8;
    const int id_base = lane * kN, id_base_flipped = kN + rank_a;
    const char* mbytes = (const char*)m;
    long long cur = 0;
    int applied = 0;
    bool first = true;
    for (;;) {
        // hop into rank `lane`, and the value that represents this rank as a partner b
        const int tprev = from_prev_lane(t);
        const int fm = m[t * kN + tprev];
        const K negf = WIDE ? (K)(0 - ((UK)(unsigned)fm << kSh)) : (K)(0 - (UK)fm);
        K pk = (K)((UK)negf + (UK)(rank_bits + 4 * t));
        if (first) {
            cur = wave_sum64((long long)(WIDE ? fm : (fm >> kSh)));
            first = false;
        }
        const int rowofs = t * (kN * 4);
        pk = from_next_lane(from_next_lane(pk));        // packed[a + 2]
        // phase 1: every diagonal's partner value and gather address; gathers go out as early as possible
        K pkd[kN / 2 + 1];
        int D[kN / 2 + 1];
#pragma unroll
        for (int d = 2; d <= kN / 2; ++d) {
            pkd[d] = pk;
            const int off = ((int)pk & 0xff) | rowofs;
            D[d] = *(const int32_t*)(mbytes + off);             // G(a, a+d)
            if (d < kN / 2) pk = from_next_lane(pk);
        }
        // phase 2: combine with the neighbour lane's gather, keep the minimum
        K best = WIDE ? (K)0x7fffffffffffffffll : (K)0x7fffffff;
#pragma unroll
        for (int d = 2; d <= kN / 2; ++d) {
            const int E = from_prev_lane(D[d]);                 // G(a-1, a-1+d)
            const K key = WIDE ? (K)(((UK)(unsigned)(E + D[d]) << kSh) + (UK)pkd[d])
                               : (K)((UK)E + (UK)D[d] + (UK)pkd[d]);
            best = key < best ? key : best;
        }
        best = (K)((UK)best + (UK)negf);
        // partner -> move id (lowest id among this lane's best partners is already selected by rank).  With
        // r = rank(b) and ra = rank(lane): the move is (lane, r) when r >= ra (b lies after the lane, or b = 0), and
        // (r + 1, ra) otherwise, i.e. id = lane*64 + r or r*64 + 64 + ra.
        const int r = ((int)best >> 8) & (kN - 1);
        const K delta = best >> kSh;
        const int id_l = r < rank_a ? (r << 6) + id_base_flipped : id_base + r;
        const K key2 = (K)(((UK)delta << kIdBits) | (UK)id_l);
        const K win = wave_min_uniform(key2);
        const K dwin = win >> kIdBits;
        if (dwin >= 0) break;
        const int id = (int)win & ((1 << kIdBits) - 1);
        const int mi = id >> 6, mj = id & (kN - 1);
        const int src = (unsigned)(lane - mi) <= (unsigned)(mj - mi) ? mi + mj - lane : lane;
        t = __shfl(t, src, kWave);
        cur += (long long)dwin;
        ++applied;
    }
    cost = cur;
    applied_out = applied;
}

// The same descent for matrices with entries below 2^16, as one hand-scheduled loop (cc_2opt_n64_loop.inc, written by
// gen_2opt_n64_loop.py).  m holds c << 14.  State across sweeps: the order t and the hop array fm = f << 14 (hop into
// rank `lane`), both one register per lane.  After a move that reverses ranks mi .. mj the hops of the reversed piece
// are the old ones read from the other end (the matrix is symmetric), so fm follows the order by the same lane
// permute, shifted by one rank, and only the two new hops are written: y = c[t[mi]][t[mj+1]] is the matrix entry the
// winning lane gathered for its best candidate, x = c[t[mi-1]][t[mj]] = delta + f[mi] + f[mj+1] - y.
__device__ __forceinline__ void descend_narrow(const int32_t* m, int lane, int& t, long long& cost, int& applied_out) {
    const int rank_a = (lane + kN - 1) & (kN - 1);
    const int rank_bits = rank_a << 8;
    const int id_base = lane * kN, id_flip = kN + rank_a;
    const int mbase = (int)(unsigned)(uintptr_t)(const char*)m;      // LDS byte offset of the matrix (256-byte aligned)
    const int lane4 = lane << 2;
    int applied = 0;
    int fm = m[t * kN + from_prev_lane(t)];
    int cur = wave_sum(fm >> kSh);
    // every operand that is written is marked early-clobber: the loop writes them long before it has read the last input
    asm volatile(CC_N64_DESCENT_LOOP_ASM
                 : [t] "+&v"(t), [fm] "+&v"(fm), [cur] "+&s"(cur), [applied] "+&s"(applied)
                 : [rank_bits] "v"(rank_bits), [ra] "v"(rank_a), [id_base] "v"(id_base), [id_flip] "v"(id_flip),
                   [lane] "v"(lane), [lane4] "v"(lane4), [mbase] "s"(mbase), [mask] "s"(0xff), [himask] "s"(0xfffff000)
                 : CC_N64_DESCENT_LOOP_CLOBBERS);
    cost = cur;
    applied_out = applied;
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 2))) void twoopt_sum_n64_kernel(const int32_t* __restrict__ c, int restarts,
                                                             uint64_t seed, int generate,
                                                             int32_t* __restrict__ tours,
                                                             int64_t* __restrict__ costs,
                                                             int32_t* __restrict__ moves) {
    __shared__ __attribute__((aligned(256))) int32_t m[kN * kN];
    __shared__ int wave_max_entry[4];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;

    // the matrix loads are issued first and stay in flight while the wave builds its initial tour
    int v[kN * kN / 256];
#pragma unroll
    for (int k = 0; k < kN * kN / 256; ++k) v[k] = c[tid + 256 * k];
    const int64_t r = (int64_t)blockIdx.x * 4 + wv;
    int t = 0;
    if (r < restarts)
        t = generate ? init_tour_in_wave(seed, (uint32_t)r, lane) : clampi(tours[r * kN + lane], 0, kN - 1);
    // entries are clamped to the contract range so that all arithmetic stays exact
    int mx = 0;
#pragma unroll
    for (int k = 0; k < kN * kN / 256; ++k) {
        v[k] = clampi(v[k], 0, kCostMax);
        mx = max(mx, v[k]);
    }
    mx = wave_max(mx);
    if (lane == 0) wave_max_entry[wv] = mx;
    __syncthreads();
    mx = max(max(wave_max_entry[0], wave_max_entry[1]), max(wave_max_entry[2], wave_max_entry[3]));
    const bool wide = mx >= (1 << 16);
    // stage, pre-shifted when 32-bit keys suffice
#pragma unroll
    for (int k = 0; k < kN * kN / 256; ++k) m[tid + 256 * k] = wide ? v[k] : (v[k] << kSh);
    __syncthreads();
    // the search reads the matrix through its upper triangle: exact deltas, hence a descent that ends, whatever
    // the caller's matrix holds
    mirror_upper_triangle_64(m, tid);
    __syncthreads();
    if (r >= restarts) return;
    long long cost;
    int applied;
    if (wide) descend<true>(m, lane, t, cost, applied);
    else descend_narrow(m, lane, t, cost, applied);
    tours[r * kN + lane] = t;
    if (lane == 0) {
        costs[r] = cost;
        moves[r] = applied;
    }
}

}  // namespace

hipError_t launch_2opt_sum_n64(const int32_t* c, int restarts, uint64_t seed, bool generate, int32_t* tours,
                               int64_t* costs, int32_t* moves, hipStream_t s) {
    const int grid = (restarts + 3) / 4;
    hipLaunchKernelGGL(twoopt_sum_n64_kernel, dim3(grid), dim3(256), 0, s, c, restarts, seed, generate ? 1 : 0, tours,
                       costs, moves);
    return hipGetLastError();
}

}  // namespace cc
