// Simulated annealing over the ring (Section 4.3: stochastic search by simulated annealing, neighbours
// obtained by reversing a random sub-array).  Proposal, temperature schedule and the integer acceptance
// rule are stated in cc.h, cc_sa_search.
//
// One wavefront per chain; the order lives in LDS.  A chain is sequential, but a rejected proposal
// leaves the order untouched, so the 64 lanes evaluate the proposals of the next 64 steps against the
// current order at once; the wave then commits the FIRST accepted one (ballot + find-first-set), and
// the steps after it are proposed again in the next round against the new order.  The result is the
// sequential chain bit for bit; a round advances 1 .. 64 steps, most of them when the chain is cold.
// What a step draws does not depend on the order: its two ring edges and the acceptance threshold E(u).  The wave
// therefore draws 64 steps at a time, one per lane (counter-based generator), into a ring of 128 entries in LDS,
// and a round only reads its entry back; steps that are proposed again after a commit cost no second draw.
// Per round a lane then gathers four ranks of the order and four matrix entries (LDS for N <= 128, else through
// L2) and tests acceptance in 64-bit integer arithmetic.  The committed reversal is done by the whole wave, one
// pair of ranks per lane.
#include "cc_device.h"
#include "cc_internal.h"
#include "cc_wave64.h"

namespace cc {
using namespace ccd;

namespace {

constexpr int kCostMax = (1 << 21) - 1;
constexpr int kDrawBase = 1024;       // low counter words below this belong to the initial shuffles
constexpr int kDrawRing = 128;        // steps whose draws a wave keeps in LDS (two blocks of 64)

// all LDS traffic of the wave issued so far is complete and visible to every lane, and the compiler keeps
// LDS accesses on their side of this point
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The acceptance rule of cc.h, "delta * 4096 * steps <= (t_start * (steps - s) + t_end * s) * E(u)", turned into
// the largest cost increase step s accepts: delta is an integer, so the rule is delta <= floor(right side / (4096 *
// steps)), and a non-positive delta passes as well (the right side is never negative).  One 64-bit division per step,
// done where the step's random word is drawn (once per step, 64 steps at a time); the search loop then compares.
__device__ __forceinline__ int largest_accepted_increase(long long step, long long steps, int t_start, int t_end, int u) {
    const int e = 31 - __clz(u);
    const int mant = u - (1 << e);
    const int frac = e >= 12 ? (mant >> (e - 12)) : (mant << (12 - e));
    const unsigned long long E = (unsigned long long)(22 * 4096 - (e * 4096 + frac));
    const unsigned long long num = (unsigned long long)((long long)t_start * (steps - step) + (long long)t_end * step);
    return (int)((num * E) / (4096ull * (unsigned long long)(steps > 0 ? steps : 1)));       // below 22 * 2^21
}

// MAT: where the matrix is read from - 0 through L2, 1 staged in LDS as int32 (N <= 128), 2 staged in LDS as 16-bit
// entries (N <= 256) when every entry is in 0 .. 2^16 - 1 (found while staging), else through L2.
template <int MAT>
__global__ __launch_bounds__(256) void sa_ring_kernel(const int32_t* __restrict__ c, int N, int chains,
                                                      long long steps, int t_start, int t_end, uint64_t seed,
                                                      int32_t* __restrict__ tours, int64_t* __restrict__ costs,
                                                      int32_t* __restrict__ accepted) {
    extern __shared__ __attribute__((aligned(16))) int32_t sm[];
    const int lane = lane_id(), wv = threadIdx.x >> 6;
    int32_t* draws = sm + wv * 2 * kDrawRing;            // per step: edges a | b << 16, threshold E
    int32_t* t = sm + 8 * kDrawRing + wv * 2 * N;        // current order
    int32_t* bt = t + N;                                 // best order so far
    const int32_t* mat = c;
    const uint16_t* m16 = nullptr;
    bool narrow = false;                                 // MAT == 2: the 16-bit copy holds the matrix
    if (MAT == 1) {
        int32_t* m = sm + 8 * kDrawRing + 8 * N;
        for (int e = threadIdx.x; e < N * N; e += 256) m[e] = clampi(c[e], 0, kCostMax);
        __syncthreads();
        mat = m;
    }
    if (MAT == 2) {
        uint16_t* m = (uint16_t*)(sm + 8 * kDrawRing + 8 * N);
        __shared__ unsigned wave_top[4];
        unsigned top = 0;
        for (int e = threadIdx.x; e < N * N; e += 256) {
            const unsigned v = (unsigned)c[e];           // a negative entry counts as too large
            top = max(top, v);
            m[e] = (uint16_t)v;
        }
        top = (unsigned)wave_max((int)min(top, 0x7fffffffu));
        if (lane == 0) wave_top[wv] = top;
        __syncthreads();
        narrow = max(max(wave_top[0], wave_top[1]), max(wave_top[2], wave_top[3])) < (1u << 16);
        m16 = m;
    }
    const int64_t r = (int64_t)blockIdx.x * 4 + wv;
    if (r >= chains) return;
    auto M = [&](int x, int y) {
        if (MAT == 1) return mat[x * N + y];
        if (MAT == 2 && narrow) return (int)m16[x * N + y];
        return clampi(c[x * N + y], 0, kCostMax);
    };

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
        // draws of the 64 steps first .. first + 63, one per lane, into their ring entries
        auto draw_block = [&](long long first) {
            const long long step = first + lane;
            const uint64_t w = splitmix64_at(seed, (chain_hi | (uint32_t)(kDrawBase + (uint32_t)step)) + 1u);
            const int a = (int)(((uint32_t)(w >> 43) * (uint32_t)N) >> 21);
            const int d = 2 + (int)((((uint32_t)(w >> 22) & 0x1FFFFFu) * (uint32_t)(N - 3)) >> 21);
            int b = a + d;
            b = b >= N ? b - N : b;
            const int u = (int)((uint32_t)w & 0x3FFFFFu) + 1;
            const int slot = (int)step & (kDrawRing - 1);
            *(int2*)(draws + 2 * slot) = make_int2(a | (b << 16), largest_accepted_increase(step, steps, t_start, t_end, u));
        };
        draw_block(0);
        draw_block(kWave);
        long long drawn = 2 * kWave;          // steps [drawn - 128, drawn) are in the ring
        wave_lds_sync();
        long long s = 0;
        while (s < steps) {
            if (s + kWave > drawn) {          // the round reaches past the ring: the older half makes room
                draw_block(drawn);
                drawn += kWave;
                wave_lds_sync();
            }
            const long long step = s + lane;
            const bool active = step < steps;
            const int2 drawn_step = *(const int2*)(draws + 2 * ((int)step & (kDrawRing - 1)));
            const int a = drawn_step.x & 0xffff, b = drawn_step.x >> 16;
            const int ap = a ? a - 1 : N - 1, bp = b ? b - 1 : N - 1;
            const int ta = t[a], tap = t[ap], tb = t[b], tbp = t[bp];
            const int delta = M(tap, tbp) + M(ta, tb) - M(ta, tap) - M(tb, tbp);
            const bool accept = active && delta <= drawn_step.y;
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
// Under this max-type objective most proposals are neutral and therefore accepted, so speculation over later steps
// does not pay; instead the wave scores ONE proposal per step with its lanes spread over the work.  A proposal
// exchanges ranks p and q; per round only the links of p and of q change, so the new round cost is
// max(link of p re-evaluated, link of q re-evaluated, largest link among the others), the last term being one of
// the round's three largest links.  Lane l handles round l >> 2, side (l >> 1) & 1 (p's or q's link) and direction
// l & 1 of that link: one gather per lane, the two directions and the two sides meet through quad permutes, the
// rounds through one wave sum.  The four lanes of a round also hold the round's three largest links
// (keys value << 10 | lower rank).  After a commit they update them from what they already have: the old three
// without p's and q's links, plus those two links' new values; that is the round's true top three whenever its
// third key is not below the old third value (every other link is at most that); otherwise the whole wave
// recomputes the round from the order (three max-reductions over value << 9 | link index).
template <int LOGN>
__global__ __launch_bounds__(256) void sa_rd_kernel(const int32_t* __restrict__ c, int chains, long long steps,
                                                    int t_start, int t_end, uint64_t seed,
                                                    int32_t* __restrict__ tours, int64_t* __restrict__ costs,
                                                    int32_t* __restrict__ accepted) {
    constexpr int N = 1 << LOGN;
    constexpr bool LDS_MATRIX = LOGN <= 7;
    constexpr int LINKS = N / 2;
    constexpr int U = LINKS > 64 ? LINKS / 64 : 1;      // links per lane when the wave recomputes a round
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

    const int my_round = lane >> 2, side = (lane >> 1) & 1, dir = lane & 1;
    const bool in_play = my_round < LOGN;
    const int my_bit = 1 << (in_play ? my_round : 0);
    int k1 = -1, k2 = -1, k3 = -1;                      // this lane's round: its three largest links, value << 10 | lower rank

    // the wave recomputes round kk from the order in LDS; the lanes of that round take the result
    auto recompute_round = [&](int kk) {
        const int bit = 1 << kk;
        int key[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = lane + 64 * u;                // link index
            const int j = ((i >> kk) << (kk + 1)) | (i & (bit - 1));
            key[u] = -1;
            if (i < LINKS) {
                const int a = t[j], b = t[j | bit];
                key[u] = (max(M(a, b), M(b, a)) << 9) | i;
            }
        }
        int found[3];
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
            found[pass] = best < 0 ? -1 : (((best >> 9) << 10) | ((i >> kk) << (kk + 1)) | (i & (bit - 1)));
            if (pass == 0) taken0 = best < 0 ? -2 : i;
            else taken1 = best < 0 ? -2 : i;
        }
        if (my_round == kk) {
            k1 = found[0];
            k2 = found[1];
            k3 = found[2];
        }
    };
    for (int kk = 0; kk < LOGN; ++kk) recompute_round(kk);
    int cur = wave_sum((in_play && (lane & 3) == 0) ? (k1 >> 10) : 0);
    int best = cur;
    int acc = 0;
    const uint64_t chain_hi = (uint64_t)(uint32_t)r << 32;

    for (long long s = 0; s < steps; ++s) {
        const uint64_t w = splitmix64_at(seed, (chain_hi | (uint32_t)(kDrawBase + (uint32_t)s)) + 1u);
        const int p = (int)(((uint32_t)(w >> 43) * (uint32_t)N) >> 21);
        const int d = 1 + (int)((((uint32_t)(w >> 22) & 0x1FFFFFu) * (uint32_t)(N - 1)) >> 21);
        const int q = (p + d) & (N - 1);
        const int u = (int)((uint32_t)w & 0x3FFFFFu) + 1;
        // this lane's link: rank `mine` (p or q) receives the node of the other rank; its partner keeps its node
        const int mine = side ? q : p, other = side ? p : q;
        const int x = t[other], y = t[mine ^ my_bit];
        const int val = in_play ? (dir ? M(y, x) : M(x, y)) : 0;
        const int link = max(val, __builtin_amdgcn_update_dpp(val, val, 0xB1, 0xf, 0xf, true));        // both directions
        const int link_other = __builtin_amdgcn_update_dpp(link, link, 0x4E, 0xf, 0xf, true);          // the other side
        const int link_p = side ? link_other : link, link_q = side ? link : link_other;
        const int lp = p & ~my_bit, lq = q & ~my_bit;
        const bool same_link = lp == lq;               // q = p xor bit: the link keeps both nodes and its value
        const int j1 = k1 & 1023, j2 = k2 & 1023;
        const bool f1 = j1 != lp && j1 != lq, f2 = j2 != lp && j2 != lq;
        const int others = (f1 ? k1 : (f2 ? k2 : k3)) >> 10;       // -1 when the round has no other link
        const int stage = same_link ? (k1 >> 10) : max(others, max(link_p, link_q));
        const int total = wave_sum((in_play && (lane & 3) == 0) ? stage : 0);
        const int delta = total - cur;
        bool accept = true;
        if (delta > 0) {
            const int e = 31 - __clz(u);
            const int mant = u - (1 << e);
            const int frac = e >= 12 ? (mant >> (e - 12)) : (mant << (12 - e));
            const long long E = 22 * 4096 - (e * 4096 + frac);
            const long long num = (long long)t_start * (steps - s) + (long long)t_end * s;
            accept = (long long)delta * 4096 * steps <= num * E;
        }
        if (!accept) continue;                          // wave-uniform
        wave_lds_sync();                               // every lane has read the order before it changes
        const int node_q = __builtin_amdgcn_readlane(x, 0), node_p = __builtin_amdgcn_readlane(x, 2);   // sides 0 and 1
        if (lane == 0) {
            t[p] = node_q;
            t[q] = node_p;
        }
        cur += delta;
        ++acc;
        // the round's three largest links after the exchange
        bool stale = false;
        if (in_play && !same_link) {
            const int f3 = (k3 & 1023) != lp && (k3 & 1023) != lq;
            int c0 = f1 ? k1 : -1, c1 = f2 ? k2 : -1, c2 = (f3 && k3 >= 0) ? k3 : -1;
            if (k1 < 0) c0 = -1;
            if (k2 < 0) c1 = -1;
            int c3 = (link_p << 10) | lp, c4 = (link_q << 10) | lq;
            const int bound = k3 >> 10;                // every link outside the candidates is at most this
            const int n1 = max(max(c0, c1), max(max(c2, c3), c4));
            c0 = c0 == n1 ? -1 : c0; c1 = c1 == n1 ? -1 : c1; c2 = c2 == n1 ? -1 : c2;
            c3 = c3 == n1 ? -1 : c3; c4 = c4 == n1 ? -1 : c4;
            const int n2 = max(max(c0, c1), max(max(c2, c3), c4));
            c0 = c0 == n2 ? -1 : c0; c1 = c1 == n2 ? -1 : c1; c2 = c2 == n2 ? -1 : c2;
            c3 = c3 == n2 ? -1 : c3; c4 = c4 == n2 ? -1 : c4;
            const int n3 = max(max(c0, c1), max(max(c2, c3), c4));
            stale = LINKS > 3 && (n3 >> 10) < bound;
            k1 = n1; k2 = n2; k3 = n3;
        }
        wave_lds_sync();
        unsigned long long redo = __ballot(stale);
        while (redo) {
            const int kk = (__ffsll((long long)redo) - 1) >> 2;
            recompute_round(kk);
            redo &= ~(0xFull << (4 * kk));
        }
        if (cur < best) {
            best = cur;
            for (int z = lane; z < N; z += kWave) bt[z] = t[z];
        }
    }
    wave_lds_sync();
    for (int z = lane; z < N; z += kWave) tours[r * N + z] = bt[z];
    if (lane == 0) {
        costs[r] = (int64_t)best;
        accepted[r] = acc;
    }
}

// N = 64: the chain of sa_rd_kernel with everything a step touches in registers.  The order is one VGPR (lane =
// rank): the two nodes of a proposal are lane reads by a scalar index, a link's far end one lane permute, the exchange
// two selects, the best order a register copy.  The matrix is folded in LDS (the larger of the two directed entries
// in both places), so a link is one gather and a step needs 12 lanes: lane 2r + side scores, for round r, the link of
// p (side 0) or q (side 1).  What a step draws does not depend on the order: 64 steps are drawn at once, one per lane
// (ranks p and q, and the acceptance threshold already as E(u)), and read back by step number.
__global__ __launch_bounds__(256) void sa_rd_n64_kernel(const int32_t* __restrict__ c, int chains, long long steps,
                                                        int t_start, int t_end, uint64_t seed,
                                                        int32_t* __restrict__ tours, int64_t* __restrict__ costs,
                                                        int32_t* __restrict__ accepted) {
    constexpr int N = 64, LOGN = 6;
    __shared__ int32_t m[N * N];
    const int lane = lane_id(), wv = threadIdx.x >> 6;
    for (int e = threadIdx.x; e < N * N; e += 256) m[e] = clampi(c[e], 0, kCostMax);
    __syncthreads();
    w64::for_each_pair_64((int)threadIdx.x, [&](int lo, int hi) {
        const int both = max(m[lo * N + hi], m[hi * N + lo]);
        m[lo * N + hi] = both;
        m[hi * N + lo] = both;
    });
    __syncthreads();
    const int64_t r = (int64_t)blockIdx.x * 4 + wv;
    if (r >= chains) return;
    const char* mbytes = (const char*)m;
    auto link_value = [&](int x, int y) { return *(const int32_t*)(mbytes + ((x << 8) | (y << 2))); };

    int t = clampi(tours[r * N + lane], 0, N - 1);
    int bt = t;
    const int my_round = lane >> 1, side = lane & 1;
    const bool in_play = my_round < LOGN;
    const int my_bit = 1 << (in_play ? my_round : 0);
    int k1 = -1, k2 = -1, k3 = -1;                      // this lane's round: its three largest links, value << 10 | lower rank

    // the wave recomputes round kk from the order; the two lanes of that round take the result
    auto recompute_round = [&](int kk) {
        const int bit = 1 << kk, i = lane & 31;         // link index (both half-waves compute the same 32 links)
        const int j = ((i >> kk) << (kk + 1)) | (i & (bit - 1));
        const int a = __builtin_amdgcn_ds_bpermute(j << 2, t), b = __builtin_amdgcn_ds_bpermute((j | bit) << 2, t);
        const int key = (link_value(a, b) << 5) | i;
        int found[3];
        int taken0 = -2, taken1 = -2;
#pragma unroll
        for (int pass = 0; pass < 3; ++pass) {
            const int best = wave_max((i == taken0 || i == taken1) ? -1 : key);
            const int bi = best & 31;
            found[pass] = ((best >> 5) << 10) | ((bi >> kk) << (kk + 1)) | (bi & (bit - 1));
            if (pass == 0) taken0 = bi;
            else taken1 = bi;
        }
        if (my_round == kk) {
            k1 = found[0];
            k2 = found[1];
            k3 = found[2];
        }
    };
    for (int kk = 0; kk < LOGN; ++kk) recompute_round(kk);
    int cur = wave_sum((in_play && side == 0) ? (k1 >> 10) : 0);
    int best = cur;
    int acc = 0;
    const uint64_t chain_hi = (uint64_t)(uint32_t)r << 32;

    int draw_pq = 0;                                    // ranks p | q << 8 of step (batch start + lane)
    int draw_most = 0;                                  // the largest cost increase it accepts
    for (long long s = 0; s < steps; ++s) {
        const int slot = (int)(s & 63);
        if (slot == 0) {
            const uint64_t w = splitmix64_at(seed, (chain_hi | (uint32_t)(kDrawBase + (uint32_t)s + (uint32_t)lane)) + 1u);
            const int p = (int)(((uint32_t)(w >> 43) * (uint32_t)N) >> 21);
            const int d = 1 + (int)((((uint32_t)(w >> 22) & 0x1FFFFFu) * (uint32_t)(N - 1)) >> 21);
            draw_pq = p | (((p + d) & (N - 1)) << 8);
            const int u = (int)((uint32_t)w & 0x3FFFFFu) + 1;
            draw_most = largest_accepted_increase(s + lane, steps, t_start, t_end, u);
        }
        const int pq = __builtin_amdgcn_readlane(draw_pq, slot);
        const int p = pq & 255, q = pq >> 8;
        const int node_p = __builtin_amdgcn_readlane(t, p), node_q = __builtin_amdgcn_readlane(t, q);
        // this lane's link: rank `mine` (p or q) receives the node of the other rank; its partner keeps its node
        const int mine = side ? q : p;
        const int x = side ? node_p : node_q;
        const int y = __builtin_amdgcn_ds_bpermute((mine ^ my_bit) << 2, t);
        const int link = in_play ? link_value(x, y) : 0;
        const int link_other = __builtin_amdgcn_update_dpp(link, link, 0xB1, 0xf, 0xf, true);          // the other side
        const int link_p = side ? link_other : link, link_q = side ? link : link_other;
        const int lp = p & ~my_bit, lq = q & ~my_bit;
        const bool same_link = lp == lq;               // q = p xor bit: the link keeps both nodes and its value
        const int j1 = k1 & 1023, j2 = k2 & 1023;
        const bool f1 = j1 != lp && j1 != lq, f2 = j2 != lp && j2 != lq;
        const int others = (f1 ? k1 : (f2 ? k2 : k3)) >> 10;
        const int stage = same_link ? (k1 >> 10) : max(others, max(link_p, link_q));
        const int total = wave_sum((in_play && side == 0) ? stage : 0);
        const int delta = total - cur;
        if (delta > __builtin_amdgcn_readlane(draw_most, slot)) continue;     // rejected (wave-uniform)
        t = lane == p ? node_q : (lane == q ? node_p : t);
        cur += delta;
        ++acc;
        // the round's three largest links after the exchange
        bool stale = false;
        if (in_play && !same_link) {
            const int f3 = (k3 & 1023) != lp && (k3 & 1023) != lq;
            int c0 = f1 ? k1 : -1, c1 = f2 ? k2 : -1, c2 = (f3 && k3 >= 0) ? k3 : -1;
            if (k1 < 0) c0 = -1;
            if (k2 < 0) c1 = -1;
            int c3 = (link_p << 10) | lp, c4 = (link_q << 10) | lq;
            const int bound = k3 >> 10;                // every link outside the candidates is at most this
            const int n1 = max(max(c0, c1), max(max(c2, c3), c4));
            c0 = c0 == n1 ? -1 : c0; c1 = c1 == n1 ? -1 : c1; c2 = c2 == n1 ? -1 : c2;
            c3 = c3 == n1 ? -1 : c3; c4 = c4 == n1 ? -1 : c4;
            const int n2 = max(max(c0, c1), max(max(c2, c3), c4));
            c0 = c0 == n2 ? -1 : c0; c1 = c1 == n2 ? -1 : c1; c2 = c2 == n2 ? -1 : c2;
            c3 = c3 == n2 ? -1 : c3; c4 = c4 == n2 ? -1 : c4;
            const int n3 = max(max(c0, c1), max(max(c2, c3), c4));
            stale = (n3 >> 10) < bound;
            k1 = n1; k2 = n2; k3 = n3;
        }
        unsigned long long redo = __ballot(stale);
        while (redo) {
            const int kk = (__ffsll((long long)redo) - 1) >> 1;
            recompute_round(kk);
            redo &= ~(0x3ull << (2 * kk));
        }
        if (cur < best) {
            best = cur;
            bt = t;
        }
    }
    tours[r * N + lane] = bt;
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

// N = 64: the chain of sa_ring_kernel with the order in one VGPR (lane = rank).  The four ranks a proposal needs are
// lane permutes, the committed proposal is read by a scalar lane index, the reversal is one lane permute, the best
// order a register copy: no order in LDS, so no write-read synchronisation within a round.  Draws as in
// sa_ring_kernel (a ring of 128 steps in LDS, 64 drawn at a time).
__global__ __launch_bounds__(256) void sa_ring_n64_kernel(const int32_t* __restrict__ c, int chains, long long steps,
                                                          int t_start, int t_end, uint64_t seed,
                                                          int32_t* __restrict__ tours, int64_t* __restrict__ costs,
                                                          int32_t* __restrict__ accepted) {
    constexpr int N = 64;
    __shared__ int32_t m[N * N];
    __shared__ __attribute__((aligned(16))) int32_t draws_all[4][2 * kDrawRing];
    const int lane = lane_id(), wv = threadIdx.x >> 6;
    for (int e = threadIdx.x; e < N * N; e += 256) m[e] = clampi(c[e], 0, kCostMax);
    __syncthreads();
    const int64_t r = (int64_t)blockIdx.x * 4 + wv;
    if (r >= chains) return;
    int32_t* draws = draws_all[wv];
    const char* mbytes = (const char*)m;
    auto M = [&](int x, int y) { return *(const int32_t*)(mbytes + ((x << 8) | (y << 2))); };
    auto node_at = [&](int rank, int order) { return __builtin_amdgcn_ds_bpermute(rank << 2, order); };

    int t = clampi(tours[r * N + lane], 0, N - 1);
    int bt = t;
    long long cur = wave_sum64((long long)M(t, __builtin_amdgcn_update_dpp(t, t, 0x13C, 0xf, 0xf, true)));
    long long best = cur;
    int acc = 0;
    const uint64_t chain_hi = (uint64_t)(uint32_t)r << 32;
    auto draw_block = [&](long long first) {
        const long long step = first + lane;
        const uint64_t w = splitmix64_at(seed, (chain_hi | (uint32_t)(kDrawBase + (uint32_t)step)) + 1u);
        const int a = (int)(((uint32_t)(w >> 43) * (uint32_t)N) >> 21);
        const int d = 2 + (int)((((uint32_t)(w >> 22) & 0x1FFFFFu) * (uint32_t)(N - 3)) >> 21);
        const int b = (a + d) & (N - 1);
        const int u = (int)((uint32_t)w & 0x3FFFFFu) + 1;
        const int slot = (int)step & (kDrawRing - 1);
        *(int2*)(draws + 2 * slot) = make_int2(a | (b << 16), largest_accepted_increase(step, steps, t_start, t_end, u));
    };
    draw_block(0);
    draw_block(kWave);
    long long drawn = 2 * kWave;              // steps [drawn - 128, drawn) are in the ring
    wave_lds_sync();
    long long s = 0;
    while (s < steps) {
        if (s + kWave > drawn) {              // the round reaches past the ring: the older half makes room
            draw_block(drawn);
            drawn += kWave;
            wave_lds_sync();
        }
        const long long step = s + lane;
        const bool active = step < steps;
        const int2 drawn_step = *(const int2*)(draws + 2 * ((int)step & (kDrawRing - 1)));
        const int a = drawn_step.x & 0xffff, b = drawn_step.x >> 16;
        const int ap = (a + N - 1) & (N - 1), bp = (b + N - 1) & (N - 1);
        const int ta = node_at(a, t), tap = node_at(ap, t), tb = node_at(b, t), tbp = node_at(bp, t);
        const int delta = M(tap, tbp) + M(ta, tb) - M(ta, tap) - M(tb, tbp);
        const bool accept = active && delta <= drawn_step.y;
        const unsigned long long mask = __ballot(accept);
        if (mask == 0ull) {
            s += kWave;
            continue;
        }
        const int k = __ffsll((long long)mask) - 1;
        const int abk = __builtin_amdgcn_readlane(drawn_step.x, k), dk = __builtin_amdgcn_readlane(delta, k);
        const int ak = abk & 0xffff, bk = abk >> 16;
        const int lo = min(ak, bk), hi = max(ak, bk);
        const int i = lo ? lo : hi, j = lo ? hi - 1 : N - 1;
        t = node_at((lane >= i && lane <= j) ? i + j - lane : lane, t);      // ranks i .. j reversed
        cur += dk;
        ++acc;
        if (cur < best) {
            best = cur;
            bt = t;
        }
        s += k + 1;
    }
    tours[r * N + lane] = bt;
    if (lane == 0) {
        costs[r] = best;
        accepted[r] = acc;
    }
}

}  // namespace

hipError_t launch_sa_ring(const int32_t* c, int N, int chains, long long steps, int t_start, int t_end, uint64_t seed,
                          bool generate, int32_t* tours, int64_t* costs, int32_t* accepted, hipStream_t s) {
    if (generate) {
        hipError_t e = launch_init_tours(N, 0, chains, seed, tours, s);
        if (e != hipSuccess) return e;
    }
    const int grid = (chains + 3) / 4;
    if (N == 64) {
        hipLaunchKernelGGL(sa_ring_n64_kernel, dim3(grid), dim3(256), 0, s, c, chains, steps, t_start, t_end, seed, tours,
                           costs, accepted);
    } else if (N <= 128) {
        const size_t lds = sizeof(int32_t) * ((size_t)8 * kDrawRing + (size_t)8 * N + (size_t)N * N);
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute((const void*)sa_ring_kernel<1>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL((sa_ring_kernel<1>), dim3(grid), dim3(256), lds, s, c, N, chains, steps, t_start, t_end,
                           seed, tours, costs, accepted);
    } else if (N <= 256) {
        const size_t lds = sizeof(int32_t) * ((size_t)8 * kDrawRing + (size_t)8 * N) + sizeof(uint16_t) * (size_t)N * N;
        hipError_t e = hipFuncSetAttribute((const void*)sa_ring_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((sa_ring_kernel<2>), dim3(grid), dim3(256), lds, s, c, N, chains, steps, t_start, t_end, seed,
                           tours, costs, accepted);
    } else {
        const size_t lds = sizeof(int32_t) * ((size_t)8 * kDrawRing + (size_t)8 * N);
        hipLaunchKernelGGL((sa_ring_kernel<0>), dim3(grid), dim3(256), lds, s, c, N, chains, steps, t_start, t_end,
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
        case 64:
            hipLaunchKernelGGL(sa_rd_n64_kernel, dim3((chains + 3) / 4), dim3(256), 0, s, c, chains, steps, t_start,
                               t_end, seed, tours, costs, accepted);
            return hipGetLastError();
        case 128: return sa_rd_launch<7>(c, chains, steps, t_start, t_end, seed, tours, costs, accepted, s);
        case 256: return sa_rd_launch<8>(c, chains, steps, t_start, t_end, seed, tours, costs, accepted, s);
        case 512: return sa_rd_launch<9>(c, chains, steps, t_start, t_end, seed, tours, costs, accepted, s);
        default: return sa_rd_launch<10>(c, chains, steps, t_start, t_end, seed, tours, costs, accepted, s);
    }
}

}  // namespace cc
