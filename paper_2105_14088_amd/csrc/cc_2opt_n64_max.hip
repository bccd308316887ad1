// 2-opt descent for N = 64 under the bottleneck (max-hop) objective, directed: one wavefront per
// restart, one ring rank per lane, the cost matrix staged once per workgroup in LDS.  Also serves the
// undirected max objective (on a symmetric matrix both walking directions of a move cost the same and
// the lower id, orientation 0, wins, which is exactly the undirected trajectory).
//
// Cyclic-diagonal sweep as in cc_2opt_n64.hip.  Exchanging ring edges a and b = a + d (edge p joins
// ranks p-1 and p) cuts the ring into S1 = ranks a..b-1 and S2 = ranks b..a-1 and rejoins them with one
// of the pieces reversed.  As a directed ring the result can be walked two ways:
//   A: S2 as it is, S1 backwards:  new hops c[t[b-1]][t[a-1]], c[t[b]][t[a]];  S2's inner hops f, S1's b
//   B: the opposite direction:     new hops c[t[a-1]][t[b-1]], c[t[a]][t[b]];  S2's inner hops b, S1's f
// (f[p] = c[t[p]][t[p-1]] is hop p as walked now, b[p] = c[t[p-1]][t[p]] the same edge the other way).
// With G(p,q) = c[t[p]][t[q]] and GT(p,q) = c[t[q]][t[p]], lane a gathers G(a,b) and GT(a,b) and takes
// G(a-1,b-1), GT(a-1,b-1) from lane a-1 by a DPP rotate; value = max of the two new hops and of the
// largest inner hop of each piece:
//   S1's inner edges a+1..b-1 grow by one edge per diagonal: a running max, fed by the rotating hop words;
//   S2's inner edges b+1..a-1 are a cyclic window of 31..61 edges: max of two windows of 32 (16 at d = 32)
//   from a doubling table M_k[p] = max f[p .. p+2^k-1] built once per sweep with lane permutes.
// In move terms (cc.h): if a < b (or b = 0) the move is (i, j) = (a, b-1) and A / B are orientations 0 / 1;
// otherwise it is (b, a-1) (or (b, 63) when a = 0) and A / B are orientations 1 / 0.  Per lane two running
// minima are kept, over key = value << 6 | rank(b), rank(b) = (b-1) mod 64, one for A and one for B; after
// the sweep both are turned into (value, move id) and min-reduced lexicographically over the wave.
//
// Matrices with entries below 2^16 take a packed form of the same sweep: the LDS matrix holds both directions of a
// pair in one word, c[x][y] | c[y][x] << 16, so one gather delivers G and GT, and every maximum above is taken on
// both halves at once (v_pk_max_u16): hop words, doubling tables, the running maximum of S1 and the two values of a
// move, A in the upper and B in the lower half.  The tables of S2 are built from the hop word with its halves
// swapped, which is the pairing the two values need (A: S2's f with S1's b; B: S2's b with S1's f).
#include "cc_device.h"
#include "cc_internal.h"
#include "cc_wave64.h"

namespace cc {
using namespace ccd;

namespace {

using namespace w64;

constexpr int kCostMax = (1 << 21) - 1;
constexpr int kNone = 0x7fffffff;

// The sweep on a plain int32 matrix (entries up to 2^21 - 1).
__device__ __forceinline__ void descend_max_wide(const int32_t* m, int lane, bool with_flip, int& t, int& cur_out,
                                                 int& applied_out) {
    const char* mbytes = (const char*)m;
    const int rank_a = (lane + kN - 1) & (kN - 1);
    // byte indices for lane permutes "take the value of lane p + k"
    const int from2 = ((lane + 2) & 63) << 2, from4 = ((lane + 4) & 63) << 2, from8 = ((lane + 8) & 63) << 2;
    const int from16 = ((lane + 16) & 63) << 2, from32 = ((lane + 32) & 63) << 2;
    const int from33 = ((lane + 33) & 63) << 2, from48 = ((lane + 48) & 63) << 2;
    auto take = [](int index, int value) { return __builtin_amdgcn_ds_bpermute(index, value); };

    int cur = 0, applied = 0;
    bool first = true;
    for (;;) {
        const int tprev = from_prev_lane(t);
        const int rowofs = t << 8, col = t << 2;
        const int f = *(const int32_t*)(mbytes + (rowofs | (tprev << 2)));
        const int bw = *(const int32_t*)(mbytes + ((tprev << 8) | col));
        if (first) {
            cur = wave_max(f);
            first = false;
        }
        // doubling tables: m5?[p] = max over hops p .. p+31, m4?[p] = max over hops p .. p+15
        int m4f, m5f, m4b, m5b;
        {
            int x = max(f, from_next_lane(f)), y = max(bw, from_next_lane(bw));
            x = max(x, take(from2, x));
            y = max(y, take(from2, y));
            x = max(x, take(from4, x));
            y = max(y, take(from4, y));
            m4f = max(x, take(from8, x));
            m4b = max(y, take(from8, y));
            m5f = max(m4f, take(from16, m4f));
            m5b = max(m4b, take(from16, m4b));
        }
        const int far_f = take(from32, m5f), far_b = take(from32, m5b);              // hops a+32 .. a+63
        const int far32_f = max(take(from33, m4f), take(from48, m4f));               // hops a+33 .. a+63
        const int far32_b = max(take(from33, m4b), take(from48, m4b));
        // words that travel round the wave, here in their state for partner a+1
        int w = from_next_lane((rank_a << 26) | (t << 8) | (t << 2));
        int fb = from_next_lane(f), bwb = from_next_lane(bw);
        int r5f = from_next_lane(from_next_lane(m5f)), r5b = from_next_lane(from_next_lane(m5b));
        int s1f = 0, s1b = 0, bestA = kNone, bestB = kNone;
#pragma unroll
        for (int d = 2; d <= kN / 2; ++d) {
            s1f = max(s1f, fb);          // edge b-1 (the previous diagonal's partner) joins S1's inner edges
            s1b = max(s1b, bwb);
            w = from_next_lane(w);
            if (d < kN / 2) {
                fb = from_next_lane(fb);
                bwb = from_next_lane(bwb);
                r5f = from_next_lane(r5f);   // max over hops b+1 .. b+32
                r5b = from_next_lane(r5b);
            }
            const int G = *(const int32_t*)(mbytes + ((w & 0xfc) | rowofs));        // c[t[a]][t[b]]
            const int GT = *(const int32_t*)(mbytes + ((w & 0x3f00) | col));        // c[t[b]][t[a]]
            const int EG = from_prev_lane(G), EGT = from_prev_lane(GT);
            const int s2f = d < kN / 2 ? max(r5f, far_f) : far32_f;
            const int s2b = d < kN / 2 ? max(r5b, far_b) : far32_b;
            const int valA = max(max(EGT, GT), max(s2f, s1b));
            const int valB = max(max(EG, G), max(s2b, s1f));
            bestA = min(bestA, (int)__builtin_amdgcn_alignbit((unsigned)valA, (unsigned)w, 26));
            bestB = min(bestB, (int)__builtin_amdgcn_alignbit((unsigned)valB, (unsigned)w, 26));
        }
        // (value, move id) of the lane's two candidates; keep the lexicographically smaller
        int val = kNone, id = kNone;
#pragma unroll
        for (int which = 0; which < 2; ++which) {
            const int key = which ? bestB : bestA;
            const int kv = key >> 6, rk = key & 63;
            const int b = (rk + 1) & 63;
            const int lo = min(lane, b), hi = max(lane, b);
            const int ij = lo ? lo * kN + hi - 1 : hi * kN + kN - 1;
            const int flip = rk < rank_a ? 1 : 0;       // the reversed piece is S2, not S1
            const int kid = ij * 2 + (which ^ flip);
            if (kv < val || (kv == val && kid < id)) { val = kv; id = kid; }
        }
        if (with_flip && lane == 0) {                   // the orientation flip: every hop walked the other way
            const int vf = max(m5b, far_b), idf = (kN + kN - 1) * 2;
            if (vf < val || (vf == val && idf < id)) { val = vf; id = idf; }
        }
        const int vwin = wave_min_uniform(val);
        if (vwin >= cur) break;
        const int idwin = wave_min_uniform(val == vwin ? id : kNone);
        const int o = idwin & 1, ij = idwin >> 1, mi = ij >> 6, mj = ij & 63;
        const int p0 = o ? (lane ? kN - lane : 0) : lane;
        const int src = (p0 >= mi && p0 <= mj) ? mi + mj - p0 : p0;
        t = __shfl(t, src, kWave);
        cur = vwin;
        ++applied;
    }
    cur_out = cur;
    applied_out = applied;
}

typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pk_max(unsigned a, unsigned b) {
    return __builtin_bit_cast(unsigned, __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, a),
                                                                  __builtin_bit_cast(ushort2_t, b)));
}

// The sweep on the packed matrix m2[x][y] = c[x][y] | c[y][x] << 16 (entries below 2^16).
__device__ __forceinline__ void descend_max_packed(const int32_t* m2, int lane, bool with_flip, int& t, int& cur_out,
                                                   int& applied_out) {
    const char* mbytes = (const char*)m2;
    const int rank_a = (lane + kN - 1) & (kN - 1);
    const int from2 = ((lane + 2) & 63) << 2, from4 = ((lane + 4) & 63) << 2, from8 = ((lane + 8) & 63) << 2;
    const int from16 = ((lane + 16) & 63) << 2, from32 = ((lane + 32) & 63) << 2;
    const int from33 = ((lane + 33) & 63) << 2, from48 = ((lane + 48) & 63) << 2;
    auto take = [](int index, unsigned value) { return (unsigned)__builtin_amdgcn_ds_bpermute(index, (int)value); };
    auto rol = [](unsigned v) { return (unsigned)from_next_lane((int)v); };
    constexpr unsigned kNoKey = 0xffffffffu;

    int cur = 0, applied = 0;
    bool first = true;
    for (;;) {
        const int tprev = from_prev_lane(t);
        const int rowofs = t << 8;
        const unsigned fb = *(const uint32_t*)(mbytes + (rowofs | (tprev << 2)));     // f[a] | b[a] << 16
        if (first) {
            cur = wave_max((int)(fb & 0xffffu));
            first = false;
        }
        // doubling tables over the hop words with their halves swapped (b | f << 16):
        // m5[p] = max over hops p .. p+31, m4[p] = over hops p .. p+15
        const unsigned bf = __builtin_amdgcn_alignbit(fb, fb, 16);
        unsigned m4, m5;
        {
            unsigned x = pk_max(bf, rol(bf));
            x = pk_max(x, take(from2, x));
            x = pk_max(x, take(from4, x));
            m4 = pk_max(x, take(from8, x));
            m5 = pk_max(m4, take(from16, m4));
        }
        const unsigned far = take(from32, m5);                                       // hops a+32 .. a+63
        const unsigned far32 = pk_max(take(from33, m4), take(from48, m4));           // hops a+33 .. a+63
        // words that travel round the wave, here in their state for partner a+1
        unsigned w = rol((unsigned)((rank_a << 10) | (t << 2)));
        unsigned fbr = rol(fb);
        unsigned r5 = rol(rol(m5));
        // S2's inner hops b+1 .. a-1 are hops b+1 .. b+32 together with hops a+33 .. a+63 for every d < 32 (the first
        // window ends at a+d+32 >= a+34), and hops a+33 .. a+63 alone at d = 32.  A move's value is the maximum over both
        // pieces anyway, so the fixed window starts the running maximum of S1 and costs nothing per diagonal.
        unsigned s1 = far32, bestA = kNoKey, bestB = kNoKey;
#pragma unroll
        for (int d = 2; d <= kN / 2; ++d) {
            s1 = pk_max(s1, fbr);        // edge b-1 (the previous diagonal's partner) joins S1's inner edges
            w = rol(w);
            if (d < kN / 2) {
                fbr = rol(fbr);
                r5 = rol(r5);            // max over hops b+1 .. b+32, halves swapped
            }
            int off;                     // (w & 0xfc) | rowofs in one instruction
            asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(off) : "v"(w), "s"(0xfc), "v"(rowofs));
            const unsigned P = *(const uint32_t*)(mbytes + off);                                 // G | GT << 16
            const unsigned EP = (unsigned)from_prev_lane((int)P);
            // lower half: max(G, EG, S2's b, S1's f) = value B; upper half: max(GT, EGT, S2's f, S1's b) = value A
            const unsigned PE = pk_max(P, EP);
            const unsigned val = d < kN / 2 ? pk_max(PE, pk_max(s1, r5)) : pk_max(PE, s1);
            bestA = min(bestA, (val & 0xffff0000u) | w);
            bestB = min(bestB, (val << 16) | w);
        }
        // (value, move id) of the lane's two candidates as one key, value << 13 | id (values are below 2^16, ids below
        // 2^13), branch-free.  With r = rank(b): the move is (lane, r) when r >= rank(lane) (b lies after the lane, or
        // b = 0) and A / B are orientations 0 / 1; otherwise it is (r + 1, rank(lane)) and A / B are 1 / 0.
        auto candidate = [&](unsigned key, int which) {
            const int rk = (int)(key >> 10) & 63;
            const bool wrapped = rk < rank_a;
            const int id = wrapped ? (rk << 7) + ((kN + rank_a) * 2 + (which ^ 1)) : (rk << 1) + (lane * kN * 2 + which);
            return (int)((key >> 3) & ~0x1fffu) | id;
        };
        int key = min(candidate(bestA, 0), candidate(bestB, 1));
        if (with_flip) {                                // the orientation flip: every hop walked the other way
            const int vf = (int)(pk_max(m5, far) & 0xffffu), idf = (kN + kN - 1) * 2;
            const int kf = (vf << 13) | idf;
            key = lane == 0 ? min(key, kf) : key;
        }
        const int win = wave_min_uniform(key);
        const int vwin = win >> 13;
        if (vwin >= cur) break;
        const int idwin = win & 0x1fff;
        const int o = idwin & 1, ij = idwin >> 1, mi = ij >> 6, mj = ij & 63;
        const int p0 = o ? (lane ? kN - lane : 0) : lane;
        const int src = (p0 >= mi && p0 <= mj) ? mi + mj - p0 : p0;
        t = __shfl(t, src, kWave);
        cur = vwin;
        ++applied;
    }
    cur_out = cur;
    applied_out = applied;
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 2)))
void twoopt_max_n64_kernel(const int32_t* __restrict__ c, int restarts, uint64_t seed, int generate, int with_flip,
                           int32_t* __restrict__ tours, int64_t* __restrict__ costs,
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
    // entries are clamped to the contract range; the largest decides between the packed and the plain sweep
    int mx = 0;
#pragma unroll
    for (int k = 0; k < kN * kN / 256; ++k) {
        v[k] = clampi(v[k], 0, kCostMax);
        mx = max(mx, v[k]);
    }
    mx = wave_max(mx);
    if (lane == 0) wave_max_entry[wv] = mx;
#pragma unroll
    for (int k = 0; k < kN * kN / 256; ++k) m[tid + 256 * k] = v[k];
    __syncthreads();
    mx = max(max(wave_max_entry[0], wave_max_entry[1]), max(wave_max_entry[2], wave_max_entry[3]));
    const bool packed = mx < (1 << 16);
    if (packed) {
        // both directions of a pair into one word, in place
        for_each_pair_64(tid, [&](int lo, int hi) {
            const int x = m[lo * kN + hi], y = m[hi * kN + lo];
            m[lo * kN + hi] = x | (y << 16);
            m[hi * kN + lo] = y | (x << 16);
        });
        __syncthreads();
    }
    if (r >= restarts) return;

    int cur, applied;
    if (packed) descend_max_packed(m, lane, with_flip != 0, t, cur, applied);
    else descend_max_wide(m, lane, with_flip != 0, t, cur, applied);
    tours[r * kN + lane] = t;
    if (lane == 0) {
        costs[r] = (int64_t)cur;
        moves[r] = applied;
    }
}

}  // namespace

hipError_t launch_2opt_max_n64(const int32_t* c, int restarts, uint64_t seed, bool generate, bool with_flip,
                               int32_t* tours, int64_t* costs, int32_t* moves, hipStream_t s) {
    const int grid = (restarts + 3) / 4;
    hipLaunchKernelGGL(twoopt_max_n64_kernel, dim3(grid), dim3(256), 0, s, c, restarts, seed, generate ? 1 : 0,
                       with_flip ? 1 : 0, tours, costs, moves);
    return hipGetLastError();
}

}  // namespace cc
