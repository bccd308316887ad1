// 2-opt descent for N = 64 under the directed ring-sum objective (matrices with c[a][b] != c[b][a]; entries below
// 2^16): one wavefront per restart, one ring rank per lane, the cost matrix staged once per workgroup in LDS.  Move
// set, ids, values and tie-breaks as stated in cc.h (cc_2opt_search); larger entries and other sizes take the
// general kernel.
//
// Cyclic-diagonal sweep with the geometry of the max-hop kernel (cc_2opt_n64_max.hip).  Exchanging ring edges a and
// b = a + d cuts the ring into S1 = ranks a..b-1 and S2 = ranks b..a-1; the result can be walked two ways:
//   A: S2 as it is, S1 backwards:  new hops GT(a-1,b-1) + GT(a,b);  S2's inner hops cost f, S1's inner hops b
//   B: the opposite direction:     new hops G(a-1,b-1) + G(a,b);    S2's inner hops cost b, S1's inner hops f
// with G(p,q) = c[t[p]][t[q]], GT(p,q) = c[t[q]][t[p]], f[p] = c[t[p]][t[p-1]] (hop p as walked now) and
// b[p] = c[t[p-1]][t[p]] (the same edge the other way).  With F = sum of f (the current cost), Bt = sum of b and
// q = sum over S1's inner hops a+1..b-1 of (b - f), which grows by one hop per diagonal,
//   value A - F = GT(a-1,b-1) + GT(a,b) - f[a] - f[b] + q
//   value B - F = G(a-1,b-1) + G(a,b) - b[a] - b[b] - q + (Bt - F).
// Lane a gathers G(a,b) and GT(a,b) and takes the (a-1, b-1) entries from lane a-1 by a DPP rotate; f[b], b[b] and
// the partner's rank and node travel round the wave one lane per diagonal.  Per lane two running minima over
// key = (partial delta) << 6 | rank(b), one per direction; the lane's own terms are added after the sweep, both are
// turned into (delta, move id) exactly as in the max-hop kernel, and the wave takes the lexicographic minimum.
#include "cc_device.h"
#include "cc_internal.h"
#include "cc_wave64.h"

namespace cc {
using namespace ccd;

namespace {

using namespace w64;
constexpr int kNone = 0x7fffffff;

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 2)))
void twoopt_dsum_n64_kernel(const int32_t* __restrict__ c, int restarts, uint64_t seed, int generate, int with_flip,
                            int32_t* __restrict__ tours, int64_t* __restrict__ costs, int32_t* __restrict__ moves,
                            const int32_t* __restrict__ flags) {
    if (flags[0] >= (1 << 16)) return;             // keys would not fit: the general kernel does the work
    __shared__ __attribute__((aligned(256))) int32_t m[kN * kN];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    int v[kN * kN / 256];
#pragma unroll
    for (int k = 0; k < kN * kN / 256; ++k) v[k] = c[tid + 256 * k];
    const int64_t r = (int64_t)blockIdx.x * 4 + wv;
    int t = 0;
    if (r < restarts)
        t = generate ? init_tour_in_wave(seed, (uint32_t)r, lane) : clampi(tours[r * kN + lane], 0, kN - 1);
#pragma unroll
    for (int k = 0; k < kN * kN / 256; ++k) m[tid + 256 * k] = clampi(v[k], 0, (1 << 16) - 1);
    __syncthreads();
    if (r >= restarts) return;

    const char* mbytes = (const char*)m;
    const int rank_a = (lane + kN - 1) & (kN - 1);
    long long cur = 0;
    int applied = 0;
    bool first = true;
    for (;;) {
        const int tprev = from_prev_lane(t);
        const int rowofs = t << 8, col = t << 2;
        const int f = *(const int32_t*)(mbytes + (rowofs | (tprev << 2)));
        const int bw = *(const int32_t*)(mbytes + ((tprev << 8) | col));
        const int turn = wave_sum(bw - f);                 // Bt - F: what walking the whole ring the other way costs
        if (first) {
            cur = wave_sum(f);
            first = false;
        }
        // words that travel round the wave, here in their state for partner a+1
        int w = from_next_lane((rank_a << 26) | (t << 8) | (t << 2));
        int fb = from_next_lane(f), bwb = from_next_lane(bw);
        int q = 0, bestA = kNone, bestB = kNone;
#pragma unroll
        for (int d = 2; d <= kN / 2; ++d) {
            q += bwb - fb;               // edge b-1 (the previous diagonal's partner) joins S1's inner hops
            w = from_next_lane(w);
            fb = from_next_lane(fb);
            bwb = from_next_lane(bwb);
            // keeps each rotate an instruction of its own: folded into the subtraction below it would become
            // v_subrev_u32_dpp, which on this chip rotates the other operand
            asm("" : "+v"(fb), "+v"(bwb));
            const int G = *(const int32_t*)(mbytes + ((w & 0xfc) | rowofs));        // c[t[a]][t[b]]
            const int GT = *(const int32_t*)(mbytes + ((w & 0x3f00) | col));        // c[t[b]][t[a]]
            const int EG = from_prev_lane(G), EGT = from_prev_lane(GT);
            const int dA = add3(EGT, GT, q - fb);
            const int dB = add3(EG, G, -q - bwb);
            bestA = min(bestA, (int)__builtin_amdgcn_alignbit((unsigned)dA, (unsigned)w, 26));
            bestB = min(bestB, (int)__builtin_amdgcn_alignbit((unsigned)dB, (unsigned)w, 26));
        }
        // (delta, move id) of the lane's two candidates; keep the lexicographically smaller
        int val = kNone, id = kNone;
#pragma unroll
        for (int which = 0; which < 2; ++which) {
            const int key = which ? bestB : bestA;
            const int kv = (key >> 6) + (which ? turn - bw : -f), rk = key & 63;
            const int b = (rk + 1) & 63;
            const int lo = min(lane, b), hi = max(lane, b);
            const int ij = lo ? lo * kN + hi - 1 : hi * kN + kN - 1;
            const int flip = rk < rank_a ? 1 : 0;       // the reversed piece is S2, not S1
            const int kid = ij * 2 + (which ^ flip);
            if (kv < val || (kv == val && kid < id)) { val = kv; id = kid; }
        }
        if (with_flip && lane == 0) {                   // the orientation flip: every hop walked the other way
            const int idf = (kN + kN - 1) * 2;
            if (turn < val || (turn == val && idf < id)) { val = turn; id = idf; }
        }
        const int dwin = wave_min_uniform(val);
        if (dwin >= 0) break;
        const int idwin = wave_min_uniform(val == dwin ? id : kNone);
        const int o = idwin & 1, ij = idwin >> 1, mi = ij >> 6, mj = ij & 63;
        const int p0 = o ? (lane ? kN - lane : 0) : lane;
        const int src = (p0 >= mi && p0 <= mj) ? mi + mj - p0 : p0;
        t = __shfl(t, src, kWave);
        cur += dwin;
        ++applied;
    }
    tours[r * kN + lane] = t;
    if (lane == 0) {
        costs[r] = cur;
        moves[r] = applied;
    }
}

}  // namespace

hipError_t launch_2opt_dsum_n64(const int32_t* c, int restarts, uint64_t seed, bool generate, bool with_flip,
                                int32_t* tours, int64_t* costs, int32_t* moves, const int32_t* flags, hipStream_t s) {
    const int grid = (restarts + 3) / 4;
    hipLaunchKernelGGL(twoopt_dsum_n64_kernel, dim3(grid), dim3(256), 0, s, c, restarts, seed, generate ? 1 : 0,
                       with_flip ? 1 : 0, tours, costs, moves, flags);
    return hipGetLastError();
}

}  // namespace cc
