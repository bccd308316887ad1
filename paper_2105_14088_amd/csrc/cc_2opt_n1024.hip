// 2-opt descent for N = 512 and N = 1024, ring-sum objective on a symmetric matrix: one workgroup of
// N/64 waves per restart (the text below gives the N = 1024 figures; N = 512 has half the slots, rows and
// waves).  The matrix (2 MiB as 16-bit entries) cannot live in LDS, so the sweep is organised by
// matrix ROW: every move needs G(a-1, b-1) + G(a, b) with G(p, q) = c[t[p]][t[q]], i.e. one entry of
// row t[a] and one of row t[a-1].  A wave owns 64 consecutive ranks a; for each it streams row t[a]
// (2 KiB, coalesced, L2-resident) straight into one of its four private LDS buffers
// (global_load_lds_dwordx4, three rows ahead, no staging registers) and gathers that row at the columns
// of the partners b = a + d.  Lanes own DIAGONALS: lane l, slot k scores d = 2 + 8l + k (d = 2 .. 513
// covers every pair of non-adjacent ring edges; 513 repeats 511), so
//   - the row-(a-1) term of a move is the same lane's gather of the previous row: no cross-lane traffic;
//   - the partner words of a lane are a window of 8 consecutive ranks that slides by one rank per row;
//     it is re-read from LDS (two aligned 16-byte loads per array) every 8 rows.
// Keys.  key = (G + G - f[a] - f[b]) << 11 | rank.  A slot sees the moves of one diagonal for all rows
// of the wave; their ids are ordered by the smaller rank of the pair: rank = 2a for a < b (the pair is
// the move (a, b-1), or (a, N-1) when b wraps to 0) and 2b+1 for b < a (the move (b, a-1)), which is
// min(2a, 2b+1).  The partner word carries 2b+1 (2047 for b = 0), the row contributes 2a (2047 for row
// 0, whose pairs (0, b) are the moves (b, N-1) and sort after everything else in their slot).
// After the sweep every slot's key is turned into (delta, move id); lanes, waves and then the
// workgroup take the lexicographic minimum, so the result is independent of the visiting order.
// Needs max(c) < 2^16 (16-bit copy of the matrix in the workspace); otherwise the general kernel runs.
#include "cc_device.h"
#include "cc_internal.h"

namespace cc {
using namespace ccd;

namespace {

constexpr int kPad = 8;                      // the partner arrays are indexed from -8
constexpr int kBufs = 4;                     // row buffers per wave: the current row and three in flight

template <int LOGN>
struct Shape {
    static constexpr int N = 1 << LOGN;
    static constexpr int kWaves = N / 64;
    static constexpr int kSlots = N / 128;                   // diagonals per lane: 8 (N = 1024) or 4 (N = 512)
    static constexpr int kRankBits = LOGN + 1;
    static constexpr int kRankMask = (1 << kRankBits) - 1;
    static constexpr int kWin = kPad + N + 64 * kSlots;      // entry x holds rank (x + 2) mod N, x in [-8, N + 64 kSlots)
    static constexpr int kRowBytes = N * 2;
    static constexpr int kRowLoads = kRowBytes / 1024;       // 16-byte loads per lane and row: 2 or 1
    static constexpr size_t t = 0;                                   // int32 [N]   tour
    static constexpr size_t f = t + sizeof(int32_t) * N;             // int32 [N]   hop into each rank
    static constexpr size_t tw = f + sizeof(int32_t) * N;            // int32 [kWin] column byte offset of the partner
    static constexpr size_t kw = tw + sizeof(int32_t) * kWin;        // int32 [kWin] -f[b] << kRankBits | 2b+1
    static constexpr size_t red = kw + sizeof(int32_t) * kWin;       // int32 [2 * kWaves + 2]
    static constexpr size_t rows = (red + sizeof(int32_t) * 64 + 255) & ~(size_t)255;   // uint16 [kWaves][kBufs][N]
    static constexpr size_t total = rows + (size_t)kWaves * kBufs * kRowBytes;
};

// waits until at most `rows_in_flight` of this wave's row transfers are outstanding
template <int ROW_LOADS>
__device__ __forceinline__ void wait_rows(int rows_in_flight) {
    if (ROW_LOADS == 2) {
        if (rows_in_flight == 3) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
        else if (rows_in_flight == 2) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else if (rows_in_flight == 1) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    } else {
        if (rows_in_flight == 3) asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
        else if (rows_in_flight == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
        else if (rows_in_flight == 1) asm volatile("s_waitcnt vmcnt(1)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
}

// 16-bit copy of the matrix (entries clamped, upper triangle mirrored); skipped when the maximum does not fit
__global__ __launch_bounds__(256) void matrix_to_u16_kernel(const int32_t* __restrict__ c, int n,
                                                            uint16_t* __restrict__ c16,
                                                            const int32_t* __restrict__ flags) {
    if (flags[0] >= (1 << 16)) return;
    for (int e = blockIdx.x * 256 + threadIdx.x; e < n * n / 2; e += gridDim.x * 256) {
        const int lo = clampi(c[upper_index(2 * e, n)], 0, 0xffff), hi = clampi(c[upper_index(2 * e + 1, n)], 0, 0xffff);
        ((uint32_t*)c16)[e] = (uint32_t)lo | ((uint32_t)hi << 16);
    }
}

template <int LOGN>
__global__ __launch_bounds__(1 << LOGN) void twoopt_sum_n1024_kernel(const uint16_t* __restrict__ c16, int restarts,
                                                                     int32_t* __restrict__ tours,
                                                                     int64_t* __restrict__ costs,
                                                                     int32_t* __restrict__ moves,
                                                                     const int32_t* __restrict__ flags) {
    using Layout = Shape<LOGN>;
    constexpr int N = Layout::N, kWaves = Layout::kWaves, kSlots = Layout::kSlots, kRankBits = Layout::kRankBits;
    constexpr int kRankMask = Layout::kRankMask, kRowBytes = Layout::kRowBytes, kRowLoads = Layout::kRowLoads;
    constexpr int kGroups = 64 / kSlots;         // a lane's window of kSlots partners is replaced every kSlots rows
    extern __shared__ __attribute__((aligned(256))) unsigned char smem[];
    if (flags[0] >= (1 << 16)) return;
    int32_t* T = (int32_t*)(smem + Layout::t);
    int32_t* F = (int32_t*)(smem + Layout::f);
    int32_t* TW = (int32_t*)(smem + Layout::tw) + kPad;
    int32_t* KW = (int32_t*)(smem + Layout::kw) + kPad;
    int32_t* red = (int32_t*)(smem + Layout::red);
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int64_t r = blockIdx.x;
    const int wbase = (int)(Layout::rows + (size_t)wv * kBufs * kRowBytes);   // byte offset of this wave's row buffer 0
    const unsigned lds_rows = (unsigned)__builtin_amdgcn_readfirstlane(
        (int)(size_t)(__attribute__((address_space(3))) unsigned char*)(smem + wbase));   // wave-uniform, in an SGPR
    const int lane16 = lane * 16;

    T[tid] = clampi(tours[r * N + tid], 0, N - 1);
    __syncthreads();

    long long cur = 0;
    int applied = 0;
    bool first = true;
    const int a0 = wv * 64;
    // Row `node` of the 16-bit matrix -> this wave's buffer `buf`, global memory to LDS without passing through
    // registers: lane l moves bytes [16l, 16l+16) and, for 2 KiB rows, [1024+16l, 1024+16l+16) of the row; M0 holds
    // the LDS address of the buffer and the instruction offset applies to both addresses.  Completion is tracked by
    // vmcnt.
    auto row_dma = [&](int node, int buf) {
        const void* rowptr = (const void*)(c16 + (size_t)node * N);
        const unsigned dst = lds_rows + (unsigned)buf * kRowBytes;
        if (kRowLoads == 2)
            asm volatile(
                "s_mov_b32 m0, %2\n\t"
                "s_nop 0\n\t"
                "global_load_lds_dwordx4 %0, %1\n\t"
                "global_load_lds_dwordx4 %0, %1 offset:1024"
                :: "v"(lane16), "s"(rowptr), "s"(dst) : "memory");
        else
            asm volatile(
                "s_mov_b32 m0, %2\n\t"
                "s_nop 0\n\t"
                "global_load_lds_dwordx4 %0, %1"
                :: "v"(lane16), "s"(rowptr), "s"(dst) : "memory");
    };
    for (;;) {
        // the wave's first rows (ranks a0-1, a0, a0+1, a0+2) are requested before anything else so that their L2
        // latency overlaps the hop gathers below; every LDS read of the previous sweep has long completed
        row_dma(__builtin_amdgcn_readfirstlane(T[(a0 + N - 1) & (N - 1)]), 3);
        row_dma(__builtin_amdgcn_readfirstlane(T[a0]), 0);
        row_dma(__builtin_amdgcn_readfirstlane(T[a0 + 1]), 1);
        row_dma(__builtin_amdgcn_readfirstlane(T[a0 + 2]), 2);
        // ---- hops and the partner arrays for the current tour
        {
            const int tp = T[tid], tq = T[(tid + N - 1) & (N - 1)];
            const int f = c16[tp * N + tq];
            F[tid] = f;
            const int kp = (int)(0u - ((unsigned)f << kRankBits)) + (tid ? 2 * tid + 1 : kRankMask);
            const int x = tid - 2;
            TW[x] = 2 * tp;
            KW[x] = kp;
            if (x + N < N + 64 * kSlots) {
                TW[x + N] = 2 * tp;
                KW[x + N] = kp;
            }
            if (first) {
                const int s = wave_sum(f);
                if (lane == 0) red[wv] = s;
                __syncthreads();
                long long tot = 0;
                for (int k = 0; k < kWaves; ++k) tot += red[k];
                cur = tot;
                first = false;
            }
        }
        __syncthreads();

        // ---- this wave's 64 rows
        const int row_node = T[a0 + lane];                              // lane q: node whose row is streamed for rank a0+q
        const int row_negf = -F[a0 + lane];
        const int row_rank = (a0 + lane) ? 2 * (a0 + lane) : kRankMask;
        const int gb = a0 + kSlots * lane;                              // window of row a0 starts at entry gb
        int cwt[kSlots], cwk[kSlots], nwt[kSlots], nwk[kSlots], dprev[kSlots], best[kSlots];
#pragma unroll
        for (int h = 0; h < kSlots; h += 4) {
            const int4 a = *(const int4*)(TW + gb + h), c4 = *(const int4*)(KW + gb + h);
            cwt[h] = a.x + wbase; cwt[h + 1] = a.y + wbase; cwt[h + 2] = a.z + wbase; cwt[h + 3] = a.w + wbase;
            cwk[h] = c4.x; cwk[h + 1] = c4.y; cwk[h + 2] = c4.z; cwk[h + 3] = c4.w;
        }
#pragma unroll
        for (int k = 0; k < kSlots; ++k) best[k] = 0x7fffffff;

        // row a0-1 only provides the "previous row" gathers of row a0; it sits in buffer 3
        {
            const int extra = TW[gb - 1] + wbase;
            wait_rows<kRowLoads>(3);                              // rows a0, a0+1, a0+2 may still be in flight
            dprev[0] = *(const uint16_t*)(smem + extra + 3 * kRowBytes);
#pragma unroll
            for (int k = 1; k < kSlots; ++k) dprev[k] = *(const uint16_t*)(smem + cwt[k - 1] + 3 * kRowBytes);
        }
#pragma unroll 1
        for (int g = 0; g < kGroups; ++g) {
            const int nb = gb + kSlots * (g + 1);
#pragma unroll
            for (int j = 0; j < kSlots; ++j) {
                const int q = kSlots * g + j;            // row a0 + q, buffer q & 3 = j & 3
                // the next window is fetched four entries at a time, each part just before its first use
                if ((j & 3) == 0) {
                    const int4 a = *(const int4*)(TW + nb + j), c4 = *(const int4*)(KW + nb + j);
                    nwt[j] = a.x + wbase; nwt[j + 1] = a.y + wbase; nwt[j + 2] = a.z + wbase; nwt[j + 3] = a.w + wbase;
                    nwk[j] = c4.x; nwk[j + 1] = c4.y; nwk[j + 2] = c4.z; nwk[j + 3] = c4.w;
                }
                // buffer (q+3) & 3 was last read by row q-1: its gathers have returned once lgkmcnt is 0
                const bool tail = (g == kGroups - 1) && (j >= kSlots - 3);   // rows 61..63: nothing left to request
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                if (!tail) row_dma(__builtin_amdgcn_readlane(row_node, q + 3), (j + 3) & 3);
                if (!tail) wait_rows<kRowLoads>(3);
                else wait_rows<kRowLoads>(kSlots - 1 - j);        // 2, 1, 0 rows still in flight
                const int negfa = __builtin_amdgcn_readlane(row_negf, q);
                const int rank2a = __builtin_amdgcn_readlane(row_rank, q);
#pragma unroll
                for (int k = 0; k < kSlots; ++k) {
                    const int idx = j + k;
                    const int twv = idx < kSlots ? cwt[idx] : nwt[idx - kSlots];
                    const int kwv = idx < kSlots ? cwk[idx] : nwk[idx - kSlots];
                    const int D = *(const uint16_t*)(smem + twv + (j & 3) * kRowBytes);
                    const int sum = dprev[k] + D + negfa;
                    const int keyfull = (int)(((unsigned)sum << kRankBits) + (unsigned)kwv);
                    const int keyalt = (keyfull & ~kRankMask) | rank2a;
                    best[k] = min(best[k], min(keyfull, keyalt));
                    dprev[k] = D;
                }
                __builtin_amdgcn_sched_barrier(0);   // keep one row's gathers in flight, not eight rows' (registers)
            }
#pragma unroll
            for (int k = 0; k < kSlots; ++k) {
                cwt[k] = nwt[k];
                cwk[k] = nwk[k];
            }
        }

        // ---- slot keys -> (delta, move id); minimum over slots, lanes, waves
        int bd = 0x7fffffff, bid = 0x7fffffff;
#pragma unroll
        for (int k = 0; k < kSlots; ++k) {
            const int d = 2 + kSlots * lane + k;
            const int delta = best[k] >> kRankBits, rank = best[k] & kRankMask;
            int id;
            if (!(rank & 1)) {
                const int a = rank >> 1;                       // pair (a, a+d): move (a, a+d-1)
                id = a * N + a + d - 1;
            } else {
                const int b = rank >> 1;
                if (b == d) id = d * N + N - 1;                // row 0: pair (0, d): move (d, N-1)
                else id = b * N + (b + N - d) - 1;             // pair (b+N-d, b): move (b, a-1)
            }
            if (delta < bd || (delta == bd && id < bid)) { bd = delta; bid = id; }
        }
        {
            int dmin = bd;
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) dmin = min(dmin, __shfl_xor(dmin, m, kWave));
            int imin = bd == dmin ? bid : 0x7fffffff;
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) imin = min(imin, __shfl_xor(imin, m, kWave));
            if (lane == 0) { red[2 * wv] = dmin; red[2 * wv + 1] = imin; }
        }
        __syncthreads();
        int gd = red[0], gid = red[1];
        for (int k = 1; k < kWaves; ++k) {
            const int d2 = red[2 * k], i2 = red[2 * k + 1];
            if (d2 < gd || (d2 == gd && i2 < gid)) { gd = d2; gid = i2; }
        }
        if (gd >= 0) break;
        // ---- reverse ranks mi..mj
        const int mi = gid >> LOGN, mj = gid & (N - 1);
        const int src = (tid >= mi && tid <= mj) ? mi + mj - tid : tid;
        const int val = T[src];
        __syncthreads();
        T[tid] = val;
        __syncthreads();
        cur += gd;
        ++applied;
    }
    tours[r * N + tid] = T[tid];
    if (tid == 0) {
        costs[r] = cur;
        moves[r] = applied;
    }
}

}  // namespace

template <int LOGN>
static hipError_t launch_rows(const int32_t* c, uint16_t* c16, int restarts, int32_t* tours, int64_t* costs,
                              int32_t* moves, const int32_t* flags, hipStream_t s) {
    using L = Shape<LOGN>;
    hipLaunchKernelGGL(matrix_to_u16_kernel, dim3(512), dim3(256), 0, s, c, L::N, c16, flags);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void*)twoopt_sum_n1024_kernel<LOGN>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)L::total);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(twoopt_sum_n1024_kernel<LOGN>, dim3(restarts), dim3(L::N), L::total, s, c16, restarts, tours, costs,
                       moves, flags);
    return hipGetLastError();
}

// N = 512 or 1024.  `tours` must hold the initial tours, flags[0] the matrix maximum, c16 room for N*N 16-bit entries.
hipError_t launch_2opt_sum_n1024(const int32_t* c, int N, uint16_t* c16, int restarts, int32_t* tours, int64_t* costs,
                                 int32_t* moves, const int32_t* flags, hipStream_t s) {
    return N == 512 ? launch_rows<9>(c, c16, restarts, tours, costs, moves, flags, s)
                    : launch_rows<10>(c, c16, restarts, tours, costs, moves, flags, s);
}

}  // namespace cc
