// Batched evaluation of the ring and halving-doubling cost models (Section 4.1) over candidate rank
// orders, plus the seeded initial-order generator and the matrix contract check.
//
// Ring, N a power of two in [8, 128]: the cost matrix (<= 64 KiB int32) is staged in LDS once per
// workgroup; the order stream is read from HBM as 16-byte vectors, N/4 lanes per order, several
// vector loads in flight per wave; each lane gathers its four hops from LDS and the N/4 lanes of an
// order are combined with a butterfly.  The stream is read exactly once, so the kernel is bound by
// HBM bandwidth (4N bytes in + 8 bytes out per order).
// Other N: one wave per order, hops gathered from the L2-resident matrix.
#include "cc_device.h"
#include "cc_internal.h"
#include "cc_wave64.h"

namespace cc {
using namespace ccd;

constexpr int kMaxRoundWeight = 1 << 30;   // round weights are clamped to [0, 2^30]: weight * cost stays below 2^51

// ------------------------------------------------------------------------------------------ ring
template <int N, bool IS_MAX>
__global__ __launch_bounds__(256) void ring_batch_lds_kernel(const int32_t* __restrict__ c,
                                                             const int4* __restrict__ perms4, int64_t B,
                                                             int64_t* __restrict__ out) {
    __shared__ int32_t m[N * N];
    for (int e = threadIdx.x; e < N * N; e += 256) m[e] = c[e];
    __syncthreads();

    constexpr int LP = N / 4;     // lanes that share one order
    constexpr int PPW = 64 / LP;  // orders covered by one 1 KiB wave-load
    constexpr int U = 4;          // wave-loads in flight
    constexpr int M = N - 1;
    const int lane = lane_id();
    const int sub = lane & (LP - 1);
    const int prev_lane = (lane & ~(LP - 1)) | ((sub + LP - 1) & (LP - 1));
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    const int64_t nloads = (B + PPW - 1) / PPW;

    for (int64_t base = wave * U; base < nloads; base += nwaves * U) {
        int4 v[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t ld = base + u;
            const int64_t b = ld * PPW + lane / LP;
            ok[u] = ld < nloads && b < B;
            v[u] = ok[u] ? perms4[ld * 64 + lane] : make_int4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int x = v[u].x & M, y = v[u].y & M, z = v[u].z & M, w = v[u].w & M;
            const int pw = __shfl(w, prev_lane, kWave);   // last node of the previous lane (cyclic in the order)
            const int h0 = m[x * N + pw], h1 = m[y * N + x], h2 = m[z * N + y], h3 = m[w * N + z];
            int acc = IS_MAX ? max(max(h0, h1), max(h2, h3)) : h0 + h1 + h2 + h3;
#pragma unroll
            for (int s = LP / 2; s >= 1; s >>= 1) {
                const int o = __shfl_xor(acc, s, kWave);
                acc = IS_MAX ? max(acc, o) : acc + o;
            }
            if (ok[u] && sub == 0) out[(base + u) * PPW + lane / LP] = (int64_t)acc;
        }
    }
}

template <bool IS_MAX>
__global__ __launch_bounds__(256) void ring_batch_generic_kernel(const int32_t* __restrict__ c, int N,
                                                                 const int32_t* __restrict__ perms, int64_t B,
                                                                 int64_t* __restrict__ out) {
    const int lane = lane_id();
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t b = wave; b < B; b += nwaves) {
        const int32_t* pi = perms + b * N;
        long long acc = 0;
        for (int p = lane; p < N; p += kWave) {
            const int a = clampi(pi[p], 0, N - 1);
            const int q = clampi(pi[p ? p - 1 : N - 1], 0, N - 1);
            const long long hop = c[(int64_t)a * N + q];
            acc = IS_MAX ? (hop > acc ? hop : acc) : acc + hop;
        }
#pragma unroll
        for (int s = 32; s >= 1; s >>= 1) {
            const long long o = __shfl_xor(acc, s, kWave);
            acc = IS_MAX ? (o > acc ? o : acc) : acc + o;
        }
        if (lane == 0) out[b] = acc;
    }
}

// Orders stored one byte per rank (N <= 256): a quarter of the HBM bytes per order.  N in {16, 32, 64, 128}: matrix
// in LDS; one lane fetches 16 ranks as an int4, N/16 adjacent lanes share an order, a wave-load covers 1024/N
// orders.  The hop into a lane's first rank needs the last rank of the lane before it (cyclically within the
// order's lanes), fetched with one lane permute.
template <int N, bool IS_MAX>
__global__ __launch_bounds__(256) void ring_batch_u8_lds_kernel(const int32_t* __restrict__ c,
                                                                const int4* __restrict__ perms16, int64_t B,
                                                                int64_t* __restrict__ out) {
    __shared__ int32_t m[N * N];
    for (int e = threadIdx.x; e < N * N; e += 256) m[e] = c[e];
    __syncthreads();

    constexpr int LP = N / 16;    // lanes that share one order
    constexpr int PPW = 64 / LP;  // orders covered by one 1 KiB wave-load
    constexpr int U = 2;          // wave-loads in flight
    constexpr unsigned M4 = (unsigned)(N - 1) * 0x01010101u;
    const int lane = lane_id();
    const int sub = lane & (LP - 1);
    const int prev_lane = (lane & ~(LP - 1)) | ((sub + LP - 1) & (LP - 1));
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    const int64_t nloads = (B + PPW - 1) / PPW;

    for (int64_t base = wave * U; base < nloads; base += nwaves * U) {
        int4 v[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t ld = base + u;
            const int64_t b = ld * PPW + lane / LP;
            ok[u] = ld < nloads && b < B;
            v[u] = ok[u] ? perms16[ld * 64 + lane] : make_int4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned w[4] = {(unsigned)v[u].x & M4, (unsigned)v[u].y & M4, (unsigned)v[u].z & M4,
                                   (unsigned)v[u].w & M4};
            int prev = (int)(w[3] >> 24);
            prev = LP > 1 ? __shfl(prev, prev_lane, kWave) : prev;   // last rank of the previous lane (or of this order)
            int acc = 0;
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const int node = (int)((w[k >> 2] >> (8 * (k & 3))) & 0xffu);
                const int hop = m[node * N + prev];
                acc = IS_MAX ? max(acc, hop) : acc + hop;
                prev = node;
            }
#pragma unroll
            for (int s = LP / 2; s >= 1; s >>= 1) {
                const int o = __shfl_xor(acc, s, kWave);
                acc = IS_MAX ? max(acc, o) : acc + o;
            }
            if (ok[u] && sub == 0) out[(base + u) * PPW + lane / LP] = (int64_t)acc;
        }
    }
}

// Orders stored one byte or two bytes per rank, any N: one wave per order, matrix through L2.
template <typename RANK, bool IS_MAX>
__global__ __launch_bounds__(256) void ring_batch_narrow_generic_kernel(const int32_t* __restrict__ c, int N,
                                                                        const RANK* __restrict__ perms, int64_t B,
                                                                        int64_t* __restrict__ out) {
    const int lane = lane_id();
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t b = wave; b < B; b += nwaves) {
        const RANK* pi = perms + b * N;
        long long acc = 0;
        for (int p = lane; p < N; p += kWave) {
            const int a = min((int)pi[p], N - 1);
            const int q = min((int)pi[p ? p - 1 : N - 1], N - 1);
            const long long hop = c[(int64_t)a * N + q];
            acc = IS_MAX ? (hop > acc ? hop : acc) : acc + hop;
        }
#pragma unroll
        for (int s = 32; s >= 1; s >>= 1) {
            const long long o = __shfl_xor(acc, s, kWave);
            acc = IS_MAX ? (o > acc ? o : acc) : acc + o;
        }
        if (lane == 0) out[b] = acc;
    }
}

static int batch_grid(int64_t work_items_per_block_pass, int64_t total) {
    int64_t blocks = (total + work_items_per_block_pass - 1) / work_items_per_block_pass;
    const int64_t cap = 256 * 8;  // 8 workgroups of 4 waves per compute unit
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return (int)blocks;
}

template <int N>
static hipError_t ring_lds(const int32_t* c, bool is_max, const int32_t* perms, int64_t B, int64_t* out,
                           hipStream_t s) {
    constexpr int PPW = 64 / (N / 4);
    const int grid = batch_grid((int64_t)PPW * 4 * 4, B);
    if (is_max)
        hipLaunchKernelGGL((ring_batch_lds_kernel<N, true>), dim3(grid), dim3(256), 0, s, c, (const int4*)perms, B, out);
    else
        hipLaunchKernelGGL((ring_batch_lds_kernel<N, false>), dim3(grid), dim3(256), 0, s, c, (const int4*)perms, B, out);
    return hipGetLastError();
}

// N = 256 for large batches: the matrix as 16-bit entries in LDS (128 KiB, one 1024-thread workgroup per compute
// unit), one wave per order: a 1 KiB wave-load is the order, four ranks per lane, the hop into a lane's first rank
// uses the previous lane's last node (cyclic), four LDS gathers per lane and one wave reduction per order.  Through
// L2 (generic kernel) the same batch runs at the L2's request rate, 256 scattered requests per order.  The workgroup
// finds the matrix maximum while staging; with an entry outside 0 .. 2^16 - 1 it scores its orders through L2 instead.
template <bool IS_MAX>
__global__ __launch_bounds__(1024) void ring_batch_n256_kernel(const int32_t* __restrict__ c,
                                                               const int4* __restrict__ perms4, int64_t B,
                                                               int64_t* __restrict__ out) {
    constexpr int N = 256, U = 4;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem256[];
    uint16_t* m16 = (uint16_t*)smem256;
    __shared__ unsigned wave_top[16];
    const int lane = lane_id(), wv = threadIdx.x >> 6;
    unsigned top = 0;
    for (int e = threadIdx.x; e < N * N; e += 1024) {
        const unsigned v = (unsigned)c[e];                 // a negative entry counts as too large
        top = max(top, v);
        m16[e] = (uint16_t)v;
    }
    top = (unsigned)wave_max((int)min(top, 0x7fffffffu));
    if (lane == 0) wave_top[wv] = top;
    __syncthreads();
    unsigned all_top = 0;
#pragma unroll
    for (int k = 0; k < 16; ++k) all_top = max(all_top, wave_top[k]);
    const bool in_lds = all_top < (1u << 16);
    const int64_t wave = (int64_t)blockIdx.x * 16 + wv;
    const int64_t nwaves = (int64_t)gridDim.x * 16;
    const char* mbytes = (const char*)m16;
    for (int64_t base = wave * U; base < B; base += nwaves * U) {
        int4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t b = base + u < B ? base + u : B - 1;
            v[u] = perms4[b * 64 + lane];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int x = v[u].x & 255, y = v[u].y & 255, z = v[u].z & 255, w = v[u].w & 255;
            const int pw = __builtin_amdgcn_update_dpp(w, w, 0x13C, 0xf, 0xf, true);   // lane p <- lane p - 1, cyclic
            int h0, h1, h2, h3;
            if (in_lds) {
                h0 = *(const uint16_t*)(mbytes + ((x << 9) | (pw << 1)));
                h1 = *(const uint16_t*)(mbytes + ((y << 9) | (x << 1)));
                h2 = *(const uint16_t*)(mbytes + ((z << 9) | (y << 1)));
                h3 = *(const uint16_t*)(mbytes + ((w << 9) | (z << 1)));
            } else {
                h0 = c[x * N + pw]; h1 = c[y * N + x]; h2 = c[z * N + y]; h3 = c[w * N + z];
            }
            long long total;
            if (IS_MAX) {
                total = max(wave_max(max(max(h0, h1), max(h2, h3))), 0);
            } else if (in_lds) {
                total = wave_sum(h0 + h1 + h2 + h3);       // at most 256 * 65535
            } else {
                total = wave_sum64((long long)h0 + h1 + h2 + h3);
            }
            if (lane == 0 && base + u < B) out[base + u] = total;
        }
    }
}

template <bool IS_MAX>
static hipError_t ring_n256_launch(const int32_t* c, const int32_t* perms, int64_t B, int64_t* out, hipStream_t s) {
    const size_t lds = sizeof(uint16_t) * 256 * 256;
    hipError_t e = hipFuncSetAttribute((const void*)ring_batch_n256_kernel<IS_MAX>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    int64_t blocks = (B + 16 * 4 - 1) / (16 * 4);
    if (blocks > 256) blocks = 256;
    hipLaunchKernelGGL(ring_batch_n256_kernel<IS_MAX>, dim3((int)blocks), dim3(1024), lds, s, c, (const int4*)perms, B,
                       out);
    return hipGetLastError();
}

hipError_t launch_ring_cost_batch(const int32_t* c, int N, bool is_max, const int32_t* perms, int64_t B,
                                  int64_t* out, hipStream_t s) {
    if (B == 0) return hipSuccess;
    const bool aligned = ((uintptr_t)perms & 15u) == 0;
    if (aligned) {
        switch (N) {
            case 8: return ring_lds<8>(c, is_max, perms, B, out, s);
            case 16: return ring_lds<16>(c, is_max, perms, B, out, s);
            case 32: return ring_lds<32>(c, is_max, perms, B, out, s);
            case 64: return ring_lds<64>(c, is_max, perms, B, out, s);
            case 128: return ring_lds<128>(c, is_max, perms, B, out, s);
            default: break;
        }
        // staging 128 KiB per compute unit pays from a few ten thousand orders on
        if (N == 256 && B >= 32768)
            return is_max ? ring_n256_launch<true>(c, perms, B, out, s) : ring_n256_launch<false>(c, perms, B, out, s);
    }
    const int grid = batch_grid(4, B);
    if (is_max)
        hipLaunchKernelGGL((ring_batch_generic_kernel<true>), dim3(grid), dim3(256), 0, s, c, N, perms, B, out);
    else
        hipLaunchKernelGGL((ring_batch_generic_kernel<false>), dim3(grid), dim3(256), 0, s, c, N, perms, B, out);
    return hipGetLastError();
}

template <int N>
static hipError_t ring_u8_lds(const int32_t* c, bool is_max, const uint8_t* perms, int64_t B, int64_t* out,
                              hipStream_t s) {
    constexpr int PPW = 64 / (N / 16);
    const int grid = batch_grid((int64_t)PPW * 2 * 4, B);
    if (is_max)
        hipLaunchKernelGGL((ring_batch_u8_lds_kernel<N, true>), dim3(grid), dim3(256), 0, s, c, (const int4*)perms, B,
                           out);
    else
        hipLaunchKernelGGL((ring_batch_u8_lds_kernel<N, false>), dim3(grid), dim3(256), 0, s, c, (const int4*)perms, B,
                           out);
    return hipGetLastError();
}

hipError_t launch_ring_cost_batch_u8(const int32_t* c, int N, bool is_max, const uint8_t* perms, int64_t B,
                                     int64_t* out, hipStream_t s) {
    if (B == 0) return hipSuccess;
    if (((uintptr_t)perms & 15u) == 0) {
        switch (N) {
            case 16: return ring_u8_lds<16>(c, is_max, perms, B, out, s);
            case 32: return ring_u8_lds<32>(c, is_max, perms, B, out, s);
            case 64: return ring_u8_lds<64>(c, is_max, perms, B, out, s);
            case 128: return ring_u8_lds<128>(c, is_max, perms, B, out, s);
            default: break;
        }
    }
    const int grid = batch_grid(4, B);
    if (is_max)
        hipLaunchKernelGGL((ring_batch_narrow_generic_kernel<uint8_t, true>), dim3(grid), dim3(256), 0, s, c, N, perms, B,
                           out);
    else
        hipLaunchKernelGGL((ring_batch_narrow_generic_kernel<uint8_t, false>), dim3(grid), dim3(256), 0, s, c, N, perms, B,
                           out);
    return hipGetLastError();
}

hipError_t launch_ring_cost_batch_u16(const int32_t* c, int N, bool is_max, const uint16_t* perms, int64_t B,
                                      int64_t* out, hipStream_t s) {
    if (B == 0) return hipSuccess;
    const int grid = batch_grid(4, B);
    if (is_max)
        hipLaunchKernelGGL((ring_batch_narrow_generic_kernel<uint16_t, true>), dim3(grid), dim3(256), 0, s, c, N, perms,
                           B, out);
    else
        hipLaunchKernelGGL((ring_batch_narrow_generic_kernel<uint16_t, false>), dim3(grid), dim3(256), 0, s, c, N, perms,
                           B, out);
    return hipGetLastError();
}

// ------------------------------------------------------------------------- halving-doubling rounds
// One wave per order.  The order is parked in the wave's LDS slice so that rank i can look up its
// partner i xor 2^k; NM = ceil(N / 64) ranks per lane.  Matrix in LDS when it fits 16 KiB (N <= 64),
// otherwise gathered through L2.
template <int NM, bool LDS_MATRIX>
__global__ __launch_bounds__(256) void rd_batch_kernel(const int32_t* __restrict__ c, int N,
                                                       const int32_t* __restrict__ weights,
                                                       const int32_t* __restrict__ perms, int64_t B,
                                                       int64_t* __restrict__ out,
                                                       const int32_t* __restrict__ skip_if_small) {
    // enqueued beside the folded-matrix kernel: flags[0] = max(c) decides which of the two does the work
    if (skip_if_small && skip_if_small[0] < (1 << 16)) return;
    extern __shared__ int32_t sm[];
    int32_t* order = sm + (threadIdx.x >> 6) * N;   // this wave's slice
    const int32_t* mat = c;
    if (LDS_MATRIX) {
        int32_t* m = sm + 4 * N;
        for (int e = threadIdx.x; e < N * N; e += 256) m[e] = c[e];
        __syncthreads();
        mat = m;
    }
    const int lane = lane_id();
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t b = wave; b < B; b += nwaves) {
        const int32_t* pi = perms + b * N;
        int a[NM];
#pragma unroll
        for (int k = 0; k < NM; ++k) {
            const int p = lane + 64 * k;
            a[k] = p < N ? clampi(pi[p], 0, N - 1) : 0;
            if (p < N) order[p] = a[k];
        }
        __builtin_amdgcn_wave_barrier();
        long long total = 0;
        int round = 0;
        for (int bit = 1; bit < N; bit <<= 1, ++round) {
            int worst = 0;
#pragma unroll
            for (int k = 0; k < NM; ++k) {
                const int p = lane + 64 * k;
                if (p < N) worst = max(worst, mat[a[k] * N + order[p ^ bit]]);
            }
            const long long w = weights ? (long long)clampi(weights[round], 0, kMaxRoundWeight) : 1ll;
            total += w * wave_max(worst);
        }
        __builtin_amdgcn_wave_barrier();   // all partner look-ups done before the slice is overwritten
        if (lane == 0) out[b] = total;
    }
}

// N = 64 with one order per LANE (orders 16-byte aligned): nothing is reduced across lanes.  A wave takes 64 orders:
// sixteen coalesced 1 KiB loads bring them in (lane l of load i holds four ranks of order 4i + l / 16), every rank
// is packed as the byte 4 * node, the packed words go through a 4.25 KiB LDS tile (17 words per order: writes two
// lanes per bank, reads conflict-free) and come back as the lane's own order, 64 bytes in 16 registers.  With all
// loops unrolled every rank of the order is a register with a constant index, so a matrix entry between the nodes
// at two ranks is { address = byte[x] << 6 | byte[y]; gather }, and the lane writes its own cost: 64 consecutive
// results per wave.
constexpr int kLaneTileStride = 17;                 // words per staged order: 16 of packed ranks, 1 of padding

// node4[p] = 4 * node at rank p of order b0 + lane (the last order again beyond the batch's end)
__device__ __forceinline__ void load_order_per_lane(const int4* __restrict__ perms4, int64_t b0, int64_t B,
                                                    uint32_t* tile, int lane, unsigned (&node4)[64]) {
    constexpr int N = 64;
    const int quarter = lane >> 4, piece = lane & 15;
    uint32_t packed[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        int64_t o = b0 + 4 * i + quarter;
        o = o < B ? o : B - 1;
        const int4 v = perms4[o * 16 + piece];
        packed[i] = (uint32_t)(clampi(v.x, 0, N - 1) << 2) | (uint32_t)(clampi(v.y, 0, N - 1) << 10) |
                    (uint32_t)(clampi(v.z, 0, N - 1) << 18) | (uint32_t)(clampi(v.w, 0, N - 1) << 26);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) tile[(4 * i + quarter) * kLaneTileStride + piece] = packed[i];
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const uint32_t word = tile[lane * kLaneTileStride + q];
#pragma unroll
        for (int j = 0; j < 4; ++j) node4[4 * q + j] = (word >> (8 * j)) & 0xffu;
    }
    __builtin_amdgcn_wave_barrier();                               // the tile is free for the next 64 orders
}

// stages the matrix; FOLD: both directed entries of a pair replaced by the larger (an exchange costs the slower way)
template <bool FOLD>
__device__ __forceinline__ void stage_matrix_64(const int32_t* __restrict__ c, int32_t* m) {
    constexpr int N = 64;
    for (int e = threadIdx.x; e < N * N; e += 256) m[e] = clampi(c[e], 0, (1 << 21) - 1);
    __syncthreads();
    if (FOLD) {
        w64::for_each_pair_64((int)threadIdx.x, [&](int lo, int hi) {
            const int both = max(m[lo * N + hi], m[hi * N + lo]);
            m[lo * N + hi] = both;
            m[hi * N + lo] = both;
        });
        __syncthreads();
    }
}

// halving-doubling: the 6 x 32 links of an order, one folded entry each
__global__ __launch_bounds__(256) void rd_batch_lanes64_kernel(const int32_t* __restrict__ c,
                                                               const int32_t* __restrict__ weights,
                                                               const int4* __restrict__ perms4, int64_t B,
                                                               int64_t* __restrict__ out) {
    constexpr int N = 64;
    __shared__ int32_t m[N * N];
    __shared__ uint32_t tile_all[4][N * kLaneTileStride];
    const int lane = lane_id(), wv = threadIdx.x >> 6;
    stage_matrix_64<true>(c, m);
    const char* mbytes = (const char*)m;
    long long w[6];
#pragma unroll
    for (int k = 0; k < 6; ++k) w[k] = weights ? (long long)clampi(weights[k], 0, kMaxRoundWeight) : 1ll;
    const int64_t tasks = (B + 63) >> 6;
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t task = (int64_t)blockIdx.x * 4 + wv; task < tasks; task += nwaves) {
        const int64_t b0 = task << 6;
        unsigned node4[N];
        load_order_per_lane(perms4, b0, B, tile_all[wv], lane, node4);
        long long total = 0;
#pragma unroll
        for (int k = 0; k < 6; ++k) {
            int worst = 0;
#pragma unroll
            for (int li = 0; li < N / 2; ++li) {
                const int lo = ((li >> k) << (k + 1)) | (li & ((1 << k) - 1)), hi = lo | (1 << k);
                worst = max(worst, *(const int32_t*)(mbytes + ((node4[lo] << 6) | node4[hi])));
            }
            total += w[k] * worst;
        }
        if (b0 + lane < B) out[b0 + lane] = total;
    }
}

// BCube, base 4: the four ranks that differ in one base-4 digit exchange pairwise; 3 rounds x 16 groups x 6 pairs,
// one folded entry each
__global__ __launch_bounds__(256) void bcube_b4_lanes64_kernel(const int32_t* __restrict__ c,
                                                               const int32_t* __restrict__ weights,
                                                               const int4* __restrict__ perms4, int64_t B,
                                                               int64_t* __restrict__ out) {
    constexpr int N = 64;
    __shared__ int32_t m[N * N];
    __shared__ uint32_t tile_all[4][N * kLaneTileStride];
    const int lane = lane_id(), wv = threadIdx.x >> 6;
    stage_matrix_64<true>(c, m);
    const char* mbytes = (const char*)m;
    long long w[3];
#pragma unroll
    for (int r = 0; r < 3; ++r) w[r] = weights ? (long long)clampi(weights[r], 0, kMaxRoundWeight) : 1ll;
    const int64_t tasks = (B + 63) >> 6;
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t task = (int64_t)blockIdx.x * 4 + wv; task < tasks; task += nwaves) {
        const int64_t b0 = task << 6;
        unsigned node4[N];
        load_order_per_lane(perms4, b0, B, tile_all[wv], lane, node4);
        long long total = 0;
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            int worst = 0;
#pragma unroll
            for (int g = 0; g < N / 4; ++g) {
                const int p0 = ((g >> (2 * r)) << (2 * r + 2)) | (g & ((1 << (2 * r)) - 1));
#pragma unroll
                for (int d = 0; d < 3; ++d)
#pragma unroll
                    for (int e = d + 1; e < 4; ++e)
                        worst = max(worst, *(const int32_t*)(mbytes + ((node4[p0 | (d << (2 * r))] << 6) |
                                                                       node4[p0 | (e << (2 * r))])));
            }
            total += w[r] * worst;
        }
        if (b0 + lane < B) out[b0 + lane] = total;
    }
}

// Double binary tree: the tree over positions LO .. HI hangs below a parent whose node and path cost are given; the
// costliest root-to-leaf path is the largest path cost met.  SHIFT: tree position p holds rank (p + SHIFT) mod 64.
template <int LO, int HI, int SHIFT>
__device__ __forceinline__ void dbt_walk_64(const char* mbytes, const unsigned (&node4)[64], unsigned parent4, int cost,
                                            bool has_parent, int& worst) {
    if constexpr (LO <= HI) {
        constexpr int M = (LO + HI) / 2;
        const unsigned here = node4[(M + SHIFT) & 63];
        const int mine = has_parent ? cost + *(const int32_t*)(mbytes + ((parent4 << 6) | here)) : 0;
        worst = max(worst, mine);
        dbt_walk_64<LO, M - 1, SHIFT>(mbytes, node4, here, mine, true, worst);
        dbt_walk_64<M + 1, HI, SHIFT>(mbytes, node4, here, mine, true, worst);
    }
}

__global__ __launch_bounds__(256) void dbt_lanes64_kernel(const int32_t* __restrict__ c,
                                                          const int4* __restrict__ perms4, int64_t B,
                                                          int64_t* __restrict__ out) {
    constexpr int N = 64;
    __shared__ int32_t m[N * N];
    __shared__ uint32_t tile_all[4][N * kLaneTileStride];
    const int lane = lane_id(), wv = threadIdx.x >> 6;
    stage_matrix_64<false>(c, m);
    const char* mbytes = (const char*)m;
    const int64_t tasks = (B + 63) >> 6;
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t task = (int64_t)blockIdx.x * 4 + wv; task < tasks; task += nwaves) {
        const int64_t b0 = task << 6;
        unsigned node4[N];
        load_order_per_lane(perms4, b0, B, tile_all[wv], lane, node4);
        int worst = 0;
        dbt_walk_64<0, N - 1, 0>(mbytes, node4, 0u, 0, false, worst);
        dbt_walk_64<0, N - 1, 1>(mbytes, node4, 0u, 0, false, worst);
        if (b0 + lane < B) out[b0 + lane] = worst;
    }
}

// N = 32 or 64 with the matrix in LDS: the rounds are unrolled, so the partner look-ups and the gathers of all rounds are
// in flight together and the rounds' maxima are reduced three at a time; the next order is requested before the
// current one is scored.
template <int LOGN>
__global__ __launch_bounds__(256) void rd_batch_small_kernel(const int32_t* __restrict__ c,
                                                             const int32_t* __restrict__ weights,
                                                             const int32_t* __restrict__ perms, int64_t B,
                                                             int64_t* __restrict__ out) {
    constexpr int N = 1 << LOGN;
    __shared__ int32_t m[N * N];
    __shared__ int32_t order_all[4][N];
    for (int e = threadIdx.x; e < N * N; e += 256) m[e] = c[e];
    __syncthreads();
    int32_t* order = order_all[threadIdx.x >> 6];
    const int lane = lane_id();
    const bool live = lane < N;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    long long w[6];
#pragma unroll
    for (int k = 0; k < 6; ++k) w[k] = (k < LOGN && weights) ? (long long)clampi(weights[k], 0, kMaxRoundWeight) : 1ll;
    int next = (wave < B && live) ? perms[wave * N + lane] : 0;
    for (int64_t b = wave; b < B; b += nwaves) {
        const int a = clampi(next, 0, N - 1);
        const int64_t bn = b + nwaves;
        next = (bn < B && live) ? perms[bn * N + lane] : 0;
        if (live) order[lane] = a;
        __builtin_amdgcn_wave_barrier();
        int v[6];
#pragma unroll
        for (int k = 0; k < 6; ++k) v[k] = (k < LOGN && live) ? m[a * N + order[lane ^ (1 << k)]] : 0;
        __builtin_amdgcn_wave_barrier();   // all partner look-ups done before the slice is overwritten
        wave_max3(v[0], v[1], v[2]);
        wave_max3(v[3], v[4], v[5]);
        long long total = 0;
#pragma unroll
        for (int k = 0; k < LOGN; ++k) total += w[k] * v[k];
        if (lane == 0) out[b] = total;
    }
}

// N = 64: a round costs the largest of its 32 links and a link costs the larger of its two directed entries, so the
// kernel folds the two entries of every pair into both places while staging (max(c[x][y], c[y][x])) and then scores
// links, not ranks: the 6 x 32 links of an order are three gathers per lane (lanes 0..31 one round, lanes 32..63 the
// next), and the six maxima come from three reductions over half waves.
__global__ __launch_bounds__(256) void rd_batch_links64_kernel(const int32_t* __restrict__ c,
                                                               const int32_t* __restrict__ weights,
                                                               const int32_t* __restrict__ perms, int64_t B,
                                                               int64_t* __restrict__ out) {
    constexpr int N = 64;
    __shared__ int32_t m[N * N];
    __shared__ int32_t order_all[4][N];
    const int lane = lane_id(), wv = threadIdx.x >> 6;
    for (int e = threadIdx.x; e < N * N; e += 256) m[e] = clampi(c[e], 0, (1 << 21) - 1);
    __syncthreads();
    w64::for_each_pair_64((int)threadIdx.x, [&](int lo, int hi) {
        const int both = max(m[lo * N + hi], m[hi * N + lo]);
        m[lo * N + hi] = both;
        m[hi * N + lo] = both;
    });
    __syncthreads();
    int32_t* order = order_all[wv];
    const int64_t wave = (int64_t)blockIdx.x * 4 + wv;
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    long long w[6];
#pragma unroll
    for (int k = 0; k < 6; ++k) w[k] = weights ? (long long)clampi(weights[k], 0, kMaxRoundWeight) : 1ll;
    // link j of this lane: round k = 2j + (lane >> 5), link index lane & 31 = the lower rank with bit k taken out
    int lower[3], upper[3];
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        const int k = 2 * j + (lane >> 5), li = lane & 31;
        lower[j] = ((li >> k) << (k + 1)) | (li & ((1 << k) - 1));
        upper[j] = lower[j] | (1 << k);
    }
    int next = wave < B ? perms[wave * N + lane] : 0;
    for (int64_t b = wave; b < B; b += nwaves) {
        order[lane] = clampi(next, 0, N - 1);
        const int64_t bn = b + nwaves;
        next = bn < B ? perms[bn * N + lane] : 0;
        __builtin_amdgcn_wave_barrier();
        int v[3];
#pragma unroll
        for (int j = 0; j < 3; ++j) v[j] = m[order[lower[j]] * N + order[upper[j]]];
        __builtin_amdgcn_wave_barrier();   // all look-ups done before the slice is overwritten
        half_wave_max3(v[0], v[1], v[2]);
        long long total = 0;
#pragma unroll
        for (int j = 0; j < 3; ++j)
            total += w[2 * j] * __builtin_amdgcn_readlane(v[j], 31) + w[2 * j + 1] * __builtin_amdgcn_readlane(v[j], 63);
        if (lane == 0) out[b] = total;
    }
}

template <int LOGN>
static hipError_t rd_small_launch(const int32_t* c, const int32_t* weights, const int32_t* perms, int64_t B,
                                  int64_t* out, hipStream_t s) {
    const int grid = batch_grid(4, B);
    hipLaunchKernelGGL(rd_batch_small_kernel<LOGN>, dim3(grid), dim3(256), 0, s, c, weights, perms, B, out);
    return hipGetLastError();
}

template <int NM>
static hipError_t rd_launch(const int32_t* c, int N, const int32_t* weights, const int32_t* perms, int64_t B,
                            int64_t* out, const int32_t* skip_if_small, hipStream_t s) {
    const int grid = batch_grid(4, B);
    if (N <= 64) {
        const size_t lds = sizeof(int32_t) * (size_t)(4 * N + N * N);
        hipLaunchKernelGGL((rd_batch_kernel<NM, true>), dim3(grid), dim3(256), lds, s, c, N, weights, perms, B, out,
                           skip_if_small);
    } else {
        const size_t lds = sizeof(int32_t) * (size_t)(4 * N);
        hipLaunchKernelGGL((rd_batch_kernel<NM, false>), dim3(grid), dim3(256), lds, s, c, N, weights, perms, B, out,
                           skip_if_small);
    }
    return hipGetLastError();
}

// N = 128 .. 1024 on a folded 16-bit copy of the matrix, folded[x][y] = max(c[x][y], c[y][x]) (fold_to_u16_kernel): a
// link, the two ranks i and i xor 2^k, is one look-up by one lane instead of one per end, so a round is N / 2
// scattered L2 requests instead of N - and that request rate is what bounds this kernel.  One wave per order, the
// order parked in LDS; every lane first takes the maximum over its links of every round (all gathers independent),
// then the rounds' maxima are reduced over the wave three at a time.  Returns at once when the matrix has an entry
// from 2^16 up (flags[0] = max(c)): the general kernel, enqueued beside it, then does the work.
template <int LOGN>
__global__ __launch_bounds__(256) void rd_batch_folded_kernel(const uint16_t* __restrict__ folded,
                                                              const int32_t* __restrict__ weights,
                                                              const int32_t* __restrict__ perms, int64_t B,
                                                              int64_t* __restrict__ out,
                                                              const int32_t* __restrict__ flags) {
    constexpr int N = 1 << LOGN, NM = N / 64, LM = NM / 2;      // ranks and links per lane
    if (flags[0] >= (1 << 16)) return;
    __shared__ int32_t order_all[4][N];
    int32_t* order = order_all[threadIdx.x >> 6];
    const int lane = lane_id();
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    long long w[LOGN];
#pragma unroll
    for (int k = 0; k < LOGN; ++k) w[k] = weights ? (long long)clampi(weights[k], 0, kMaxRoundWeight) : 1ll;
    for (int64_t b = wave; b < B; b += nwaves) {
        const int32_t* pi = perms + b * N;
#pragma unroll
        for (int k = 0; k < NM; ++k) order[lane + 64 * k] = clampi(pi[lane + 64 * k], 0, N - 1);
        __builtin_amdgcn_wave_barrier();
        int worst[LOGN + 2];
        worst[LOGN] = worst[LOGN + 1] = 0;
#pragma unroll
        for (int k = 0; k < LOGN; ++k) {
            const int bit = 1 << k;
            int v = 0;
#pragma unroll
            for (int u = 0; u < LM; ++u) {
                const int i = lane + 64 * u;                                      // link index
                const int j = ((i >> k) << (k + 1)) | (i & (bit - 1));            // its lower rank
                const unsigned at = ((unsigned)order[j] << (LOGN + 1)) | ((unsigned)order[j | bit] << 1);
                v = max(v, (int)*(const uint16_t*)((const char*)folded + at));
            }
            worst[k] = v;
        }
        __builtin_amdgcn_wave_barrier();   // all look-ups done before the slice is overwritten
#pragma unroll
        for (int k = 0; k < LOGN; k += 3) wave_max3(worst[k], worst[k + 1], worst[k + 2]);
        long long total = 0;
#pragma unroll
        for (int k = 0; k < LOGN; ++k) total += w[k] * worst[k];
        if (lane == 0) out[b] = total;
    }
}

// N = 128, 256 for large batches, matrix in LDS: a 1024-thread workgroup per compute unit stages the matrix as 16-bit
// entries, folds the two directions of every pair into both places (as rdswap_block_kernel does) and then scores one
// order per wave as rd_batch_folded_kernel / bcube_b4_folded_kernel do, with LDS gathers instead of L2 requests.
// The workgroup finds the matrix maximum while staging; with an entry outside 0 .. 2^16 - 1 its links are scored from
// the caller's matrix through L2 (both directions per link).  BCUBE4: base-4 BCube rounds instead of halving-doubling.
template <int LOGN, bool BCUBE4>
__global__ __launch_bounds__(1024) void links_batch_lds16_kernel(const int32_t* __restrict__ c,
                                                                 const int32_t* __restrict__ weights,
                                                                 const int32_t* __restrict__ perms, int64_t B,
                                                                 int64_t* __restrict__ out) {
    constexpr int N = 1 << LOGN, NM = N / 64, ROUNDS = BCUBE4 ? LOGN / 2 : LOGN;
    static_assert(!BCUBE4 || LOGN % 2 == 0, "base 4 needs an even log2 N");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_links[];
    uint16_t* m16 = (uint16_t*)smem_links;                                  // [N * N]
    int32_t* order_all = (int32_t*)(smem_links + sizeof(uint16_t) * N * N);  // [16][N]
    __shared__ unsigned wave_top[16];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    unsigned top = 0;
    for (int e = tid; e < N * N; e += 1024) {
        const unsigned v = (unsigned)c[e];                 // a negative entry counts as too large
        top = max(top, v);
        m16[e] = (uint16_t)v;
    }
    top = (unsigned)wave_max((int)min(top, 0x7fffffffu));
    if (lane == 0) wave_top[wv] = top;
    __syncthreads();
    unsigned all_top = 0;
#pragma unroll
    for (int k = 0; k < 16; ++k) all_top = max(all_top, wave_top[k]);
    const bool in_lds = all_top < (1u << 16);
    if (in_lds) {
        // the threads of rank p take the pairs {p, p + j}, j = 1 .. N/2: every unordered pair exactly once
        const int p = tid & (N - 1);
        for (int j = 1 + (tid >> LOGN); j <= N / 2; j += 1024 / N) {
            const int b = (p + j) & (N - 1);
            if (j < N / 2 || p < N / 2) {
                const uint16_t both = max(m16[p * N + b], m16[b * N + p]);
                m16[p * N + b] = both;
                m16[b * N + p] = both;
            }
        }
    }
    __syncthreads();
    auto pair_value = [&](int x, int y) {
        if (in_lds) return (int)*(const uint16_t*)((const char*)m16 + ((x << (LOGN + 1)) | (y << 1)));
        return max(clampi(c[x * N + y], 0, (1 << 21) - 1), clampi(c[y * N + x], 0, (1 << 21) - 1));
    };
    int32_t* order = order_all + wv * N;
    long long w[ROUNDS];
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) w[r] = weights ? (long long)clampi(weights[r], 0, kMaxRoundWeight) : 1ll;
    const int64_t nwaves = (int64_t)gridDim.x * 16;
    for (int64_t b = (int64_t)blockIdx.x * 16 + wv; b < B; b += nwaves) {
        const int32_t* pi = perms + b * N;
#pragma unroll
        for (int k = 0; k < NM; ++k) order[lane + 64 * k] = clampi(pi[lane + 64 * k], 0, N - 1);
        __builtin_amdgcn_wave_barrier();
        int worst[ROUNDS + 2];
        worst[ROUNDS] = worst[ROUNDS + 1] = 0;
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            int v = 0;
            if (BCUBE4) {
#pragma unroll
                for (int u = 0; u < N / 256; ++u) {
                    const int g = lane + 64 * u;                                   // group: the rank without digit r
                    const int p0 = ((g >> (2 * r)) << (2 * r + 2)) | (g & ((1 << (2 * r)) - 1));
                    int node[4];
#pragma unroll
                    for (int d = 0; d < 4; ++d) node[d] = order[p0 | (d << (2 * r))];
#pragma unroll
                    for (int d = 0; d < 3; ++d)
#pragma unroll
                        for (int e = d + 1; e < 4; ++e) v = max(v, pair_value(node[d], node[e]));
                }
            } else {
                const int bit = 1 << r;
#pragma unroll
                for (int u = 0; u < NM / 2; ++u) {
                    const int i = lane + 64 * u;                                   // link index
                    const int j = ((i >> r) << (r + 1)) | (i & (bit - 1));         // its lower rank
                    v = max(v, pair_value(order[j], order[j | bit]));
                }
            }
            worst[r] = v;
        }
        __builtin_amdgcn_wave_barrier();   // all look-ups done before the slice is overwritten
#pragma unroll
        for (int r = 0; r < ROUNDS; r += 3) wave_max3(worst[r], worst[r + 1], worst[r + 2]);
        long long total = 0;
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) total += w[r] * worst[r];
        if (lane == 0) out[b] = total;
    }
}

constexpr int64_t kLdsBatchMinOrders = 32768;      // staging a matrix per compute unit pays from here on

template <int LOGN, bool BCUBE4>
static hipError_t links_lds16_launch(const int32_t* c, const int32_t* weights, const int32_t* perms, int64_t B,
                                     int64_t* out, hipStream_t s) {
    constexpr int N = 1 << LOGN;
    const size_t lds = sizeof(uint16_t) * N * N + sizeof(int32_t) * 16 * N;
    hipError_t e = hipFuncSetAttribute((const void*)links_batch_lds16_kernel<LOGN, BCUBE4>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    int64_t blocks = (B + 15) / 16;
    if (blocks > 256) blocks = 256;
    hipLaunchKernelGGL((links_batch_lds16_kernel<LOGN, BCUBE4>), dim3((int)blocks), dim3(1024), lds, s, c, weights, perms,
                       B, out);
    return hipGetLastError();
}

template <int LOGN>
static hipError_t rd_folded_launch(const uint16_t* folded, const int32_t* weights, const int32_t* perms, int64_t B,
                                   int64_t* out, const int32_t* flags, hipStream_t s) {
    hipLaunchKernelGGL(rd_batch_folded_kernel<LOGN>, dim3(batch_grid(4, B)), dim3(256), 0, s, folded, weights, perms, B,
                       out, flags);
    return hipGetLastError();
}

hipError_t launch_rd_cost_batch(const int32_t* c, int N, const int32_t* weights, const int32_t* perms, int64_t B,
                                int64_t* out, hipStream_t s, int32_t* flags, uint16_t* folded) {
    if (B == 0) return hipSuccess;
    if (N == 64) {
        if (((uintptr_t)perms & 15u) == 0)
            hipLaunchKernelGGL(rd_batch_lanes64_kernel, dim3(batch_grid(4 * 64, B)), dim3(256), 0, s, c, weights,
                               (const int4*)perms, B, out);
        else
            hipLaunchKernelGGL(rd_batch_links64_kernel, dim3(batch_grid(4, B)), dim3(256), 0, s, c, weights, perms, B, out);
        return hipGetLastError();
    }
    if (N == 32) return rd_small_launch<5>(c, weights, perms, B, out, s);
    if (N <= 64) return rd_launch<1>(c, N, weights, perms, B, out, nullptr, s);
    if (B >= kLdsBatchMinOrders) {
        if (N == 128) return links_lds16_launch<7, false>(c, weights, perms, B, out, s);
        if (N == 256) return links_lds16_launch<8, false>(c, weights, perms, B, out, s);
    }
    const int32_t* skip = nullptr;
    if (flags && folded) {
        // both kernels are enqueued; the matrix maximum, computed on the device, decides which of them works
        hipError_t e = launch_matrix_max(c, N, flags, s);
        if (e == hipSuccess) e = launch_fold_to_u16(c, N, folded, flags, s);
        if (e == hipSuccess)
            e = N == 128   ? rd_folded_launch<7>(folded, weights, perms, B, out, flags, s)
                : N == 256 ? rd_folded_launch<8>(folded, weights, perms, B, out, flags, s)
                : N == 512 ? rd_folded_launch<9>(folded, weights, perms, B, out, flags, s)
                           : rd_folded_launch<10>(folded, weights, perms, B, out, flags, s);
        if (e != hipSuccess) return e;
        skip = flags;
    }
    if (N == 128) return rd_launch<2>(c, N, weights, perms, B, out, skip, s);
    if (N == 256) return rd_launch<4>(c, N, weights, perms, B, out, skip, s);
    if (N == 512) return rd_launch<8>(c, N, weights, perms, B, out, skip, s);
    return rd_launch<16>(c, N, weights, perms, B, out, skip, s);
}

// ------------------------------------------------------------------------------- BCube cost model
// Section 4.1, equation C_b: round i pairs every rank with the base-1 ranks that differ from it in
// base-`base` digit i only; the round costs its slowest exchange.  Same gather-max-sum shape as the
// halving-doubling kernel with base-1 gathers per rank and round.
template <int NM, bool LDS_MATRIX>
__global__ __launch_bounds__(256) void bcube_batch_kernel(const int32_t* __restrict__ c, int N, int base,
                                                          const int32_t* __restrict__ weights,
                                                          const int32_t* __restrict__ perms, int64_t B,
                                                          int64_t* __restrict__ out,
                                                          const int32_t* __restrict__ skip_if_small) {
    // enqueued beside the folded-matrix kernel: flags[0] = max(c) decides which of the two does the work
    if (skip_if_small && skip_if_small[0] < (1 << 16)) return;
    extern __shared__ int32_t sm[];
    int32_t* order = sm + (threadIdx.x >> 6) * N;
    const int32_t* mat = c;
    if (LDS_MATRIX) {
        int32_t* m = sm + 4 * N;
        for (int e = threadIdx.x; e < N * N; e += 256) m[e] = c[e];
        __syncthreads();
        mat = m;
    }
    const int lane = lane_id();
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t b = wave; b < B; b += nwaves) {
        const int32_t* pi = perms + b * N;
        int a[NM];
#pragma unroll
        for (int k = 0; k < NM; ++k) {
            const int p = lane + 64 * k;
            a[k] = p < N ? clampi(pi[p], 0, N - 1) : 0;
            if (p < N) order[p] = a[k];
        }
        __builtin_amdgcn_wave_barrier();
        long long total = 0;
        int round = 0;
        for (int stride = 1; stride < N; stride *= base, ++round) {
            int worst = 0;
#pragma unroll
            for (int k = 0; k < NM; ++k) {
                const int p = lane + 64 * k;
                if (p < N) {
                    const int digit = (p / stride) % base;
                    const int* row = mat + a[k] * N;
                    int peer_digit = digit;
                    for (int step = 1; step < base; ++step) {
                        peer_digit = peer_digit + 1 == base ? 0 : peer_digit + 1;
                        worst = max(worst, row[order[p + (peer_digit - digit) * stride]]);
                    }
                }
            }
            const long long w = weights ? (long long)clampi(weights[round], 0, kMaxRoundWeight) : 1ll;
            total += w * wave_max(worst);
        }
        __builtin_amdgcn_wave_barrier();
        if (lane == 0) out[b] = total;
    }
}

template <int NM>
static hipError_t bcube_launch(const int32_t* c, int N, int base, const int32_t* weights, const int32_t* perms,
                               int64_t B, int64_t* out, const int32_t* skip_if_small, hipStream_t s) {
    const int grid = batch_grid(4, B);
    if (N <= 64) {
        const size_t lds = sizeof(int32_t) * (size_t)(4 * N + N * N);
        hipLaunchKernelGGL((bcube_batch_kernel<NM, true>), dim3(grid), dim3(256), lds, s, c, N, base, weights, perms, B,
                           out, skip_if_small);
    } else {
        const size_t lds = sizeof(int32_t) * (size_t)(4 * N);
        hipLaunchKernelGGL((bcube_batch_kernel<NM, false>), dim3(grid), dim3(256), lds, s, c, N, base, weights, perms, B,
                           out, skip_if_small);
    }
    return hipGetLastError();
}

// N = 64, base 4 (the paper's BCube setting at the size of the bench's batch): lane = rank, the nine peers of a rank
// (three per round) are fixed lane numbers computed once, the three rounds' maxima are reduced together, the next
// order of the wave is requested while this one is scored.
__global__ __launch_bounds__(256) void bcube_batch_b4n64_kernel(const int32_t* __restrict__ c,
                                                                const int32_t* __restrict__ weights,
                                                                const int32_t* __restrict__ perms, int64_t B,
                                                                int64_t* __restrict__ out) {
    constexpr int N = 64;
    __shared__ int32_t m[N * N];
    __shared__ int32_t order_all[4][N];
    for (int e = threadIdx.x; e < N * N; e += 256) m[e] = c[e];
    __syncthreads();
    const int lane = lane_id();
    int32_t* order = order_all[threadIdx.x >> 6];
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    long long w[3];
    int peer[3][3];
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        w[r] = weights ? (long long)clampi(weights[r], 0, kMaxRoundWeight) : 1ll;
        const int digit = (lane >> (2 * r)) & 3, rest = lane & ~(3 << (2 * r));
#pragma unroll
        for (int s = 1; s <= 3; ++s) peer[r][s - 1] = rest | (((digit + s) & 3) << (2 * r));
    }
    int next = wave < B ? perms[wave * N + lane] : 0;
    for (int64_t b = wave; b < B; b += nwaves) {
        const int a = clampi(next, 0, N - 1);
        const int64_t bn = b + nwaves;
        next = bn < B ? perms[bn * N + lane] : 0;
        order[lane] = a;
        __builtin_amdgcn_wave_barrier();
        int v[3];
#pragma unroll
        for (int r = 0; r < 3; ++r)
            v[r] = max(m[a * N + order[peer[r][0]]], max(m[a * N + order[peer[r][1]]], m[a * N + order[peer[r][2]]]));
        __builtin_amdgcn_wave_barrier();   // all look-ups done before the slice is overwritten
        wave_max3(v[0], v[1], v[2]);
        if (lane == 0) out[b] = w[0] * v[0] + w[1] * v[1] + w[2] * v[2];
    }
}

// Base 4 at N = 256, 1024 on the folded 16-bit copy of the matrix (as rd_batch_folded_kernel): the four ranks that
// differ in one base-4 digit exchange pairwise, and both directions of a pair are one folded entry, so a round is the
// maximum over N / 4 groups of six entries - 1.5 N look-ups instead of 3 N.  A lane takes whole groups: four order
// look-ups in LDS, six gathers.  Returns at once when flags[0] = max(c) is 2^16 or more.
template <int ROUNDS>
__global__ __launch_bounds__(256) void bcube_b4_folded_kernel(const uint16_t* __restrict__ folded,
                                                              const int32_t* __restrict__ weights,
                                                              const int32_t* __restrict__ perms, int64_t B,
                                                              int64_t* __restrict__ out,
                                                              const int32_t* __restrict__ flags) {
    constexpr int LOGN = 2 * ROUNDS, N = 1 << LOGN, NM = N / 64, GM = N / 256;      // ranks and groups per lane
    if (flags[0] >= (1 << 16)) return;
    __shared__ int32_t order_all[4][N];
    int32_t* order = order_all[threadIdx.x >> 6];
    const int lane = lane_id();
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    long long w[ROUNDS];
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) w[r] = weights ? (long long)clampi(weights[r], 0, kMaxRoundWeight) : 1ll;
    for (int64_t b = wave; b < B; b += nwaves) {
        const int32_t* pi = perms + b * N;
#pragma unroll
        for (int k = 0; k < NM; ++k) order[lane + 64 * k] = clampi(pi[lane + 64 * k], 0, N - 1);
        __builtin_amdgcn_wave_barrier();
        int worst[ROUNDS + 2];
        worst[ROUNDS] = worst[ROUNDS + 1] = 0;
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            int v = 0;
#pragma unroll
            for (int u = 0; u < GM; ++u) {
                const int g = lane + 64 * u;                                       // group: the rank without digit r
                const int p0 = ((g >> (2 * r)) << (2 * r + 2)) | (g & ((1 << (2 * r)) - 1));
                unsigned node[4];
#pragma unroll
                for (int d = 0; d < 4; ++d) node[d] = (unsigned)order[p0 | (d << (2 * r))];
#pragma unroll
                for (int d = 0; d < 3; ++d)
#pragma unroll
                    for (int e = d + 1; e < 4; ++e)
                        v = max(v, (int)*(const uint16_t*)((const char*)folded +
                                                            ((node[d] << (LOGN + 1)) | (node[e] << 1))));
            }
            worst[r] = v;
        }
        __builtin_amdgcn_wave_barrier();   // all look-ups done before the slice is overwritten
#pragma unroll
        for (int r = 0; r < ROUNDS; r += 3) wave_max3(worst[r], worst[r + 1], worst[r + 2]);
        long long total = 0;
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) total += w[r] * worst[r];
        if (lane == 0) out[b] = total;
    }
}

hipError_t launch_bcube_cost_batch(const int32_t* c, int N, int base, const int32_t* weights, const int32_t* perms,
                                   int64_t B, int64_t* out, hipStream_t s, int32_t* flags, uint16_t* folded) {
    if (B == 0) return hipSuccess;
    if (base == 2) return launch_rd_cost_batch(c, N, weights, perms, B, out, s, flags, folded);
    if (N == 64 && base == 4) {
        if (((uintptr_t)perms & 15u) == 0)
            hipLaunchKernelGGL(bcube_b4_lanes64_kernel, dim3(batch_grid(4 * 64, B)), dim3(256), 0, s, c, weights,
                               (const int4*)perms, B, out);
        else
            hipLaunchKernelGGL(bcube_batch_b4n64_kernel, dim3(batch_grid(4, B)), dim3(256), 0, s, c, weights, perms, B, out);
        return hipGetLastError();
    }
    if (base == 4 && N == 256 && B >= kLdsBatchMinOrders) return links_lds16_launch<8, true>(c, weights, perms, B, out, s);
    const int32_t* skip = nullptr;
    if (flags && folded && base == 4 && (N == 256 || N == 1024)) {
        // both kernels are enqueued; the matrix maximum, computed on the device, decides which of them works
        hipError_t e = launch_matrix_max(c, N, flags, s);
        if (e == hipSuccess) e = launch_fold_to_u16(c, N, folded, flags, s);
        if (e != hipSuccess) return e;
        const int grid = batch_grid(4, B);
        if (N == 256)
            hipLaunchKernelGGL(bcube_b4_folded_kernel<4>, dim3(grid), dim3(256), 0, s, folded, weights, perms, B, out, flags);
        else
            hipLaunchKernelGGL(bcube_b4_folded_kernel<5>, dim3(grid), dim3(256), 0, s, folded, weights, perms, B, out, flags);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        skip = flags;
    }
    if (N <= 64) return bcube_launch<1>(c, N, base, weights, perms, B, out, skip, s);
    if (N <= 128) return bcube_launch<2>(c, N, base, weights, perms, B, out, skip, s);
    if (N <= 256) return bcube_launch<4>(c, N, base, weights, perms, B, out, skip, s);
    if (N <= 512) return bcube_launch<8>(c, N, base, weights, perms, B, out, skip, s);
    return bcube_launch<16>(c, N, base, weights, perms, B, out, skip, s);
}

// --------------------------------------------------------------------- double-binary-tree cost model
// Section 4.1, equation C_dbt: the ranks form an in-order binary tree whose subtree roots are the middle
// ranks of their ranges; a tree costs its most expensive root-to-leaf path; the second tree has the same
// shape one position further along the order; the result is the larger of the two.  Every lane walks from
// the root to its own position (a binary search, at most 10 hops), adding c[parent][child] per hop; the
// largest path over the wave is the tree's cost.
template <bool LDS_MATRIX>
__global__ __launch_bounds__(256) void dbt_batch_kernel(const int32_t* __restrict__ c, int N,
                                                        const int32_t* __restrict__ perms, int64_t B,
                                                        int64_t* __restrict__ out) {
    extern __shared__ int32_t sm[];
    int32_t* order = sm + (threadIdx.x >> 6) * N;
    const int32_t* mat = c;
    if (LDS_MATRIX) {
        int32_t* m = sm + 4 * N;
        for (int e = threadIdx.x; e < N * N; e += 256) m[e] = c[e];
        __syncthreads();
        mat = m;
    }
    const int lane = lane_id();
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t b = wave; b < B; b += nwaves) {
        const int32_t* pi = perms + b * N;
        for (int p = lane; p < N; p += kWave) order[p] = clampi(pi[p], 0, N - 1);
        __builtin_amdgcn_wave_barrier();
        int worst = 0;
        for (int shift = 0; shift < 2; ++shift) {
            for (int p = lane; p < N; p += kWave) {
                int lo = 0, hi = N - 1, m = (N - 1) >> 1, acc = 0;
                int at = m + shift;
                int prev = order[at >= N ? at - N : at];
                for (int depth = 0; depth < 11 && m != p; ++depth) {
                    if (p < m) hi = m - 1;
                    else lo = m + 1;
                    m = (lo + hi) >> 1;
                    at = m + shift;
                    const int cur = order[at >= N ? at - N : at];
                    acc += mat[prev * N + cur];
                    prev = cur;
                }
                worst = max(worst, acc);
            }
        }
        const int total = wave_max(worst);
        __builtin_amdgcn_wave_barrier();
        if (lane == 0) out[b] = total;
    }
}

// N = 64: the tree's shape does not depend on the order, so every lane (tree position) finds its parent once, by
// the same binary search, and the positions 2 and 4 levels up by two look-ups.  Per order a lane gathers the one
// edge into its position for each of the two trees; path costs are then sums over ancestors, formed by pointer
// jumping in three lane-permute steps (the root's edge is 0 and it is its own ancestor, so chains that have reached
// the root add nothing).
__global__ __launch_bounds__(256) void dbt_batch_n64_kernel(const int32_t* __restrict__ c,
                                                            const int32_t* __restrict__ perms, int64_t B,
                                                            int64_t* __restrict__ out) {
    constexpr int N = 64;
    __shared__ int32_t m[N * N];
    __shared__ int32_t order_all[4][N];
    for (int e = threadIdx.x; e < N * N; e += 256) m[e] = c[e];
    const int lane = lane_id();
    int32_t* order = order_all[threadIdx.x >> 6];
    // parent of tree position `lane`
    int parent = lane;
    {
        int lo = 0, hi = N - 1, mid = (N - 1) >> 1;
        for (int depth = 0; depth < 7 && mid != lane; ++depth) {
            parent = mid;
            if (lane < mid) hi = mid - 1;
            else lo = mid + 1;
            mid = (lo + hi) >> 1;
        }
    }
    const bool is_root = parent == lane;
    order[lane] = parent;                                  // borrowed for the ancestor look-ups
    __builtin_amdgcn_wave_barrier();
    const int up2 = order[parent];
    const int up4 = order[order[up2]];
    __builtin_amdgcn_wave_barrier();
    __syncthreads();                                       // the matrix is staged
    const int from1 = parent << 2, from2 = up2 << 2, from4 = up4 << 2;
    const int parent_shifted = (parent + 1) & (N - 1);     // second tree: position q holds rank q + 1
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    int next = wave < B ? perms[wave * N + lane] : 0;
    for (int64_t b = wave; b < B; b += nwaves) {
        const int a = clampi(next, 0, N - 1);
        const int64_t bn = b + nwaves;
        next = bn < B ? perms[bn * N + lane] : 0;
        order[lane] = a;
        __builtin_amdgcn_wave_barrier();
        // node at tree position `lane` of the second tree: the next lane's (cyclic over the 64 lanes)
        const int a_shifted = __builtin_amdgcn_update_dpp(a, a, 0x134, 0xf, 0xf, true);
        int cost0 = is_root ? 0 : m[order[parent] * N + a];
        int cost1 = is_root ? 0 : m[order[parent_shifted] * N + a_shifted];
        __builtin_amdgcn_wave_barrier();                   // all look-ups done before the slice is overwritten
        cost0 += __builtin_amdgcn_ds_bpermute(from1, cost0);
        cost1 += __builtin_amdgcn_ds_bpermute(from1, cost1);
        cost0 += __builtin_amdgcn_ds_bpermute(from2, cost0);
        cost1 += __builtin_amdgcn_ds_bpermute(from2, cost1);
        cost0 += __builtin_amdgcn_ds_bpermute(from4, cost0);
        cost1 += __builtin_amdgcn_ds_bpermute(from4, cost1);
        const int total = wave_max(max(cost0, cost1));
        if (lane == 0) out[b] = total;
    }
}

hipError_t launch_dbt_cost_batch(const int32_t* c, int N, const int32_t* perms, int64_t B, int64_t* out,
                                 hipStream_t s) {
    if (B == 0) return hipSuccess;
    const int grid = batch_grid(4, B);
    if (N == 64 && ((uintptr_t)perms & 15u) == 0) {
        hipLaunchKernelGGL(dbt_lanes64_kernel, dim3(batch_grid(4 * 64, B)), dim3(256), 0, s, c, (const int4*)perms, B, out);
    } else if (N == 64) {
        hipLaunchKernelGGL(dbt_batch_n64_kernel, dim3(grid), dim3(256), 0, s, c, perms, B, out);
    } else if (N <= 64) {
        const size_t lds = sizeof(int32_t) * (size_t)(4 * N + N * N);
        hipLaunchKernelGGL((dbt_batch_kernel<true>), dim3(grid), dim3(256), lds, s, c, N, perms, B, out);
    } else {
        const size_t lds = sizeof(int32_t) * (size_t)(4 * N);
        hipLaunchKernelGGL((dbt_batch_kernel<false>), dim3(grid), dim3(256), lds, s, c, N, perms, B, out);
    }
    return hipGetLastError();
}

// --------------------------------------------------------------------------------- initial orders
// One wave per order.  N <= 64: no serial chain - lane v follows node v through the shuffle: at step k (k = N-1 .. 1)
// ranks k and j_k swap, so a node sitting at rank k moves to j_k and a node sitting at j_k moves to k, where it
// stays (later steps only touch ranks below k); the partners j_k are drawn in parallel, one per lane, and read
// step by step; each lane finally stores its node at the rank where it ended.  N <= 256: the same with up to four
// nodes per lane and the partners read from LDS (one broadcast read per step).  Larger N: the partners are drawn in
// parallel, lane 0 replays the swaps in order in LDS, all lanes store the result coalesced.
__global__ __launch_bounds__(256) void init_tours_kernel(int N, int64_t first, int64_t count, uint64_t seed,
                                                         int32_t* __restrict__ tours) {
    extern __shared__ int32_t sm[];
    int32_t* t = sm + (threadIdx.x >> 6) * 2 * N;
    int32_t* partner = t + N;
    const int lane = lane_id();
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t w = wave; w < count; w += nwaves) {
        const uint32_t r = (uint32_t)(first + w);
        if (N <= kWave) {
            const int mine = (lane > 0 && lane < N) ? shuffle_partner(seed, r, lane) : 0;
            int pos = lane;
            for (int k = N - 1; k >= 1; --k) {
                const int j = __builtin_amdgcn_readlane(mine, k);
                const int moved = (pos == k) ? j : pos;
                pos = (pos == j) ? k : moved;
            }
            if (lane < N) tours[w * N + pos] = lane;
            continue;
        }
        for (int k = lane; k < N; k += kWave) {
            t[k] = k;
            partner[k] = k ? shuffle_partner(seed, r, k) : 0;
        }
        __builtin_amdgcn_wave_barrier();
        if (N <= 4 * kWave) {
            int pos[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) pos[i] = lane + kWave * i;       // node ids; those >= N never match a rank
            for (int k = N - 1; k >= 1; --k) {
                const int j = partner[k];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int moved = (pos[i] == k) ? j : pos[i];
                    pos[i] = (pos[i] == j) ? k : moved;
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (lane + kWave * i < N) tours[w * N + pos[i]] = lane + kWave * i;
            __builtin_amdgcn_wave_barrier();
            continue;
        }
        if (lane == 0) {
            for (int k = N - 1; k >= 1; --k) {
                const int j = partner[k];
                const int tk = t[k], tj = t[j];
                t[k] = tj;
                t[j] = tk;
            }
        }
        __builtin_amdgcn_wave_barrier();
        for (int k = lane; k < N; k += kWave) tours[w * N + k] = t[k];
        __builtin_amdgcn_wave_barrier();
    }
}

hipError_t launch_init_tours(int N, int64_t first, int64_t count, uint64_t seed, int32_t* tours, hipStream_t s) {
    if (count == 0) return hipSuccess;
    const int grid = batch_grid(4, count);
    hipLaunchKernelGGL(init_tours_kernel, dim3(grid), dim3(256), sizeof(int32_t) * 8 * (size_t)N, s, N, first, count,
                       seed, tours);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------ matrix contract
// flags[0] bit 0: an entry outside [0, 2^21 - 1]; bit 1: c[a][b] != c[b][a] somewhere.
__global__ __launch_bounds__(256) void validate_kernel(const int32_t* __restrict__ c, int N, int require_symmetric,
                                                       int32_t* __restrict__ flags) {
    int bad = 0;
    const int64_t total = (int64_t)N * N;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        const int v = c[e];
        if (v < 0 || v > (1 << 21) - 1) bad |= 1;
        if (require_symmetric) {
            const int a = (int)(e / N), b = (int)(e % N);
            if (c[(int64_t)b * N + a] != v) bad |= 2;
        }
    }
    if (bad) atomicOr(flags, bad);
}

hipError_t launch_validate(const int32_t* c, int N, bool require_symmetric, int32_t* flags, hipStream_t s) {
    const int64_t total = (int64_t)N * N;
    int grid = (int)((total + 255) / 256);
    if (grid > 1024) grid = 1024;
    hipLaunchKernelGGL(validate_kernel, dim3(grid), dim3(256), 0, s, c, N, require_symmetric ? 1 : 0, flags);
    return hipGetLastError();
}

}  // namespace cc
