// Host-side launch functions behind the C ABI (one per kernel family).  Each validates nothing:
// the ABI layer has already checked shapes, pointers and limits.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cc {

// Environment pin for A/B profiling and for parity tests of the fallback kernels: with CC_FORCE_PATH=general every
// search call (2-opt, wider move sets, pair swaps) runs its general kernel - one workgroup per restart, every
// objective, any N - instead of the kernel specialised for its size and value range.  Read at every call; results are
// the same bit for bit, only the time differs.
bool force_general_path();

hipError_t launch_ring_cost_batch(const int32_t* c, int N, bool is_max, const int32_t* perms, int64_t B,
                                  int64_t* out, hipStream_t s);
hipError_t launch_ring_cost_batch_u8(const int32_t* c, int N, bool is_max, const uint8_t* perms, int64_t B,
                                     int64_t* out, hipStream_t s);
hipError_t launch_ring_cost_batch_u16(const int32_t* c, int N, bool is_max, const uint16_t* perms, int64_t B,
                                      int64_t* out, hipStream_t s);
// weights: device int32 [rounds] or nullptr (every round weighs 1)
hipError_t launch_rd_cost_batch(const int32_t* c, int N, const int32_t* weights, const int32_t* perms, int64_t B,
                                int64_t* out, hipStream_t s, int32_t* flags = nullptr, uint16_t* folded = nullptr);
// folded[x][y] = max(c[x][y], c[y][x]) as 16-bit entries, N * N of them; does nothing when flags[0] (the matrix
// maximum, launch_matrix_max) is 2^16 or more.
hipError_t launch_fold_to_u16(const int32_t* c, int N, uint16_t* folded, const int32_t* flags, hipStream_t s);
hipError_t launch_bcube_cost_batch(const int32_t* c, int N, int base, const int32_t* weights, const int32_t* perms,
                                   int64_t B, int64_t* out, hipStream_t s, int32_t* flags = nullptr,
                                   uint16_t* folded = nullptr);
hipError_t launch_dbt_cost_batch(const int32_t* c, int N, const int32_t* perms, int64_t B, int64_t* out,
                                 hipStream_t s);
hipError_t launch_probes_percentile(const int32_t* samples, int N, int K, int rank, bool symmetrize, int32_t* out,
                                    hipStream_t s);
hipError_t launch_sa_ring(const int32_t* c, int N, int chains, long long steps, int t_start, int t_end, uint64_t seed,
                          bool generate, int32_t* tours, int64_t* costs, int32_t* accepted, hipStream_t s);
hipError_t launch_sa_rd(const int32_t* c, int N, int chains, long long steps, int t_start, int t_end, uint64_t seed,
                        bool generate, int32_t* tours, int64_t* costs, int32_t* accepted, hipStream_t s);
hipError_t launch_init_tours(int N, int64_t first, int64_t count, uint64_t seed, int32_t* tours, hipStream_t s);
hipError_t launch_validate(const int32_t* c, int N, bool require_symmetric, int32_t* flags, hipStream_t s);

// 2-opt descent of `restarts` tours, then the lexicographic minimum over (cost, restart).
// `tours` ([restarts, N]) receives the final tours; if `tours_hold_init` it holds the initial tours on
// entry, otherwise restart r starts from the seeded shuffle (seed, r).  `flags` is a small int32
// device scratch area (>= 64 B); `mat16` has room for N*N 16-bit entries when N > 256.
// `classes` is the set of move classes (cc.h, CC_MOVES_*): 2-opt alone takes the specialised kernels.
constexpr int kMoves2opt = 1, kMovesOropt = 2, kMovesFlip = 4;
hipError_t launch_2opt(const int32_t* c, int N, int objective, int classes, int restarts, uint64_t seed,
                       bool tours_hold_init, int32_t* tours, int64_t* costs, int32_t* moves, int32_t* flags,
                       uint16_t* mat16, int32_t* best_perm, int64_t* best_cost, int32_t* best_restart, hipStream_t s);

// Descent over segment insertions, with or without the 2-opt moves, ring-sum objective (cc_local.hip).  `tours`
// must hold the initial tours.
hipError_t launch_insertion_search(const int32_t* c, int N, bool with_2opt, int restarts, int32_t* tours,
                                   int64_t* costs, int32_t* moves, int32_t* flags, hipStream_t s);
// The same search for N = 64 and max(c) < 2^16, one wavefront per restart (cc_local_n64.hip); returns at once if
// flags[0] >= 2^16 (flags[0] = matrix maximum, launch_matrix_max).
// N = 128 / 192 / 256, several ranks per lane, 16-bit matrix in LDS (cc_local_multi.hip); same flags convention.
hipError_t launch_local_multi(const int32_t* c, int N, bool with_2opt, int restarts, int32_t* tours, int64_t* costs,
                              int32_t* moves, const int32_t* flags, hipStream_t s);
hipError_t launch_local_n64(const int32_t* c, bool with_2opt, int restarts, int32_t* tours, int64_t* costs,
                            int32_t* moves, const int32_t* flags, hipStream_t s);

// N = 64, ring-sum objective: one wavefront per restart (cc_2opt_n64.hip).
hipError_t launch_2opt_sum_n64(const int32_t* c, int restarts, uint64_t seed, bool generate, int32_t* tours,
                               int64_t* costs, int32_t* moves, hipStream_t s);

// N = 64, max-hop objective, directed or undirected: one wavefront per restart (cc_2opt_n64_max.hip).
hipError_t launch_2opt_max_n64(const int32_t* c, int restarts, uint64_t seed, bool generate, bool with_flip, int32_t* tours,
                               int64_t* costs, int32_t* moves, hipStream_t s);

// N = 64, directed ring-sum objective, max(c) < 2^16: one wavefront per restart (cc_2opt_n64_dsum.hip); returns at once
// if flags[0] >= 2^16 (flags[0] = matrix maximum, launch_matrix_max).
hipError_t launch_2opt_dsum_n64(const int32_t* c, int restarts, uint64_t seed, bool generate, bool with_flip, int32_t* tours,
                                int64_t* costs, int32_t* moves, const int32_t* flags, hipStream_t s);

// N = 128 / 192 / 256, ring-sum objective, max(c) < 2^16: one wavefront per restart, 16-bit matrix in LDS
// (cc_2opt_multi.hip).  launch_matrix_max writes max(c) to flags[0]; the kernel returns at once if
// flags[0] >= 2^16.  `tours` must hold the initial tours.
hipError_t launch_matrix_max(const int32_t* c, int N, int32_t* flags, hipStream_t s);
// Any 4 <= N <= 256, ring-sum objective, max(c) < 2^16: one wavefront per restart, order and partner data in LDS
// (cc_2opt_multi.hip).  Same flags convention.
hipError_t launch_2opt_sum_flex(const int32_t* c, int N, int restarts, int32_t* tours, int64_t* costs, int32_t* moves,
                                const int32_t* flags, hipStream_t s);
hipError_t launch_2opt_sum_multi(const int32_t* c, int N, int restarts, int32_t* tours, int64_t* costs,
                                 int32_t* moves, const int32_t* flags, hipStream_t s);

// N = 128 / 192 / 256, max-hop objective (directed or not), max(c) < 2^16: one wavefront per restart, 16-bit matrix in
// LDS (cc_2opt_multi_max.hip).  Same flags convention.  `tours` must hold the initial tours.
hipError_t launch_2opt_max_multi(const int32_t* c, int N, bool directed, int restarts, bool with_flip, int32_t* tours,
                                 int64_t* costs, int32_t* moves, const int32_t* flags, hipStream_t s);

// N = 128 / 192 / 256, directed ring sum: one wavefront per restart, 16-bit matrix in LDS (cc_2opt_multi_dsum.hip).
// Runs when flags[0] (the matrix maximum) is below dsum_multi_limit(N), so that its 32-bit keys hold every partial
// delta; otherwise it returns at once and the general kernel, given the same limit, does the work.
__host__ __device__ constexpr int dsum_multi_limit(int N) { return (1 << 22) / (N + 2); }
hipError_t launch_2opt_dsum_multi(const int32_t* c, int N, int restarts, bool with_flip, int32_t* tours, int64_t* costs,
                                  int32_t* moves, const int32_t* flags, hipStream_t s);

// N = 512 or 1024, ring-sum objective, max(c) < 2^16: one workgroup of N/64 waves per restart, matrix rows
// streamed through LDS (cc_2opt_n1024.hip).  Same flags convention as above.
hipError_t launch_2opt_sum_n1024(const int32_t* c, int N, uint16_t* c16, int restarts, int32_t* tours, int64_t* costs,
                                 int32_t* moves, const int32_t* flags, hipStream_t s);

// Pair-swap descent under the halving-doubling model for `restarts` tours (cc_rdswap.hip); same tour
// convention as launch_2opt.  The best-of-restarts step is launch_best_restart.
// `mat16` has room for N*N 16-bit entries when N > 256 (the folded copy of the matrix).
hipError_t launch_rdswap(const int32_t* c, int N, int restarts, uint64_t seed, bool tours_hold_init, int32_t* tours,
                         int64_t* costs, int32_t* moves, int32_t* flags, uint16_t* mat16, hipStream_t s);
hipError_t launch_best_restart(const int64_t* costs, const int32_t* tours, int N, int restarts, int32_t* best_perm,
                               int64_t* best_cost, int32_t* best_restart, hipStream_t s);

}  // namespace cc
