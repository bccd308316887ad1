/*
 * cc.h -- C ABI of the rank-order search library for MI355X (gfx950).
 *
 * Problem (paper Section 4): N nodes, a measured N x N point-to-point cost matrix c, a collective
 * algorithm whose cost model is a function of the rank order; find a permutation of the node list
 * that minimises the model.  This library
 *   - evaluates the cost models of Section 4.1 (ring, halving-doubling, BCube, double binary tree) over
 *     batches of candidate orders;
 *   - runs many independent searches: best-improvement 2-opt over the ring, pair-swap descent under the
 *     halving-doubling model, and simulated annealing for both (Section 4.3);
 *   - builds the cost matrix from latency probes (Section 4.2).
 *
 * Conventions
 *   - Every buffer pointer is a DEVICE pointer owned by the caller unless stated otherwise.  The
 *     library never frees or keeps caller memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue work on
 *     it and return; results are valid once the caller has synchronised the stream.  Only
 *     cc_validate_matrix synchronises by itself.
 *   - cost_matrix: row-major int32 [N, N]; cost_matrix[a*N + b] = cost of node a talking to node b
 *     (the flattened c'_{iN+j} of Section 4.3).  Entries must satisfy 0 <= c <= CC_COST_MAX.
 *   - A rank order ("perm", "tour") is int32 [N]; perm[p] = original node placed at rank p (the r_p of
 *     Section 4.3).  The reordered node list is new_list[p] = old_list[perm[p]].
 *   - Return value: CC_OK (0) or a negative cc_status.  Argument errors are detected on the host
 *     before anything is launched.  Data errors (entries out of range, indices out of range, an
 *     asymmetric matrix given to an undirected objective) are not detected by the compute calls:
 *     results are then unspecified, but all memory accesses stay inside the caller's buffers
 *     (indices and entries are clamped) and every call ends: the ring-sum searches read the matrix
 *     through its upper triangle (entry (min(a,b), max(a,b)) for the pair a, b), so their move
 *     values are exact for the matrix they see; the max-hop and directed searches score true costs
 *     of the orders they produce; the annealing calls run a fixed number of steps.
 *     cc_validate_matrix checks the matrix contract.
 *   - All arithmetic is exact integer; costs are returned as int64.
 *   - Kernel choice never changes a result.  Each search call picks, from N, the objective and the size of
 *     the matrix entries, either a kernel specialised for that case or a general kernel that serves every
 *     case.  The environment variable CC_FORCE_PATH=general (read at every call) pins the general kernels:
 *     for comparing the two on the same input, nothing else.
 *   - CC_LDS_POISON=1 in the environment (a debugging aid, read at every call) makes every call first fill the
 *     on-chip shared memory of all compute units with 0x7f bytes, so that a kernel reading shared memory it has
 *     not written cannot pass a test on what an earlier launch left there.  Costs one extra launch per call.
 */
#ifndef CC_H_
#define CC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CC_MAX_N 1024
#define CC_COST_MAX ((1 << 21) - 1)
#define CC_SA_MAX_STEPS (1 << 24)
#define CC_MAX_PROBES 16384
#define CC_STATIC_SCRATCH_BYTES (8u << 20)

typedef enum {
    CC_OK = 0,
    CC_ERR_INVALID_ARG = -1,     /* null required pointer, negative count, bad objective, misaligned pointer */
    CC_ERR_UNSUPPORTED_N = -2,   /* N < 2, N > CC_MAX_N, or (halving-doubling) N not a power of two */
    CC_ERR_WORKSPACE = -3,       /* workspace missing or smaller than cc_2opt_workspace_bytes() */
    CC_ERR_HIP = -4,             /* a HIP runtime call failed; see cc_last_hip_error() */
    CC_ERR_NOT_SYMMETRIC = -5,   /* cc_validate_matrix: matrix is not symmetric */
    CC_ERR_COST_RANGE = -6,      /* cc_validate_matrix: an entry is outside [0, CC_COST_MAX] */
    CC_ERR_SCRATCH_LIMIT = -7    /* cc_2opt_search_noalloc: the search needs more than CC_STATIC_SCRATCH_BYTES */
} cc_status;

/* Objectives over the ring (Section 4.1, ring model).  SUM is the paper's sum of hop costs; MAX is
 * the largest hop (the bottleneck transfer on the critical path, Sections 5.3 and 6).  The DIRECTED
 * variants make the local search score every move for both walking directions of the resulting
 * ring, for matrices with c[a][b] != c[b][a]. */
typedef enum {
    CC_RING_SUM = 0,
    CC_RING_MAX = 1,
    CC_RING_SUM_DIRECTED = 2,
    CC_RING_MAX_DIRECTED = 3
} cc_objective;

/* Move classes of the ring search (a bitmask; cc_local_search). */
typedef enum {
    CC_MOVES_2OPT = 1,           /* reversal of a sub-array: the move set of cc_2opt_search */
    CC_MOVES_OROPT = 2,          /* a segment of 1 to 3 ranks taken out and put back elsewhere, kept or reversed */
    CC_MOVES_FLIP = 4            /* the whole ring walked the other way (directed objectives) */
} cc_move_class;

/*
 * Ring cost model (Section 4.1, equation C_r): for each of the B orders,
 *     out_costs[b] = sum over ranks p of c[perm_b[p]][perm_b[(p-1) mod N]]      (objective SUM)
 *     out_costs[b] = max over ranks p of the same hops                          (objective MAX)
 * The DIRECTED bit of `objective` is ignored (evaluation is always directional).
 * perms: int32 [B, N] row-major; out_costs: int64 [B].  2 <= N <= CC_MAX_N.  B = 0 is a no-op.
 */
int cc_ring_cost_batch(const int32_t* cost_matrix, int32_t N, int32_t objective, const int32_t* perms,
                       int64_t B, int64_t* out_costs, void* stream);

/*
 * The same with the orders stored one byte per rank (perms: uint8 [B, N] row-major, N <= 256, else
 * CC_ERR_UNSUPPORTED_N): the order stream is what this call reads from HBM, and this form reads a quarter of it.
 */
int cc_ring_cost_batch_u8(const int32_t* cost_matrix, int32_t N, int32_t objective, const uint8_t* perms, int64_t B,
                          int64_t* out_costs, void* stream);

/*
 * The same with two bytes per rank (perms: uint16 [B, N] row-major, any N up to CC_MAX_N): half the order stream of
 * cc_ring_cost_batch, for the sizes whose ranks do not fit a byte.
 */
int cc_ring_cost_batch_u16(const int32_t* cost_matrix, int32_t N, int32_t objective, const uint16_t* perms, int64_t B,
                           int64_t* out_costs, void* stream);

/*
 * Halving-doubling (recursive-doubling) cost model (Section 4.1, equation C_hd, with every round
 * weighted equally as in the latency-only view of Section 4.2):
 *     out_costs[b] = sum over k in [0, log2 N) of  max over ranks i of c[perm_b[i]][perm_b[i xor 2^k]]
 * N must be a power of two (Section 4.1 assumes it), 2 <= N <= CC_MAX_N.
 */
int cc_rd_cost_batch(const int32_t* cost_matrix, int32_t N, const int32_t* perms, int64_t B,
                     int64_t* out_costs, void* stream);

/*
 * cc_rd_cost_batch with caller-provided workspace: the same costs, faster for N >= 128.  A link of round k, the two
 * ranks i and i xor 2^k, contributes max(c[x][y], c[y][x]) of its two nodes to the round's maximum; with every entry
 * below 2^16 (decided on the device) the call first writes that larger value for every pair of nodes into the
 * workspace as 16-bit entries, and then scores a link by one look-up instead of one per end.  Other matrices, and
 * N < 128, are scored as by cc_rd_cost_batch.
 *   workspace  device memory, 256-byte aligned, at least cc_rd_batch_workspace_bytes(N) bytes (else
 *              CC_ERR_WORKSPACE); owned by the caller, contents undefined afterwards; calls that overlap in time
 *              need workspaces of their own.
 * Enqueues kernels only (no allocation, no memset).
 */
int cc_rd_cost_batch_ex(const int32_t* cost_matrix, int32_t N, const int32_t* perms, int64_t B, int64_t* out_costs,
                        void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace cc_rd_cost_batch_ex and cc_bcube_cost_batch_ex need for a matrix of N x N, 2 <= N <= CC_MAX_N
 * (0 for any other N): 256 + 2 N^2, rounded up to a multiple of 256. Host-only computation. */
size_t cc_rd_batch_workspace_bytes(int32_t N);

/*
 * BCube cost model (Section 4.1, equation C_b; Section 2.2 for the peering pattern): ranks are
 * numbered in base `base`; in round i every rank exchanges with the base-1 ranks whose number differs
 * from its own in digit i only (the printed peer index j + k*base^i is taken modulo `base` within
 * that digit); a round costs its slowest exchange and the rounds add up:
 *     out_costs[b] = sum over digits i of  max over ranks j, k in [1, base) of c[perm_b[j]][perm_b[peer(j, i, k)]]
 * N must be a power of `base` (else CC_ERR_UNSUPPORTED_N), base >= 2, 2 <= N <= CC_MAX_N.  base = 2 is
 * the halving-doubling model.  perms, out_costs, B as for cc_rd_cost_batch.
 */
int cc_bcube_cost_batch(const int32_t* cost_matrix, int32_t N, int32_t base, const int32_t* perms, int64_t B,
                        int64_t* out_costs, void* stream);

/*
 * The same with size-weighted rounds (Section 4.1: round i of halving-doubling moves S / 2^(i+1) bytes, round
 * i of BCube S / base^(i+1)): with a per-byte cost matrix, round i costs round_weights[i] times its slowest
 * exchange.  round_weights: DEVICE int32 [log_base N], each in [0, 2^30] (values outside are clamped); all
 * ones gives cc_bcube_cost_batch.  base = 2 is halving-doubling with weighted rounds.
 */
int cc_bcube_cost_batch_weighted(const int32_t* cost_matrix, int32_t N, int32_t base, const int32_t* round_weights,
                                 const int32_t* perms, int64_t B, int64_t* out_costs, void* stream);

/*
 * cc_bcube_cost_batch / cc_bcube_cost_batch_weighted with caller-provided workspace: the same costs.  round_weights
 * may be NULL (every round weighs 1).  For base 2 with N >= 128, and for base 4 with N = 256 or 1024, the call
 * scores on a folded 16-bit copy of the matrix as cc_rd_cost_batch_ex does (an exchange between two ranks costs the
 * larger of the two directed entries, so each pair of a round needs one look-up); other cases are scored as by
 * cc_bcube_cost_batch.  workspace: as for cc_rd_cost_batch_ex, at least cc_rd_batch_workspace_bytes(N) bytes.
 * Enqueues kernels only.
 */
int cc_bcube_cost_batch_ex(const int32_t* cost_matrix, int32_t N, int32_t base, const int32_t* round_weights,
                           const int32_t* perms, int64_t B, int64_t* out_costs, void* workspace, size_t workspace_bytes,
                           void* stream);

/*
 * Double-binary-tree cost model (Section 4.1, equation C_dbt and its recursion T(i, j)): the ranks i .. j
 * form a subtree rooted at the middle rank m = floor((i+j)/2) whose children are the middle ranks of
 * i .. m-1 and m+1 .. j (the printed child indices are read as those middles); a tree costs its most
 * expensive root-to-leaf path, sum of c[perm[parent]][perm[child]] over the path's hops; the second tree is
 * the same shape with tree position p holding rank (p+1) mod N; out_costs[b] is the larger of the two
 * trees' costs.  2 <= N <= CC_MAX_N.  perms, out_costs, B as for cc_rd_cost_batch.
 */
int cc_dbt_cost_batch(const int32_t* cost_matrix, int32_t N, const int32_t* perms, int64_t B, int64_t* out_costs,
                      void* stream);

/*
 * Multi-start 2-opt search for a ring order (Section 4.3: stochastic neighbour search started from
 * random orders, neighbours obtained by permuting a sub-array; here the deterministic
 * best-improvement form).
 *
 *   Moves.  Rank 0 is an anchor.  Move (i, j, o), 1 <= i < j <= N-1, (i, j) != (1, N-1): reverse
 *   perm[i..j]; if o = 1 also reverse perm[1..N-1] (the same ring walked the other way).  Undirected
 *   objectives use o = 0 only.  Move id = i*N + j (undirected) or (i*N + j)*2 + o (directed).
 *   The value of a move is the objective of the order it produces.
 *   One restart.  Score every move; take the lexicographically smallest (value, id); if the value is
 *   strictly below the current cost apply the move and repeat, otherwise stop.
 *   Restarts.  Restart r starts from the Fisher-Yates shuffle of the identity driven by SplitMix64:
 *   for k = N-1 down to 1, u = high 32 bits of output number ((r << 32) | k) + 1 of the generator
 *   started at state `seed`, swap perm[k] with perm[(u * (k+1)) >> 32].
 *   Result.  The lexicographically smallest (final cost, r); best_perm (int32 [N]) receives that
 *   restart's final order as it stands, best_cost (int64 [1]) its cost.
 *
 * N < 4 has no moves: the result is restart 0's initial order.  Undirected objectives require a
 * symmetric matrix.  This call allocates its workspace from the stream-ordered device allocator.
 */
int cc_2opt_search(const int32_t* cost_matrix, int32_t N, int32_t objective, int32_t restarts, uint64_t seed,
                   int32_t* best_perm, int64_t* best_cost, void* stream);

/*
 * The same search with caller-provided workspace and optional extra outputs.
 *   init_tours     int32 [restarts, N] or NULL.  NULL: generate from `seed` as above.
 *   best_restart   int32 [1] or NULL: index of the winning restart.
 *   restart_costs  int64 [restarts] or NULL: final cost of every restart.
 *   restart_tours  int32 [restarts, N] or NULL: final order of every restart.
 *   restart_moves  int32 [restarts] or NULL: number of moves each restart applied.
 *   workspace      device memory, 256-byte aligned, at least cc_2opt_workspace_bytes(N, objective,
 *                  restarts) bytes; contents on entry are irrelevant and on exit unspecified.
 * best_perm and best_cost are required, except that both may be NULL together: the call then stops after the
 * per-restart results (restart_costs and restart_tours are then required, best_restart must be NULL) and
 * cc_best_of_restarts can pick the winner later.
 */
int cc_2opt_search_ex(const int32_t* cost_matrix, int32_t N, int32_t objective, int32_t restarts,
                      uint64_t seed, const int32_t* init_tours, int32_t* best_perm, int64_t* best_cost,
                      int32_t* best_restart, int64_t* restart_costs, int32_t* restart_tours,
                      int32_t* restart_moves, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The ring search of cc_2opt_search over a wider move set (Section 4.3 searches with sub-array and pair permutations
 * "alongside standard heuristics"; the two classes added here are the usual companions of 2-opt).  One restart,
 * restarts and result exactly as in cc_2opt_search: every move of the enabled classes is scored, the
 * lexicographically smallest (value, id) is applied if it strictly lowers the cost.
 *
 *   CC_MOVES_2OPT   the moves (i, j, o) of cc_2opt_search with their ids.
 *   CC_MOVES_OROPT  segment insertion: the L in {1, 2, 3} consecutive ranks s .. s+L-1 (1 <= s, s+L-1 <= N-1,
 *                   L <= N-3) are taken out of the ring and put back, kept (o = 0) or reversed (o = 1, L > 1
 *                   only), between the nodes that stood at ranks g and (g+1) mod N, g outside s-1 .. s+L-1; all
 *                   other nodes keep their order and rank 0 keeps its node.
 *                   id = N*N + (variant*N + s)*N + g with variant 0 (L = 1), 1, 2 (L = 2: kept, reversed),
 *                   3, 4 (L = 3): above every 2-opt id, so a 2-opt move wins a tie.
 *   CC_MOVES_FLIP   the pair (i, j) = (1, N-1) that the 2-opt set leaves out, o = 0: reverse perm[1..N-1].
 *
 * Defined combinations: CC_MOVES_2OPT with every objective (then identical to cc_2opt_search);
 * CC_MOVES_OROPT and CC_MOVES_2OPT | CC_MOVES_OROPT with CC_RING_SUM (symmetric matrix);
 * CC_MOVES_2OPT | CC_MOVES_FLIP with the two directed objectives.  Anything else: CC_ERR_INVALID_ARG.
 * Arguments, outputs and workspace (cc_2opt_workspace_bytes) as for cc_2opt_search / cc_2opt_search_ex.
 */
int cc_local_search(const int32_t* cost_matrix, int32_t N, int32_t objective, int32_t move_classes, int32_t restarts,
                    uint64_t seed, int32_t* best_perm, int64_t* best_cost, void* stream);

int cc_local_search_ex(const int32_t* cost_matrix, int32_t N, int32_t objective, int32_t move_classes,
                       int32_t restarts, uint64_t seed, const int32_t* init_tours, int32_t* best_perm,
                       int64_t* best_cost, int32_t* best_restart, int64_t* restart_costs, int32_t* restart_tours,
                       int32_t* restart_moves, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Section 4.3 keeps the cheapest order its search has seen; with many independent descents that is the cheapest
 * final order, and this call is that selection, the last step of every search call, on its own (so that a caller can
 * time or capture the descents apart from it, or merge restarts from several calls): the lexicographically
 * smallest (restart_costs[r], r) over r in [0, restarts); best_perm (int32 [N]) receives restart_tours[r],
 * best_cost (int64 [1]) the cost, best_restart (int32 [1] or NULL) r.  restart_costs int64 [restarts], restart_tours int32 [restarts, N].
 */
int cc_best_of_restarts(const int64_t* restart_costs, const int32_t* restart_tours, int32_t N, int32_t restarts,
                        int32_t* best_perm, int64_t* best_cost, int32_t* best_restart, void* stream);

/* Bytes of workspace cc_2opt_search_ex needs (0 on invalid arguments). Host-only computation. */
size_t cc_2opt_workspace_bytes(int32_t N, int32_t objective, int32_t restarts);

/*
 * cc_2opt_search for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): same arguments, same result, but the per-restart costs, move counts
 * and orders (and the 16-bit matrix copy of N > 256) live in a static device array of CC_STATIC_SCRATCH_BYTES
 * (8 MiB) that every GPU the library runs on holds until the process ends.  The call allocates and frees nothing;
 * it only enqueues kernels on `stream`.
 *   Limit.  cc_2opt_workspace_bytes(N, objective, restarts) must not exceed CC_STATIC_SCRATCH_BYTES (for example
 *   N = 64 with up to 31,000 restarts, N = 256 with up to 8,000, N = 1024 with up to 1,500); otherwise the call
 *   returns CC_ERR_SCRATCH_LIMIT and launches nothing.
 *   Sharing.  All calls on one GPU use that GPU's one array, which keeps the previous call's contents (the search
 *   overwrites every part it reads, so nothing has to be cleared).  Two calls that overlap in time on one GPU -
 *   different streams, or different host threads - race on it; the caller serialises them.
 *   The device that is current when the call is made must be the device of `stream` and of the buffers.
 */
int cc_2opt_search_noalloc(const int32_t* cost_matrix, int32_t N, int32_t objective, int32_t restarts, uint64_t seed,
                           int32_t* best_perm, int64_t* best_cost, void* stream);

/*
 * Multi-start pair-swap search under the halving-doubling model (Section 4.3: neighbours obtained by
 * permuting a pair of ranks; Section 4.1 equation C_hd as evaluated by cc_rd_cost_batch).
 *
 *   Moves.  Move (p, q), 0 <= p < q <= N-1: exchange the nodes at ranks p and q.  Move id = p*N + q.
 *   The value of a move is the halving-doubling cost of the order it produces.  No rank is anchored.
 *   One restart, restarts, result: exactly as in cc_2opt_search (lexicographically smallest (value, id),
 *   applied only if strictly better; seeded Fisher-Yates starts; lexicographically smallest
 *   (final cost, restart) wins).
 *
 * N must be a power of two, 2 <= N <= CC_MAX_N.  Arguments, workspace and outputs as for
 * cc_2opt_search / cc_2opt_search_ex; the workspace size is cc_rd_swap_workspace_bytes(N, restarts).
 */
int cc_rd_swap_search(const int32_t* cost_matrix, int32_t N, int32_t restarts, uint64_t seed, int32_t* best_perm,
                      int64_t* best_cost, void* stream);

int cc_rd_swap_search_ex(const int32_t* cost_matrix, int32_t N, int32_t restarts, uint64_t seed,
                         const int32_t* init_tours, int32_t* best_perm, int64_t* best_cost, int32_t* best_restart,
                         int64_t* restart_costs, int32_t* restart_tours, int32_t* restart_moves, void* workspace,
                         size_t workspace_bytes, void* stream);

size_t cc_rd_swap_workspace_bytes(int32_t N, int32_t restarts);

/*
 * Simulated annealing over the ring, sum objective (Section 4.3: stochastic search by simulated
 * annealing, a neighbour obtained by permuting a random sub-array).  The paper fixes neither schedule
 * nor random numbers; this is an all-integer definition, so every implementation gives the same result.
 *
 *   Chain r starts from the seeded order of restart r (cc_2opt_search) or from init_tours[r].
 *   Step s = 0 .. steps-1 draws w = output number ((r << 32) | (1024 + s)) + 1 of the SplitMix64 generator
 *   started at state `seed`.
 *   Proposal: ring edges a = (w[63:43] * N) >> 21 and b = (a + d) mod N, d = 2 + ((w[42:22] * (N-3)) >> 21)
 *   (edge p joins ranks p-1 and p); exchanging them is the 2-opt move (i, j) = (lo, hi-1), or (hi, N-1) when
 *   lo = 0, lo = min(a, b), hi = max(a, b).  delta = cost after - cost before.
 *   Temperature: linear from t_start to t_end, num_s = t_start*(steps-s) + t_end*s (= T_s * steps).  T is the
 *   cost increase that is accepted with probability one half (Boltzmann factor 2^(-delta/T)).
 *   Acceptance: u = w[21:0] + 1; L = 4096*e + f, e = floor(log2 u), f = the 12 bits of u below its leading
 *   one (zero-padded); E = 22*4096 - L.  Accept iff delta <= 0 or delta * 4096 * steps <= num_s * E.
 *   Each chain reports the cheapest order it visited (the earliest such) and that cost; the result is the
 *   lexicographically smallest (cost, r).
 *
 * Requires a symmetric matrix.  0 <= steps <= CC_SA_MAX_STEPS, 0 <= t_start, t_end <= CC_COST_MAX,
 * chains >= 1 (else CC_ERR_INVALID_ARG).  N < 4 has no proposals.  cc_sa_search allocates its workspace
 * from the stream-ordered device allocator.  In cc_sa_search_ex: init_tours int32 [chains, N] or NULL;
 * best_chain int32 [1], chain_costs int64 [chains], chain_tours int32 [chains, N] (each chain's best
 * order), chain_accepted int32 [chains] (accepted proposals) may be NULL; workspace as in
 * cc_2opt_search_ex, at least cc_sa_workspace_bytes(N, chains) bytes.  The orders a search returns can be
 * passed to cc_2opt_search_ex as init_tours for a final descent.
 */
int cc_sa_search(const int32_t* cost_matrix, int32_t N, int32_t chains, int64_t steps, int32_t t_start, int32_t t_end,
                 uint64_t seed, int32_t* best_perm, int64_t* best_cost, void* stream);

int cc_sa_search_ex(const int32_t* cost_matrix, int32_t N, int32_t chains, int64_t steps, int32_t t_start,
                    int32_t t_end, uint64_t seed, const int32_t* init_tours, int32_t* best_perm, int64_t* best_cost,
                    int32_t* best_chain, int64_t* chain_costs, int32_t* chain_tours, int32_t* chain_accepted,
                    void* workspace, size_t workspace_bytes, void* stream);

size_t cc_sa_workspace_bytes(int32_t N, int32_t chains);

/*
 * Simulated annealing under the halving-doubling model with the pair neighbour (Section 4.3: permuting random
 * pairs; cost: Section 4.1 equation C_hd as evaluated by cc_rd_cost_batch).  Exactly cc_sa_search (same random word
 * per step, temperature, acceptance rule, report, limits, arguments, workspace) except for the proposal and the
 * cost: p = (w[63:43] * N) >> 21, q = (p + d) mod N with d = 1 + ((w[42:22] * (N-1)) >> 21); the move exchanges the
 * nodes at ranks p and q; delta = halving-doubling cost after - before.  No rank is anchored; the matrix need not
 * be symmetric.  N must be a power of two (else CC_ERR_UNSUPPORTED_N).
 */
int cc_sa_rd_search(const int32_t* cost_matrix, int32_t N, int32_t chains, int64_t steps, int32_t t_start,
                    int32_t t_end, uint64_t seed, int32_t* best_perm, int64_t* best_cost, void* stream);

int cc_sa_rd_search_ex(const int32_t* cost_matrix, int32_t N, int32_t chains, int64_t steps, int32_t t_start,
                       int32_t t_end, uint64_t seed, const int32_t* init_tours, int32_t* best_perm, int64_t* best_cost,
                       int32_t* best_chain, int64_t* chain_costs, int32_t* chain_tours, int32_t* chain_accepted,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * The random initial orders of Section 4.3's search (the provider's list arrives in random order, Section 1):
 * initial orders of restarts first .. first+count-1 for `seed` (the shuffle described above);
 * tours: int32 [count, N].  `first` lets a caller draw any slice of the restart sequence (one shard of a search
 * split over several calls draws its own restarts with their global ids).  Also the generator of the seeded
 * random orders used to exercise the batch calls.
 */
int cc_init_tours(int32_t N, int64_t first, int64_t count, uint64_t seed, int32_t* tours, void* stream);

/*
 * Cost matrix from latency probes (Section 4.2): cost_matrix[a][b] = the sample of rank
 * max(1, ceil(percentile * K / 100)) among the K samples of the ordered pair a -> b in ascending order (the
 * paper takes the 10th percentile to filter out interference); if symmetrize != 0 both directions then get
 * the larger of the two (c[a][b] <- MAX(c[a][b], c[b][a])).  The diagonal is not read and is set to 0.
 * samples: int32 [N, N, K], samples[(a*N + b)*K + s]; values are limited to [0, CC_COST_MAX].
 * 1 <= N <= CC_MAX_N, 1 <= K <= CC_MAX_PROBES, 0 <= percentile <= 100.  cost_matrix: int32 [N, N], written in
 * full; it satisfies the contract of every other call (symmetric if symmetrize != 0).
 */
int cc_cost_matrix_from_probes(const int32_t* samples, int32_t N, int32_t K, int32_t percentile, int32_t symmetrize,
                               int32_t* cost_matrix, void* stream);

/*
 * Checks the matrix contract that the other calls take on trust.  Section 4.2 makes the matrix symmetric
 * (c_ij <- MAX(c_ij, c_ji)) before the undirected models of Section 4.1 are applied to it, and this library
 * keeps costs in integer units with a fixed ceiling so that every sum over N <= CC_MAX_N hops fits 32 bits:
 * every entry in [0, CC_COST_MAX] (else CC_ERR_COST_RANGE), and, if require_symmetric != 0,
 * c[a][b] == c[b][a].  Synchronises `stream` and returns CC_OK, CC_ERR_COST_RANGE or
 * CC_ERR_NOT_SYMMETRIC.  Allocates and frees four bytes of device memory.
 */
int cc_validate_matrix(const int32_t* cost_matrix, int32_t N, int32_t require_symmetric, void* stream);

/* Static, human-readable text for a cc_status value (host pointer, never freed). */
const char* cc_status_string(int status);

/* hipError_t of the most recent failing HIP call made by this library on the calling thread (0 = none). */
int cc_last_hip_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int cc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CC_H_ */
