/*
 * CPU oracle for rank-order search on a measured point-to-point cost matrix.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, single-threaded C written from the paper's statement of
 * the problem (Section 4.1 cost models, Section 4.3 rank variables and neighbour search).  It shares
 * no code with the GPU library and must never be called from a product path: only the test-suite,
 * the smoke check and the benchmark's CPU-baseline leg load it.
 *
 * Notation (Section 4.1 / 4.3):
 *   N        number of ranks
 *   c        row-major N x N int32, c[a*N+b] = cost of node a talking to node b (flattened c'_{iN+j})
 *   t / pi   permutation array, t[p] = original node placed at rank p (the r_p of Section 4.3)
 *   prev(p)  (p - 1 + N) mod N   (ranks alias modulo N, Section 4.1)
 *
 * All arithmetic is exact 64-bit integer.
 *
 * Pins (see tests/test_oracle_*.py): closed forms for constant / additive / line-metric / cyclic
 * shift / clean-hierarchy matrices, rotation and reversal invariances, hypercube automorphisms,
 * brute force over all rings for N <= 10, every move's fast value against apply-and-recompute,
 * local-optimum certification, published SplitMix64 output vectors; for the pair-swap search under the
 * halving-doubling model: every swap's fast value against swap-and-recompute, replayed trajectories,
 * brute force over all 8! orders; for the BCube model: base 2 against the halving-doubling model, closed forms,
 * digit automorphisms; for the annealing chain: the acceptance rule against the Boltzmann factor, proposal
 * statistics, bookkeeping against recomputation, the Boltzmann distribution of a constant-temperature chain
 * over an enumerated state space; for segment insertion and the orientation flip: a list-operation model of the
 * move, every move's fast value against apply-and-recompute, the set of reachable tours by brute force, closed
 * forms on a circle metric and on a one-way ring, every step of a descent against a scan of the whole move set.
 * Parity unpinned: none of the functions below against their stated definitions.  The annealing schedule,
 * random-number use and acceptance rule are this project's own definition (the paper names the method only),
 * so there is nothing in the paper to pin those choices to.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { CCO_SUM = 0, CCO_MAX = 1, CCO_SUM_DIRECTED = 2, CCO_MAX_DIRECTED = 3 };
enum { CCO_OK = 0, CCO_ERR_ARG = -1, CCO_ERR_NOT_SYMMETRIC = -2, CCO_ERR_NOMEM = -3 };

#define C_(a, b) ((int64_t)c[(int64_t)(a) * N + (b)])

static int64_t max64(int64_t a, int64_t b) { return a > b ? a : b; }

/* ------------------------------------------------------------------------------------------------
 * Counter-based random numbers: SplitMix64 (Steele, Lea, Flood 2014; public-domain reference by
 * Vigna).  The generator's state advances by the golden-gamma constant and the output is a
 * two-round xor-shift-multiply finaliser of the state, so the n-th output (n = 1, 2, ...) of a
 * generator started at state `seed` is mix(seed + n * gamma) and can be computed directly.
 * ---------------------------------------------------------------------------------------------- */
uint64_t cco_splitmix64_at(uint64_t seed, uint64_t n)
{
    uint64_t z = seed + n * 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/* Initial tour of restart r: Fisher-Yates from the identity, k = N-1 down to 1, swap t[k] with
 * t[jdx], jdx = floor(u * (k+1) / 2^32) where u = high 32 bits of output number ((r<<32)|k)+1.
 * (The paper only says the initial order is random, Section 1; this fixes one reproducible draw.) */
void cco_init_tour(uint64_t seed, uint32_t r, int32_t N, int32_t *t)
{
    for (int32_t p = 0; p < N; ++p) t[p] = p;
    for (int32_t k = N - 1; k >= 1; --k) {
        uint64_t ctr = (((uint64_t)r << 32) | (uint64_t)(uint32_t)k) + 1u;
        uint64_t u = cco_splitmix64_at(seed, ctr) >> 32;
        int32_t jdx = (int32_t)((u * (uint64_t)(k + 1)) >> 32);
        int32_t tmp = t[k]; t[k] = t[jdx]; t[jdx] = tmp;
    }
}

void cco_init_tours(uint64_t seed, int32_t N, int64_t first, int64_t count, int32_t *tours)
{
    for (int64_t r = 0; r < count; ++r) cco_init_tour(seed, (uint32_t)(first + r), N, tours + r * N);
}

/* ------------------------------------------------------------------------------------------------
 * Cost models (Section 4.1).
 * ---------------------------------------------------------------------------------------------- */

/* Ring: sum over ranks p of the hop c[pi(p)][pi(p-1)] (the equation's c_{i,i-1}); objective MAX
 * takes the largest hop instead (bottleneck link on the critical path, Section 5.3 / Section 6). */
int64_t cco_ring_cost(const int32_t *c, int32_t N, const int32_t *pi, int32_t objective)
{
    int64_t acc = 0;
    for (int32_t p = 0; p < N; ++p) {
        int32_t pp = (p - 1 + N) % N;
        int64_t hop = C_(pi[p], pi[pp]);
        if (objective & 1) acc = (p == 0) ? hop : max64(acc, hop);
        else acc += hop;
    }
    return acc;
}

/* Halving-doubling / recursive doubling: one round per bit k of the rank id; a round costs the
 * slowest of its exchanges, rank i talking to rank i xor 2^k; rounds add up. */
int64_t cco_rd_cost(const int32_t *c, int32_t N, const int32_t *pi)
{
    int64_t total = 0;
    for (int32_t bit = 1; bit < N; bit <<= 1) {
        int64_t worst = 0;
        for (int32_t i = 0; i < N; ++i) worst = max64(worst, C_(pi[i], pi[i ^ bit]));
        total += worst;
    }
    return total;
}

int cco_ring_cost_batch(const int32_t *c, int32_t N, int32_t objective, const int32_t *perms, int64_t B,
                        int64_t *out)
{
    if (!c || N < 2 || B < 0 || (B > 0 && (!perms || !out))) return CCO_ERR_ARG;
    for (int64_t b = 0; b < B; ++b) out[b] = cco_ring_cost(c, N, perms + b * N, objective);
    return CCO_OK;
}

int cco_rd_cost_batch(const int32_t *c, int32_t N, const int32_t *perms, int64_t B, int64_t *out)
{
    if (!c || N < 2 || (N & (N - 1)) || B < 0 || (B > 0 && (!perms || !out))) return CCO_ERR_ARG;
    for (int64_t b = 0; b < B; ++b) out[b] = cco_rd_cost(c, N, perms + b * N);
    return CCO_OK;
}

/* ------------------------------------------------------------------------------------------------
 * 2-opt neighbourhood (the "permute a sub-array" neighbour of Section 4.3, made deterministic).
 * Rank 0 is an anchor.  Move (i, j, o): 1 <= i < j <= N-1, (i, j) != (1, N-1); reverse t[i..j];
 * if o = 1 additionally reverse t[1..N-1] (same ring walked the other way round).
 * Undirected objectives use o = 0 only.
 * ---------------------------------------------------------------------------------------------- */
static void reverse_span(int32_t *t, int32_t lo, int32_t hi)
{
    while (lo < hi) { int32_t tmp = t[lo]; t[lo] = t[hi]; t[hi] = tmp; ++lo; --hi; }
}

void cco_apply_move(int32_t *t, int32_t N, int32_t i, int32_t j, int32_t o)
{
    reverse_span(t, i, j);
    if (o) reverse_span(t, 1, N - 1);
}

int64_t cco_move_id(int32_t N, int32_t objective, int32_t i, int32_t j, int32_t o)
{
    int64_t id = (int64_t)i * N + j;
    return (objective & 2) ? id * 2 + o : id;
}

/* Definition tier: value of a move = objective of the tour obtained by applying it. */
int64_t cco_move_value_by_definition(const int32_t *c, int32_t N, int32_t objective, const int32_t *t,
                                     int32_t i, int32_t j, int32_t o)
{
    int32_t *u = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    memcpy(u, t, sizeof(int32_t) * (size_t)N);
    cco_apply_move(u, N, i, j, o);
    int64_t v = cco_ring_cost(c, N, u, objective);
    free(u);
    return v;
}

/* Delta tier: O(1) value per move from the hop arrays
 *   f[p] = c[t[p]][t[prev p]]  (hop as walked now),  b[p] = c[t[prev p]][t[p]]  (same edge, other way)
 * With q = (j+1) mod N, inside I = {i+1..j}, outside O = all ranks except I, i and q:
 *   reversing t[i..j] replaces hops i and q by x0 = c[t[j]][t[i-1]], y0 = c[t[q]][t[i]], and walks
 *   the inside edges the other way (b instead of f); orientation 1 flips every hop of that ring:
 *   x1 = c[t[i-1]][t[j]], y1 = c[t[i]][t[q]], outside b, inside f.
 * Scans all moves in increasing id and returns the lexicographic minimum of (value, id).
 * Returns 0 if the neighbourhood is empty (N < 4). */
typedef struct { int64_t value; int64_t id; int32_t i, j, o; } cco_best;

static int scan_moves(const int32_t *c, int32_t N, int32_t objective, const int32_t *t, int64_t cur,
                      int64_t *ws /* 6N int64 */, cco_best *best, int64_t *all_values /* optional */)
{
    const int directed = (objective & 2) != 0, is_max = (objective & 1) != 0;
    int64_t *f = ws, *b = ws + N, *pf = ws + 2 * N, *pb = ws + 3 * N, *sf = ws + 4 * N, *sb = ws + 5 * N;
    /* pf/pb: inclusive prefix (sum or max) over ranks 0..p; sf/sb: inclusive suffix over p..N-1 */
    int found = 0;
    int64_t nvals = 0;
    if (N < 4) return 0;
    for (int32_t p = 0; p < N; ++p) {
        int32_t pp = (p - 1 + N) % N;
        f[p] = C_(t[p], t[pp]);
        b[p] = C_(t[pp], t[p]);
    }
    for (int32_t p = 0; p < N; ++p) {
        if (is_max) { pf[p] = p ? max64(pf[p - 1], f[p]) : f[p]; pb[p] = p ? max64(pb[p - 1], b[p]) : b[p]; }
        else        { pf[p] = (p ? pf[p - 1] : 0) + f[p];          pb[p] = (p ? pb[p - 1] : 0) + b[p]; }
    }
    for (int32_t p = N - 1; p >= 0; --p) {
        if (is_max) { sf[p] = p < N - 1 ? max64(sf[p + 1], f[p]) : f[p]; sb[p] = p < N - 1 ? max64(sb[p + 1], b[p]) : b[p]; }
        else        { sf[p] = (p < N - 1 ? sf[p + 1] : 0) + f[p];          sb[p] = (p < N - 1 ? sb[p + 1] : 0) + b[p]; }
    }
    for (int32_t i = 1; i <= N - 2; ++i) {
        int64_t in_f = 0, in_b = 0;              /* sum or max of f / b over I, grown as j advances */
        for (int32_t j = i + 1; j <= N - 1; ++j) {
            int32_t q = (j + 1) % N;
            if (is_max) { in_f = max64(in_f, f[j]); in_b = max64(in_b, b[j]); }
            else        { in_f += f[j];              in_b += b[j]; }
            if (i == 1 && j == N - 1) continue;
            int64_t x0 = C_(t[j], t[i - 1]), y0 = C_(t[q], t[i]);
            int64_t x1 = C_(t[i - 1], t[j]), y1 = C_(t[i], t[q]);
            int64_t v0, v1 = 0;
            if (!is_max) {
                if (!directed) {
                    v0 = cur + x0 + y0 - f[i] - f[q];
                } else {
                    int64_t out_f = pf[N - 1] - f[i] - f[q] - in_f;
                    int64_t out_b = pb[N - 1] - b[i] - b[q] - in_b;
                    v0 = x0 + y0 + out_f + in_b;
                    v1 = x1 + y1 + out_b + in_f;
                }
            } else {
                /* outside = ranks 0..i-1 and j+2..N-1 (empty when q = 0 wraps: then rank 0 is q itself
                 * and the prefix must skip it) */
                int64_t out_f = 0, out_b = 0;
                if (q == 0) {
                    /* ranks 1..i-1 */
                    for (int32_t p = 1; p <= i - 1; ++p) { out_f = max64(out_f, f[p]); out_b = max64(out_b, b[p]); }
                } else {
                    out_f = pf[i - 1]; out_b = pb[i - 1];
                    if (j + 2 <= N - 1) { out_f = max64(out_f, sf[j + 2]); out_b = max64(out_b, sb[j + 2]); }
                }
                v0 = max64(max64(x0, y0), max64(out_f, in_b));
                v1 = max64(max64(x1, y1), max64(out_b, in_f));
            }
            for (int32_t o = 0; o <= directed; ++o) {
                int64_t v = o ? v1 : v0;
                int64_t id = cco_move_id(N, objective, i, j, o);
                if (all_values) all_values[nvals] = v;
                ++nvals;
                if (!found || v < best->value || (v == best->value && id < best->id)) {
                    best->value = v; best->id = id; best->i = i; best->j = j; best->o = o;
                    found = 1;
                }
            }
        }
    }
    return found;
}

/* Number of moves in the neighbourhood: N(N-3)/2 undirected, N(N-3) directed. */
int64_t cco_neighbourhood_size(int32_t N, int32_t objective)
{
    if (N < 4) return 0;
    int64_t m = (int64_t)N * (N - 3) / 2;
    return (objective & 2) ? 2 * m : m;
}

/* Values of every move in increasing id order (delta tier), for checking against the definition. */
int cco_all_move_values(const int32_t *c, int32_t N, int32_t objective, const int32_t *t, int64_t *values)
{
    int64_t *ws = (int64_t *)malloc(sizeof(int64_t) * 6 * (size_t)N);
    if (!ws) return CCO_ERR_NOMEM;
    cco_best best;
    scan_moves(c, N, objective, t, cco_ring_cost(c, N, t, objective), ws, &best, values);
    free(ws);
    return CCO_OK;
}

static int is_symmetric(const int32_t *c, int32_t N)
{
    for (int32_t a = 0; a < N; ++a)
        for (int32_t b2 = a + 1; b2 < N; ++b2)
            if (c[(int64_t)a * N + b2] != c[(int64_t)b2 * N + a]) return 0;
    return 1;
}

/* One best-improvement descent: score the whole neighbourhood, take the lexicographically smallest
 * (value, id); apply it if it strictly lowers the cost, else stop.  `use_definition` scores every
 * move by apply-and-recompute instead of the delta formulas (tests compare the two trajectories).
 * trace (optional, capacity trace_cap): ids of the applied moves. */
int cco_2opt_descend(const int32_t *c, int32_t N, int32_t objective, int32_t *t, int64_t *cost,
                     int32_t *moves, int32_t use_definition, int64_t *trace, int32_t trace_cap)
{
    if (!c || !t || N < 2 || objective < 0 || objective > 3) return CCO_ERR_ARG;
    int64_t *ws = (int64_t *)malloc(sizeof(int64_t) * 6 * (size_t)N);
    if (!ws) return CCO_ERR_NOMEM;
    const int directed = (objective & 2) != 0;
    int64_t cur = cco_ring_cost(c, N, t, objective);
    int32_t applied = 0;
    for (;;) {
        cco_best best;
        int found;
        if (!use_definition) {
            found = scan_moves(c, N, objective, t, cur, ws, &best, NULL);
        } else {
            found = 0;
            for (int32_t i = 1; i <= N - 2; ++i)
                for (int32_t j = i + 1; j <= N - 1; ++j) {
                    if (i == 1 && j == N - 1) continue;
                    for (int32_t o = 0; o <= directed; ++o) {
                        int64_t v = cco_move_value_by_definition(c, N, objective, t, i, j, o);
                        int64_t id = cco_move_id(N, objective, i, j, o);
                        if (!found || v < best.value || (v == best.value && id < best.id)) {
                            best.value = v; best.id = id; best.i = i; best.j = j; best.o = o; found = 1;
                        }
                    }
                }
        }
        if (!found || best.value >= cur) break;
        cco_apply_move(t, N, best.i, best.j, best.o);
        cur = best.value;
        if (trace && applied < trace_cap) trace[applied] = best.id;
        ++applied;
    }
    free(ws);
    *cost = cur;
    if (moves) *moves = applied;
    return CCO_OK;
}

/* Restarts [r0, r1) of a multi-start search.  Per-restart outputs are indexed by r - r0.
 * init_tours (optional, [restarts_total, N], indexed by r) overrides the seeded shuffle.
 * Undirected objectives require a symmetric matrix. */
int cco_2opt_restarts(const int32_t *c, int32_t N, int32_t objective, uint64_t seed, int64_t r0, int64_t r1,
                      const int32_t *init_tours, int64_t *restart_costs, int32_t *restart_tours,
                      int32_t *restart_moves)
{
    if (!c || N < 2 || objective < 0 || objective > 3 || r0 < 0 || r1 < r0) return CCO_ERR_ARG;
    if (!(objective & 2) && !is_symmetric(c, N)) return CCO_ERR_NOT_SYMMETRIC;
    int32_t *t = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    if (!t) return CCO_ERR_NOMEM;
    for (int64_t r = r0; r < r1; ++r) {
        if (init_tours) memcpy(t, init_tours + r * N, sizeof(int32_t) * (size_t)N);
        else cco_init_tour(seed, (uint32_t)r, N, t);
        int64_t cost; int32_t mv;
        int rc = cco_2opt_descend(c, N, objective, t, &cost, &mv, 0, NULL, 0);
        if (rc != CCO_OK) { free(t); return rc; }
        if (restart_costs) restart_costs[r - r0] = cost;
        if (restart_moves) restart_moves[r - r0] = mv;
        if (restart_tours) memcpy(restart_tours + (r - r0) * N, t, sizeof(int32_t) * (size_t)N);
    }
    free(t);
    return CCO_OK;
}

/* Whole search: all restarts, then the lexicographic minimum of (final cost, restart id). */
int cco_2opt_search(const int32_t *c, int32_t N, int32_t objective, int32_t restarts, uint64_t seed,
                    const int32_t *init_tours, int32_t *best_perm, int64_t *best_cost, int32_t *best_restart,
                    int64_t *restart_costs, int32_t *restart_tours, int32_t *restart_moves)
{
    if (restarts < 1 || !best_perm || !best_cost) return CCO_ERR_ARG;
    int64_t *costs = restart_costs ? restart_costs : (int64_t *)malloc(sizeof(int64_t) * (size_t)restarts);
    int32_t *tours = restart_tours ? restart_tours : (int32_t *)malloc(sizeof(int32_t) * (size_t)restarts * N);
    if (!costs || !tours) return CCO_ERR_NOMEM;
    int rc = cco_2opt_restarts(c, N, objective, seed, 0, restarts, init_tours, costs, tours, restart_moves);
    if (rc == CCO_OK) {
        int32_t arg = 0;
        for (int32_t r = 1; r < restarts; ++r) if (costs[r] < costs[arg]) arg = r;
        *best_cost = costs[arg];
        if (best_restart) *best_restart = arg;
        memcpy(best_perm, tours + (int64_t)arg * N, sizeof(int32_t) * (size_t)N);
    }
    if (!restart_costs) free(costs);
    if (!restart_tours) free(tours);
    return rc;
}

/* ------------------------------------------------------------------------------------------------
 * Exhaustive reference for N <= 12: every ring with t[0] = 0, in lexicographic order of t[1..N-1];
 * half_only = 1 keeps one of each mirror pair (t[1] < t[N-1]) for symmetric matrices.
 * Reports the number of rings visited, the minimum cost and the first ring that attains it; if
 * all_rings / all_costs are given (capacity cap) also every ring visited and its cost, in order.
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
    const int32_t *c; int32_t N, objective, half_only;
    int64_t count, best_cost; int32_t *best; int32_t *all_rings; int64_t *all_costs; int64_t cap;
    int32_t t[16]; uint8_t used[16];
} enum_state;

static void enum_rec(enum_state *s, int32_t depth)
{
    const int32_t N = s->N;
    if (depth == N) {
        if (s->half_only && N > 2 && !(s->t[1] < s->t[N - 1])) return;
        int64_t v = cco_ring_cost(s->c, N, s->t, s->objective);
        if (s->count < s->cap) {
            if (s->all_rings) memcpy(s->all_rings + s->count * N, s->t, sizeof(int32_t) * (size_t)N);
            if (s->all_costs) s->all_costs[s->count] = v;
        }
        if (s->count == 0 || v < s->best_cost) {
            s->best_cost = v;
            if (s->best) memcpy(s->best, s->t, sizeof(int32_t) * (size_t)N);
        }
        ++s->count;
        return;
    }
    for (int32_t v = 1; v < N; ++v) {
        if (s->used[v]) continue;
        s->used[v] = 1; s->t[depth] = v;
        enum_rec(s, depth + 1);
        s->used[v] = 0;
    }
}

int cco_exhaustive_rings(const int32_t *c, int32_t N, int32_t objective, int32_t half_only, int64_t *count,
                         int64_t *best_cost, int32_t *best_ring, int32_t *all_rings, int64_t *all_costs,
                         int64_t cap)
{
    if (!c || N < 2 || N > 12) return CCO_ERR_ARG;
    enum_state s;
    memset(&s, 0, sizeof s);
    s.c = c; s.N = N; s.objective = objective; s.half_only = half_only;
    s.best = best_ring; s.all_rings = all_rings; s.all_costs = all_costs; s.cap = cap;
    s.t[0] = 0; s.used[0] = 1;
    enum_rec(&s, 1);
    if (count) *count = s.count;
    if (best_cost) *best_cost = s.best_cost;
    return CCO_OK;
}

/* ------------------------------------------------------------------------------------------------
 * Pair-swap local search for the halving-doubling model (the "permute random pairs" neighbour of
 * Section 4.3, made exhaustive and deterministic; Section 5.3 explains why this landscape is flat:
 * a swap changes the cost only if it moves a round's critical pair).
 * Move (p, q), 0 <= p < q <= N-1: exchange the nodes at ranks p and q.  Move id = p*N + q.
 * Value of a move = halving-doubling cost of the order it produces.  No rank is anchored.
 * ---------------------------------------------------------------------------------------------- */
void cco_apply_swap(int32_t *t, int32_t p, int32_t q)
{
    int32_t tmp = t[p]; t[p] = t[q]; t[q] = tmp;
}

int64_t cco_rd_swap_value_by_definition(const int32_t *c, int32_t N, const int32_t *t, int32_t p, int32_t q)
{
    int32_t *u = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    memcpy(u, t, sizeof(int32_t) * (size_t)N);
    cco_apply_swap(u, p, q);
    int64_t v = cco_rd_cost(c, N, u);
    free(u);
    return v;
}

int64_t cco_rd_swap_neighbourhood_size(int32_t N) { return (int64_t)N * (N - 1) / 2; }

/* Delta tier.  In round k ranks i and i xor 2^k form a link whose value is the larger of its two
 * directed costs; the round costs the largest link.  Swapping ranks p and q touches, in each round,
 * only the links of p and of q (the same link when q = p xor 2^k, and then its value is unchanged
 * because both directed costs are still present).  So the new round cost is the maximum of the two
 * re-evaluated links and of the largest link among all others, which is one of the round's three
 * largest links. */
typedef struct { int64_t v[3]; int32_t link[3]; int32_t n; } cco_top3;

static int scan_swaps(const int32_t *c, int32_t N, const int32_t *t, cco_best *best, int64_t *all_values)
{
    int stages = 0;
    for (int32_t bit = 1; bit < N; bit <<= 1) ++stages;
    cco_top3 *top = (cco_top3 *)malloc(sizeof(cco_top3) * (size_t)(stages ? stages : 1));
    int64_t *round_cost = (int64_t *)malloc(sizeof(int64_t) * (size_t)(stages ? stages : 1));
    int k = 0;
    for (int32_t bit = 1; bit < N; bit <<= 1, ++k) {
        top[k].n = 0;
        round_cost[k] = 0;
        for (int32_t j = 0; j < N; ++j) {
            if (j & bit) continue;                      /* j = lower rank of the link */
            int64_t lv = max64(C_(t[j], t[j | bit]), C_(t[j | bit], t[j]));
            round_cost[k] = max64(round_cost[k], lv);
            /* insert into the sorted top-3 */
            int pos = top[k].n;
            while (pos > 0 && top[k].v[pos - 1] < lv) --pos;
            if (pos < 3) {
                int last = top[k].n < 3 ? top[k].n : 2;
                for (int m = last; m > pos; --m) { top[k].v[m] = top[k].v[m - 1]; top[k].link[m] = top[k].link[m - 1]; }
                top[k].v[pos] = lv; top[k].link[pos] = j;
                if (top[k].n < 3) ++top[k].n;
            }
        }
    }
    int found = 0;
    int64_t nvals = 0;
    for (int32_t p = 0; p < N - 1; ++p)
        for (int32_t q = p + 1; q < N; ++q) {
            int64_t total = 0;
            k = 0;
            for (int32_t bit = 1; bit < N; bit <<= 1, ++k) {
                if (q == (p ^ bit)) { total += round_cost[k]; continue; }
                int32_t lp = p & ~bit, lq = q & ~bit;
                int64_t others = 0;
                for (int m = 0; m < top[k].n; ++m)
                    if (top[k].link[m] != lp && top[k].link[m] != lq) { others = top[k].v[m]; break; }
                int32_t pb = t[p ^ bit], qb = t[q ^ bit];
                int64_t link_p = max64(C_(t[q], pb), C_(pb, t[q]));     /* rank p now holds t[q] */
                int64_t link_q = max64(C_(t[p], qb), C_(qb, t[p]));     /* rank q now holds t[p] */
                total += max64(others, max64(link_p, link_q));
            }
            int64_t id = (int64_t)p * N + q;
            if (all_values) all_values[nvals] = total;
            ++nvals;
            if (!found || total < best->value || (total == best->value && id < best->id)) {
                best->value = total; best->id = id; best->i = p; best->j = q; best->o = 0;
                found = 1;
            }
        }
    free(top);
    free(round_cost);
    return found;
}

int cco_rd_swap_all_values(const int32_t *c, int32_t N, const int32_t *t, int64_t *values)
{
    cco_best best;
    scan_swaps(c, N, t, &best, values);
    return CCO_OK;
}

int cco_rd_swap_descend(const int32_t *c, int32_t N, int32_t *t, int64_t *cost, int32_t *moves,
                        int32_t use_definition, int64_t *trace, int32_t trace_cap)
{
    if (!c || !t || N < 2 || (N & (N - 1))) return CCO_ERR_ARG;
    int64_t cur = cco_rd_cost(c, N, t);
    int32_t applied = 0;
    for (;;) {
        cco_best best;
        int found = 0;
        if (!use_definition) {
            found = scan_swaps(c, N, t, &best, NULL);
        } else {
            for (int32_t p = 0; p < N - 1; ++p)
                for (int32_t q = p + 1; q < N; ++q) {
                    int64_t v = cco_rd_swap_value_by_definition(c, N, t, p, q);
                    int64_t id = (int64_t)p * N + q;
                    if (!found || v < best.value || (v == best.value && id < best.id)) {
                        best.value = v; best.id = id; best.i = p; best.j = q; found = 1;
                    }
                }
        }
        if (!found || best.value >= cur) break;
        cco_apply_swap(t, best.i, best.j);
        cur = best.value;
        if (trace && applied < trace_cap) trace[applied] = best.id;
        ++applied;
    }
    *cost = cur;
    if (moves) *moves = applied;
    return CCO_OK;
}

int cco_rd_swap_restarts(const int32_t *c, int32_t N, uint64_t seed, int64_t r0, int64_t r1,
                         const int32_t *init_tours, int64_t *restart_costs, int32_t *restart_tours,
                         int32_t *restart_moves)
{
    if (!c || N < 2 || (N & (N - 1)) || r0 < 0 || r1 < r0) return CCO_ERR_ARG;
    int32_t *t = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    if (!t) return CCO_ERR_NOMEM;
    for (int64_t r = r0; r < r1; ++r) {
        if (init_tours) memcpy(t, init_tours + r * N, sizeof(int32_t) * (size_t)N);
        else cco_init_tour(seed, (uint32_t)r, N, t);
        int64_t cost; int32_t mv;
        int rc = cco_rd_swap_descend(c, N, t, &cost, &mv, 0, NULL, 0);
        if (rc != CCO_OK) { free(t); return rc; }
        if (restart_costs) restart_costs[r - r0] = cost;
        if (restart_moves) restart_moves[r - r0] = mv;
        if (restart_tours) memcpy(restart_tours + (r - r0) * N, t, sizeof(int32_t) * (size_t)N);
    }
    free(t);
    return CCO_OK;
}

/* ------------------------------------------------------------------------------------------------
 * BCube cost model (Section 4.1, equation C_b; Section 2.2: ranks are grouped by the base-B digits of
 * their id; in round i a rank exchanges with the B-1 ranks that differ from it in digit i only).
 * Round i costs the slowest of all those exchanges; rounds add up.  N must be a power of B.
 * The printed index set (j < N/B, k up to B, j + k*B^i) is read as digit arithmetic modulo B.
 * B = 2 is the halving-doubling model.
 * ---------------------------------------------------------------------------------------------- */
int64_t cco_bcube_cost(const int32_t *c, int32_t N, int32_t B, const int32_t *pi)
{
    int64_t total = 0;
    for (int64_t stride = 1; stride < N; stride *= B) {
        int64_t worst = 0;
        for (int32_t j = 0; j < N; ++j) {
            int32_t digit = (int32_t)((j / stride) % B);
            for (int32_t k = 1; k < B; ++k) {
                int32_t peer = (int32_t)(j - digit * stride + ((digit + k) % B) * stride);
                worst = max64(worst, C_(pi[j], pi[peer]));
            }
        }
        total += worst;
    }
    return total;
}

int cco_bcube_cost_batch(const int32_t *c, int32_t N, int32_t B, const int32_t *perms, int64_t count, int64_t *out)
{
    if (!c || N < 2 || B < 2 || count < 0 || (count > 0 && (!perms || !out))) return CCO_ERR_ARG;
    int64_t pw = 1;
    while (pw < N) pw *= B;
    if (pw != N) return CCO_ERR_ARG;
    for (int64_t b = 0; b < count; ++b) out[b] = cco_bcube_cost(c, N, B, perms + b * N);
    return CCO_OK;
}

/* ------------------------------------------------------------------------------------------------
 * Simulated annealing over the ring (Section 4.3: stochastic search by simulated annealing, a neighbour
 * obtained by permuting a random sub-array).  The paper fixes neither the schedule nor the random
 * numbers; this is one fully integer definition so that any two implementations agree bit for bit.
 *
 *   Chain r starts from init_tour(seed, r).  Step s = 0 .. steps-1 draws w = output number
 *   ((r << 32) | (1024 + s)) + 1 of the same SplitMix64 generator (initial tours use the low words below 1024).
 *   Proposal.  Two ring edges (edge p joins ranks p-1 and p): a = (w[63:43] * N) >> 21,
 *   d = 2 + ((w[42:22] * (N-3)) >> 21), b = (a + d) mod N, so every ordered pair of non-adjacent edges is
 *   (nearly) equally likely.  Exchanging them is the 2-opt move (i, j) = (lo, hi-1), or (hi, N-1) when lo = 0,
 *   lo = min(a,b), hi = max(a,b): the reversal of that span of ranks.
 *   delta = ring_sum(after) - ring_sum(before) = c[t[a-1]][t[b-1]] + c[t[a]][t[b]] - c[t[a]][t[a-1]] - c[t[b]][t[b-1]]
 *   on a symmetric matrix.
 *   Temperature.  Linear from t_start (step 0) towards t_end: T_s = (t_start*(steps-s) + t_end*s) / steps, kept
 *   as the exact numerator num_s.  T is the cost increase accepted with probability one half.
 *   Acceptance (Metropolis with the Boltzmann factor 2^(-delta/T)).  u = w[21:0] + 1 in [1, 2^22];
 *   L(u) = 4096*e + frac, e = floor(log2 u), frac = the next 12 bits of u below its leading one (piecewise-linear
 *   log2 in 1/4096 units); E = 22*4096 - L(u), i.e. -log2(u / 2^22).  Accept iff delta <= 0 or
 *   delta * 4096 * steps <= num_s * E.
 *   The chain reports the lowest-cost order it has visited (the earliest such), that cost, and how many
 *   proposals it accepted.  N < 4 has no proposals.
 * Limits: steps <= 2^24, 0 <= t_start, t_end <= 2^21 - 1, entries <= 2^21 - 1: every product fits int64.
 * ---------------------------------------------------------------------------------------------- */
enum { CCO_SA_STREAM_BASE = 1024, CCO_SA_MAX_STEPS = 1 << 24, CCO_SA_MAX_T = (1 << 21) - 1 };

void cco_sa_proposal(uint64_t seed, uint32_t r, uint32_t s, int32_t N, int32_t *a, int32_t *b, int32_t *u)
{
    uint64_t w = cco_splitmix64_at(seed, (((uint64_t)r << 32) | (uint64_t)(CCO_SA_STREAM_BASE + s)) + 1u);
    uint64_t hi21 = w >> 43, mid21 = (w >> 22) & 0x1FFFFFu;
    int32_t ea = (int32_t)((hi21 * (uint64_t)N) >> 21);
    int32_t d = 2 + (int32_t)((mid21 * (uint64_t)(N - 3)) >> 21);
    *a = ea;
    *b = (ea + d) % N;
    *u = (int32_t)(w & 0x3FFFFFu) + 1;
}

/* piecewise-linear log2(u) in units of 1/4096, exact at powers of two; 1 <= u <= 2^22 */
int32_t cco_sa_log2_fix(int32_t u)
{
    int32_t e = 0;
    while ((u >> (e + 1)) != 0) ++e;
    int32_t m = u - (1 << e);
    int32_t frac = e >= 12 ? (m >> (e - 12)) : (m << (12 - e));
    return e * 4096 + frac;
}

int cco_sa_accepts(int64_t delta, int64_t steps, int64_t num, int32_t u)
{
    if (delta <= 0) return 1;
    int64_t E = 22 * 4096 - cco_sa_log2_fix(u);
    return delta * 4096 * steps <= num * E;
}

/* One chain, in place on t.  use_definition != 0: delta by applying the move to a copy and recomputing the ring
 * sum.  trace (or NULL): int64 [steps], the current cost after every step. */
int cco_sa_chain(const int32_t *c, int32_t N, int32_t *t, int64_t steps, int32_t t_start, int32_t t_end, uint64_t seed,
                 uint32_t r, int32_t use_definition, int32_t *best_tour, int64_t *best_cost, int64_t *final_cost,
                 int32_t *accepted, int64_t *trace)
{
    if (!c || !t || N < 2 || steps < 0 || steps > CCO_SA_MAX_STEPS || t_start < 0 || t_end < 0 ||
        t_start > CCO_SA_MAX_T || t_end > CCO_SA_MAX_T)
        return CCO_ERR_ARG;
    int64_t cur = cco_ring_cost(c, N, t, CCO_SUM);
    int64_t best = cur;
    int32_t acc = 0;
    if (best_tour) memcpy(best_tour, t, sizeof(int32_t) * (size_t)N);
    int32_t *tmp = use_definition ? (int32_t *)malloc(sizeof(int32_t) * (size_t)N) : NULL;
    if (use_definition && !tmp) return CCO_ERR_NOMEM;
    for (int64_t s = 0; s < steps && N >= 4; ++s) {
        int32_t a, b, u;
        cco_sa_proposal(seed, r, (uint32_t)s, N, &a, &b, &u);
        int32_t lo = a < b ? a : b, hi = a < b ? b : a;
        int32_t i = lo ? lo : hi, j = lo ? hi - 1 : N - 1;
        int64_t delta;
        if (use_definition) {
            memcpy(tmp, t, sizeof(int32_t) * (size_t)N);
            cco_apply_move(tmp, N, i, j, 0);
            delta = cco_ring_cost(c, N, tmp, CCO_SUM) - cur;
        } else {
            int32_t ap = (a + N - 1) % N, bp = (b + N - 1) % N;
            delta = C_(t[ap], t[bp]) + C_(t[a], t[b]) - C_(t[a], t[ap]) - C_(t[b], t[bp]);
        }
        int64_t num = (int64_t)t_start * (steps - s) + (int64_t)t_end * s;
        if (cco_sa_accepts(delta, steps, num, u)) {
            cco_apply_move(t, N, i, j, 0);
            cur += delta;
            ++acc;
            if (cur < best) {
                best = cur;
                if (best_tour) memcpy(best_tour, t, sizeof(int32_t) * (size_t)N);
            }
        }
        if (trace) trace[s] = cur;
    }
    free(tmp);
    if (best_cost) *best_cost = best;
    if (final_cost) *final_cost = cur;
    if (accepted) *accepted = acc;
    return CCO_OK;
}

/* Chains r0 .. r1-1.  init (or NULL): int32 [r1-r0, N] starting orders instead of the seeded ones.
 * costs / tours: each chain's best cost and best order; accepted: accepted proposals. */
int cco_sa_chains(const int32_t *c, int32_t N, int64_t steps, int32_t t_start, int32_t t_end, uint64_t seed, int64_t r0,
                  int64_t r1, const int32_t *init, int64_t *costs, int32_t *tours, int32_t *accepted)
{
    if (!c || N < 2 || r0 < 0 || r1 < r0 || !costs || !tours) return CCO_ERR_ARG;
    if (!is_symmetric(c, N)) return CCO_ERR_NOT_SYMMETRIC;
    int32_t *t = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    if (!t) return CCO_ERR_NOMEM;
    int rc = CCO_OK;
    for (int64_t r = r0; r < r1 && rc == CCO_OK; ++r) {
        if (init) memcpy(t, init + (r - r0) * N, sizeof(int32_t) * (size_t)N);
        else cco_init_tour(seed, (uint32_t)r, N, t);
        int32_t acc = 0;
        rc = cco_sa_chain(c, N, t, steps, t_start, t_end, seed, (uint32_t)r, 0, tours + (r - r0) * N, costs + (r - r0),
                          NULL, &acc, NULL);
        if (accepted) accepted[r - r0] = acc;
    }
    free(t);
    return rc;
}

/* ------------------------------------------------------------------------------------------------
 * Double-binary-tree cost model (Section 4.1, equation C_dbt with the recursion T(i, j)).
 * The ranks i .. j form a subtree whose root is the middle rank m = floor((i+j)/2); its children are the
 * roots of the subtrees on i .. m-1 and m+1 .. j (the middle ranks of those ranges; the printed child
 * indices (3i+j)/2 - 1 and (i+3j)/2 + 1 are not the middles of those ranges and are read as such).
 * T(i, j) = 0 for i >= j, else the larger of  c[root][left child] + T(i, m-1)  (if the left range is not
 * empty) and  c[root][right child] + T(m+1, j): the most expensive root-to-leaf path.  The second tree has
 * the same shape with every rank moved down by one position (tree position p holds rank p+1 mod N); the
 * total is the larger of the two trees (Section 4.1: the maximum cost of all trees).  Latency-only view:
 * every hop weighs 1, as for the other models.
 * ---------------------------------------------------------------------------------------------- */
static int64_t dbt_T(const int32_t *c, int32_t N, const int32_t *pi, int32_t shift, int32_t i, int32_t j)
{
    if (i >= j) return 0;
    int32_t m = (i + j) / 2;
    int32_t root = pi[(m + shift) % N];
    int64_t worst = 0;
    if (i <= m - 1) {
        int32_t child = pi[((i + m - 1) / 2 + shift) % N];
        worst = max64(worst, C_(root, child) + dbt_T(c, N, pi, shift, i, m - 1));
    }
    int32_t child = pi[((m + 1 + j) / 2 + shift) % N];
    worst = max64(worst, C_(root, child) + dbt_T(c, N, pi, shift, m + 1, j));
    return worst;
}

/* one tree: shift = 0 (first tree) or 1 (second tree) */
int64_t cco_dbt_tree_cost(const int32_t *c, int32_t N, const int32_t *pi, int32_t shift)
{
    return dbt_T(c, N, pi, shift, 0, N - 1);
}

int64_t cco_dbt_cost(const int32_t *c, int32_t N, const int32_t *pi)
{
    return max64(cco_dbt_tree_cost(c, N, pi, 0), cco_dbt_tree_cost(c, N, pi, 1));
}

int cco_dbt_cost_batch(const int32_t *c, int32_t N, const int32_t *perms, int64_t count, int64_t *out)
{
    if (!c || N < 2 || count < 0 || (count > 0 && (!perms || !out))) return CCO_ERR_ARG;
    for (int64_t b = 0; b < count; ++b) out[b] = cco_dbt_cost(c, N, perms + b * N);
    return CCO_OK;
}

/* ------------------------------------------------------------------------------------------------
 * Size-weighted rounds (Section 4.1: round i of halving-doubling moves S / 2^(i+1) bytes, round i of BCube
 * S / B^(i+1)).  With a per-byte cost matrix (the bandwidth-bound end of c(S)) round i costs weight[i] times
 * its slowest exchange; weight[i] is whatever the caller derives from S.  All weights 1 is the latency-only
 * model above.  base = 2 is halving-doubling.
 * ---------------------------------------------------------------------------------------------- */
int64_t cco_bcube_cost_weighted(const int32_t *c, int32_t N, int32_t B, const int32_t *weights, const int32_t *pi)
{
    int64_t total = 0;
    int32_t round = 0;
    for (int64_t stride = 1; stride < N; stride *= B, ++round) {
        int64_t worst = 0;
        for (int32_t j = 0; j < N; ++j) {
            int32_t digit = (int32_t)((j / stride) % B);
            for (int32_t k = 1; k < B; ++k) {
                int32_t peer = (int32_t)(j - digit * stride + ((digit + k) % B) * stride);
                worst = max64(worst, C_(pi[j], pi[peer]));
            }
        }
        total += (int64_t)weights[round] * worst;
    }
    return total;
}

int cco_bcube_cost_weighted_batch(const int32_t *c, int32_t N, int32_t B, const int32_t *weights, const int32_t *perms,
                                  int64_t count, int64_t *out)
{
    if (!c || !weights || N < 2 || B < 2 || count < 0 || (count > 0 && (!perms || !out))) return CCO_ERR_ARG;
    int64_t pw = 1;
    while (pw < N) pw *= B;
    if (pw != N) return CCO_ERR_ARG;
    for (int64_t b = 0; b < count; ++b) out[b] = cco_bcube_cost_weighted(c, N, B, weights, perms + b * N);
    return CCO_OK;
}

/* ------------------------------------------------------------------------------------------------
 * Cost matrix from probes (Section 4.2): every ordered pair of nodes is probed K times; the pair's cost is
 * the RTT at the given percentile of its samples (the 10th in the paper, to filter out interference), and
 * the matrix is made symmetric by keeping the larger of the two directions.
 * Percentile by nearest rank: the sample of rank max(1, ceil(percentile * K / 100)) in ascending order.
 * samples: int32 [N, N, K]; the diagonal is not read and comes out 0.  Samples are limited to [0, 2^21 - 1].
 * ---------------------------------------------------------------------------------------------- */
static int cmp_i32(const void *x, const void *y)
{
    int32_t a = *(const int32_t *)x, b = *(const int32_t *)y;
    return (a > b) - (a < b);
}

int cco_cost_matrix_from_probes(const int32_t *samples, int32_t N, int32_t K, int32_t percentile, int32_t symmetrize,
                                int32_t *out)
{
    if (!samples || !out || N < 1 || K < 1 || percentile < 0 || percentile > 100) return CCO_ERR_ARG;
    int64_t rank = ((int64_t)percentile * K + 99) / 100;
    if (rank < 1) rank = 1;
    int32_t *buf = (int32_t *)malloc(sizeof(int32_t) * (size_t)K);
    if (!buf) return CCO_ERR_NOMEM;
    for (int32_t a = 0; a < N; ++a)
        for (int32_t b = 0; b < N; ++b) {
            if (a == b) { out[(int64_t)a * N + b] = 0; continue; }
            const int32_t *src = samples + ((int64_t)a * N + b) * K;
            for (int32_t s = 0; s < K; ++s) buf[s] = src[s] < 0 ? 0 : (src[s] > (1 << 21) - 1 ? (1 << 21) - 1 : src[s]);
            qsort(buf, (size_t)K, sizeof(int32_t), cmp_i32);
            out[(int64_t)a * N + b] = buf[rank - 1];
        }
    free(buf);
    if (symmetrize)
        for (int32_t a = 0; a < N; ++a)
            for (int32_t b = a + 1; b < N; ++b) {
                int32_t m = out[(int64_t)a * N + b] > out[(int64_t)b * N + a] ? out[(int64_t)a * N + b] : out[(int64_t)b * N + a];
                out[(int64_t)a * N + b] = m;
                out[(int64_t)b * N + a] = m;
            }
    return CCO_OK;
}

/* ------------------------------------------------------------------------------------------------
 * Simulated annealing under the halving-doubling model with the pair neighbour (Section 4.3: "permuting
 * random pairs").  Same chain as cco_sa_chain (same random word per step, same temperature, same
 * acceptance rule, same report) with a different proposal and cost:
 *   p = (w[63:43] * N) >> 21,  d = 1 + ((w[42:22] * (N-1)) >> 21),  q = (p + d) mod N: an ordered pair of
 *   distinct ranks, every one equally likely (nearly); the move exchanges the nodes at ranks p and q;
 *   delta = rd_cost(after) - rd_cost(before), here by swapping and recomputing.
 * N must be a power of two.  N = 1 is not a valid matrix; N = 2 has one move (delta 0 on any matrix whose
 * model takes both directions).
 * ---------------------------------------------------------------------------------------------- */
void cco_sa_rd_proposal(uint64_t seed, uint32_t r, uint32_t s, int32_t N, int32_t *p, int32_t *q, int32_t *u)
{
    uint64_t w = cco_splitmix64_at(seed, (((uint64_t)r << 32) | (uint64_t)(CCO_SA_STREAM_BASE + s)) + 1u);
    uint64_t hi21 = w >> 43, mid21 = (w >> 22) & 0x1FFFFFu;
    int32_t rp = (int32_t)((hi21 * (uint64_t)N) >> 21);
    int32_t d = 1 + (int32_t)((mid21 * (uint64_t)(N - 1)) >> 21);
    *p = rp;
    *q = (rp + d) % N;
    *u = (int32_t)(w & 0x3FFFFFu) + 1;
}

int cco_sa_rd_chain(const int32_t *c, int32_t N, int32_t *t, int64_t steps, int32_t t_start, int32_t t_end, uint64_t seed,
                    uint32_t r, int32_t *best_tour, int64_t *best_cost, int64_t *final_cost, int32_t *accepted,
                    int64_t *trace)
{
    if (!c || !t || N < 2 || (N & (N - 1)) || steps < 0 || steps > CCO_SA_MAX_STEPS || t_start < 0 || t_end < 0 ||
        t_start > CCO_SA_MAX_T || t_end > CCO_SA_MAX_T)
        return CCO_ERR_ARG;
    int64_t cur = cco_rd_cost(c, N, t);
    int64_t best = cur;
    int32_t acc = 0;
    if (best_tour) memcpy(best_tour, t, sizeof(int32_t) * (size_t)N);
    for (int64_t s = 0; s < steps; ++s) {
        int32_t p, q, u;
        cco_sa_rd_proposal(seed, r, (uint32_t)s, N, &p, &q, &u);
        cco_apply_swap(t, p, q);
        int64_t delta = cco_rd_cost(c, N, t) - cur;
        int64_t num = (int64_t)t_start * (steps - s) + (int64_t)t_end * s;
        if (cco_sa_accepts(delta, steps, num, u)) {
            cur += delta;
            ++acc;
            if (cur < best) {
                best = cur;
                if (best_tour) memcpy(best_tour, t, sizeof(int32_t) * (size_t)N);
            }
        } else {
            cco_apply_swap(t, p, q);    /* undo */
        }
        if (trace) trace[s] = cur;
    }
    if (best_cost) *best_cost = best;
    if (final_cost) *final_cost = cur;
    if (accepted) *accepted = acc;
    return CCO_OK;
}

int cco_sa_rd_chains(const int32_t *c, int32_t N, int64_t steps, int32_t t_start, int32_t t_end, uint64_t seed,
                     int64_t r0, int64_t r1, const int32_t *init, int64_t *costs, int32_t *tours, int32_t *accepted)
{
    if (!c || N < 2 || r0 < 0 || r1 < r0 || !costs || !tours) return CCO_ERR_ARG;
    int32_t *t = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    if (!t) return CCO_ERR_NOMEM;
    int rc = CCO_OK;
    for (int64_t r = r0; r < r1 && rc == CCO_OK; ++r) {
        if (init) memcpy(t, init + (r - r0) * N, sizeof(int32_t) * (size_t)N);
        else cco_init_tour(seed, (uint32_t)r, N, t);
        int32_t acc = 0;
        rc = cco_sa_rd_chain(c, N, t, steps, t_start, t_end, seed, (uint32_t)r, tours + (r - r0) * N, costs + (r - r0),
                             NULL, &acc, NULL);
        if (accepted) accepted[r - r0] = acc;
    }
    free(t);
    return rc;
}

/* ------------------------------------------------------------------------------------------------
 * Wider neighbourhoods for the ring search (Section 4.3 names two neighbour moves, sub-array permutation and
 * pair permutation, "alongside standard heuristics"; the two classes below are the textbook companions of
 * 2-opt and are this project's choice, like the descent itself).
 *
 * Move classes, a bitmask:
 *   1  2-opt moves as above.
 *   2  segment insertion (Or-opt): the L in {1, 2, 3} consecutive ranks s .. s+L-1 (1 <= s, s+L-1 <= N-1,
 *      L <= N-3) are taken out of the ring and put back, kept (o = 0) or reversed (o = 1, L > 1 only), into the
 *      gap between ranks g and g+1 (mod N) of the original numbering, g outside s-1 .. s+L-1.  The order of all
 *      other nodes is kept; rank 0 keeps its node.  Ring-sum objective on a symmetric matrix only.
 *      id = N*N + (variant*N + s)*N + g, variant = 0 (L = 1), 1, 2 (L = 2, o = 0, 1), 3, 4 (L = 3): every
 *      segment-insertion id is above every 2-opt id, so among equal values a 2-opt move wins.
 *   4  the orientation flip, i.e. the pair (i, j) = (1, N-1) that the 2-opt set leaves out: reverse t[1..N-1].
 *      Directed objectives only (on a symmetric matrix it changes nothing); id as a 2-opt move with o = 0.
 * A sweep scores every move of the enabled classes and applies the lexicographic minimum of (value, id) if it
 * strictly lowers the cost.
 * ---------------------------------------------------------------------------------------------- */
enum { CCO_MOVES_2OPT = 1, CCO_MOVES_OROPT = 2, CCO_MOVES_FLIP = 4 };

int cco_oropt_is_move(int32_t N, int32_t s, int32_t L, int32_t g, int32_t o)
{
    if (L < 1 || L > 3 || L > N - 3) return 0;
    if (s < 1 || s + L - 1 > N - 1) return 0;
    if (g < 0 || g > N - 1) return 0;
    if (g >= s - 1 && g <= s + L - 1) return 0;
    if (o < 0 || o > 1 || (o == 1 && L == 1)) return 0;
    return 1;
}

int64_t cco_oropt_move_id(int32_t N, int32_t s, int32_t L, int32_t g, int32_t o)
{
    int64_t variant = L == 1 ? 0 : 2 * L - 3 + o;
    return (int64_t)N * N + (variant * N + s) * N + g;
}

/* Takes the segment out and puts it back behind the node that sits at rank g. */
void cco_oropt_apply(int32_t *t, int32_t N, int32_t s, int32_t L, int32_t g, int32_t o)
{
    int32_t seg[3];
    int32_t *rest = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    for (int32_t k = 0; k < L; ++k) seg[k] = o ? t[s + L - 1 - k] : t[s + k];
    int32_t n = 0, at = -1;
    for (int32_t p = 0; p < N; ++p) {
        if (p >= s && p <= s + L - 1) continue;
        rest[n++] = t[p];
        if (p == g) at = n;                 /* the segment goes in front of rest[at] */
    }
    int32_t w = 0;
    for (int32_t k = 0; k < n; ++k) {
        if (k == at) for (int32_t x = 0; x < L; ++x) t[w++] = seg[x];
        t[w++] = rest[k];
    }
    if (at == n) for (int32_t x = 0; x < L; ++x) t[w++] = seg[x];
    free(rest);
}

int64_t cco_oropt_value_by_definition(const int32_t *c, int32_t N, const int32_t *t, int32_t s, int32_t L, int32_t g,
                                      int32_t o)
{
    int32_t *u = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    memcpy(u, t, sizeof(int32_t) * (size_t)N);
    cco_oropt_apply(u, N, s, L, g, o);
    int64_t v = cco_ring_cost(c, N, u, CCO_SUM);
    free(u);
    return v;
}

int64_t cco_oropt_neighbourhood_size(int32_t N)
{
    int64_t n = 0;
    for (int32_t L = 1; L <= 3 && L <= N - 3; ++L) n += (int64_t)(N - L) * (N - L - 1) * (L == 1 ? 1 : 2);
    return n;
}

/* Delta tier (symmetric matrix): with A, B the nodes before and behind the segment, S1 and S2 its first and last
 * node, P and Q the nodes at the two sides of the gap, the move removes the edges A-S1, S2-B, P-Q and adds A-B and
 * P-S1, S2-Q (kept) or P-S2, S1-Q (reversed).  Scans in increasing id. */
static int scan_insertions(const int32_t *c, int32_t N, const int32_t *t, int64_t cur, cco_best *best,
                           int64_t *all_values)
{
    int found = 0;
    int64_t nvals = 0;
    for (int32_t variant = 0; variant < 5; ++variant) {
        int32_t L = variant == 0 ? 1 : (variant + 3) / 2, o = variant == 0 ? 0 : (variant + 1) % 2;
        if (L > N - 3) continue;
        for (int32_t s = 1; s + L - 1 <= N - 1; ++s) {
            int32_t A = t[s - 1], S1 = t[s], S2 = t[s + L - 1], B = t[(s + L) % N];
            int64_t without = cur - C_(A, S1) - C_(S2, B) + C_(A, B);
            for (int32_t g = 0; g < N; ++g) {
                if (g >= s - 1 && g <= s + L - 1) continue;
                int32_t P = t[g], Q = t[(g + 1) % N];
                int64_t v = without - C_(P, Q) + (o ? C_(P, S2) + C_(S1, Q) : C_(P, S1) + C_(S2, Q));
                int64_t id = cco_oropt_move_id(N, s, L, g, o);
                if (all_values) all_values[nvals] = v;
                ++nvals;
                if (!found || v < best->value || (v == best->value && id < best->id)) {
                    best->value = v; best->id = id; best->i = s; best->j = g; best->o = variant;
                    found = 1;
                }
            }
        }
    }
    return found;
}

int cco_oropt_all_values(const int32_t *c, int32_t N, const int32_t *t, int64_t *values)
{
    cco_best best;
    scan_insertions(c, N, t, cco_ring_cost(c, N, t, CCO_SUM), &best, values);
    return CCO_OK;
}

/* Which class combinations are defined for which objective. */
int cco_local_classes_ok(int32_t objective, int32_t classes)
{
    if (objective < 0 || objective > 3) return 0;
    if (classes == CCO_MOVES_2OPT) return 1;
    if (classes == CCO_MOVES_OROPT || classes == (CCO_MOVES_2OPT | CCO_MOVES_OROPT)) return objective == CCO_SUM;
    if (classes == (CCO_MOVES_2OPT | CCO_MOVES_FLIP)) return (objective & 2) != 0;
    return 0;
}

/* One best-improvement descent over the enabled classes.  use_definition: every move scored by
 * apply-and-recompute.  trace: ids of the applied moves. */
int cco_local_descend(const int32_t *c, int32_t N, int32_t objective, int32_t classes, int32_t *t, int64_t *cost,
                      int32_t *moves, int32_t use_definition, int64_t *trace, int32_t trace_cap)
{
    if (!c || !t || N < 2 || !cco_local_classes_ok(objective, classes)) return CCO_ERR_ARG;
    int64_t *ws = (int64_t *)malloc(sizeof(int64_t) * 6 * (size_t)N);
    if (!ws) return CCO_ERR_NOMEM;
    const int directed = (objective & 2) != 0;
    int64_t cur = cco_ring_cost(c, N, t, objective);
    int32_t applied = 0;
    for (;;) {
        cco_best best, cand;
        int found = 0, kind = 0;      /* kind: 0 = reversal (2-opt or flip), 1 = insertion */
        if (classes & CCO_MOVES_2OPT) {
            if (!use_definition) {
                found = scan_moves(c, N, objective, t, cur, ws, &best, NULL);
            } else {
                for (int32_t i = 1; i <= N - 2; ++i)
                    for (int32_t j = i + 1; j <= N - 1; ++j) {
                        if (i == 1 && j == N - 1) continue;
                        for (int32_t o = 0; o <= directed; ++o) {
                            int64_t v = cco_move_value_by_definition(c, N, objective, t, i, j, o);
                            int64_t id = cco_move_id(N, objective, i, j, o);
                            if (!found || v < best.value || (v == best.value && id < best.id)) {
                                best.value = v; best.id = id; best.i = i; best.j = j; best.o = o; found = 1;
                            }
                        }
                    }
            }
        }
        if ((classes & CCO_MOVES_FLIP) && N >= 3) {
            int64_t v;
            if (use_definition) {
                v = cco_move_value_by_definition(c, N, objective, t, 1, N - 1, 0);
            } else {                   /* every hop walked the other way */
                v = 0;
                for (int32_t p = 0; p < N; ++p) {
                    int64_t back = C_(t[(p - 1 + N) % N], t[p]);
                    v = (objective & 1) ? max64(v, back) : v + back;
                }
            }
            int64_t id = cco_move_id(N, objective, 1, N - 1, 0);
            if (!found || v < best.value || (v == best.value && id < best.id)) {
                best.value = v; best.id = id; best.i = 1; best.j = N - 1; best.o = 0; found = 1;
            }
        }
        if (classes & CCO_MOVES_OROPT) {
            int f2 = 0;
            if (!use_definition) {
                f2 = scan_insertions(c, N, t, cur, &cand, NULL);
            } else {
                for (int32_t variant = 0; variant < 5; ++variant) {
                    int32_t L = variant == 0 ? 1 : (variant + 3) / 2, o = variant == 0 ? 0 : (variant + 1) % 2;
                    for (int32_t s = 1; s <= N - 1; ++s)
                        for (int32_t g = 0; g < N; ++g) {
                            if (!cco_oropt_is_move(N, s, L, g, o)) continue;
                            int64_t v = cco_oropt_value_by_definition(c, N, t, s, L, g, o);
                            int64_t id = cco_oropt_move_id(N, s, L, g, o);
                            if (!f2 || v < cand.value || (v == cand.value && id < cand.id)) {
                                cand.value = v; cand.id = id; cand.i = s; cand.j = g; cand.o = variant; f2 = 1;
                            }
                        }
                }
            }
            if (f2 && (!found || cand.value < best.value || (cand.value == best.value && cand.id < best.id))) {
                best = cand; found = 1; kind = 1;
            }
        }
        if (!found || best.value >= cur) break;
        if (kind == 0) {
            cco_apply_move(t, N, best.i, best.j, best.o);
        } else {
            int32_t variant = best.o;
            cco_oropt_apply(t, N, best.i, variant == 0 ? 1 : (variant + 3) / 2, best.j, variant == 0 ? 0 : (variant + 1) % 2);
        }
        cur = best.value;
        if (trace && applied < trace_cap) trace[applied] = best.id;
        ++applied;
    }
    free(ws);
    *cost = cur;
    if (moves) *moves = applied;
    return CCO_OK;
}

/* Restarts [r0, r1); init_tours (optional) is indexed by the restart number. */
int cco_local_restarts(const int32_t *c, int32_t N, int32_t objective, int32_t classes, uint64_t seed, int64_t r0,
                       int64_t r1, const int32_t *init_tours, int64_t *restart_costs, int32_t *restart_tours,
                       int32_t *restart_moves)
{
    if (!c || N < 2 || !cco_local_classes_ok(objective, classes) || r0 < 0 || r1 < r0) return CCO_ERR_ARG;
    if (!(objective & 2) && !is_symmetric(c, N)) return CCO_ERR_NOT_SYMMETRIC;
    int32_t *t = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    if (!t) return CCO_ERR_NOMEM;
    for (int64_t r = r0; r < r1; ++r) {
        if (init_tours) memcpy(t, init_tours + r * N, sizeof(int32_t) * (size_t)N);
        else cco_init_tour(seed, (uint32_t)r, N, t);
        int64_t cost; int32_t mv;
        int rc = cco_local_descend(c, N, objective, classes, t, &cost, &mv, 0, NULL, 0);
        if (rc != CCO_OK) { free(t); return rc; }
        if (restart_costs) restart_costs[r - r0] = cost;
        if (restart_moves) restart_moves[r - r0] = mv;
        if (restart_tours) memcpy(restart_tours + (r - r0) * N, t, sizeof(int32_t) * (size_t)N);
    }
    free(t);
    return CCO_OK;
}
