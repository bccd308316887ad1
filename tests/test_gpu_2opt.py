"""GPU parity, 2-opt search: cc_2opt_search / cc_2opt_search_ex against the CPU oracle.  The search is
deterministic, so exactly one result is right: per restart the final order, its cost and the number of
applied moves; over restarts the winner.  All integers: bit-exact."""
import os
import time

import numpy as np
import pytest
import torch

import oracle
import paper_2105_14088_amd as cc
from gen import COST_MAX, WORKLOADS, make_matrix, random_matrix, random_perms
from gpu_util import assert_search_equal, dev, gpu_search, report, say

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("built_library")]
THREADS = min(16, os.cpu_count() or 1)


def _oracle_rows(c, obj, seed, rows, init=None):
    costs, tours, moves = [], [], []
    for r in rows:
        a = oracle.restarts(c, obj, seed, int(r), int(r) + 1, init)
        costs.append(a[0]); tours.append(a[1]); moves.append(a[2])
    return dict(costs=np.concatenate(costs), tours=np.concatenate(tours), moves=np.concatenate(moves))


@pytest.mark.parametrize("n", [2, 3, 4, 5, 8, 13, 31, 64, 65, 100])
@pytest.mark.parametrize("obj", [0, 1, 2, 3])
def test_small_searches_every_objective(n, obj):
    say(f"2-opt N={n} obj={obj} R=40")
    c = random_matrix(n, 900 + n + obj, symmetric=not (obj & 2), lo=1, hi=4000)
    want = oracle.search(c, obj, 40, seed=77 + n)
    got = gpu_search(c, obj, 40, seed=77 + n)
    assert_search_equal(got, want)


@pytest.mark.parametrize("obj", [0, 2])
def test_large_costs_up_to_cost_max(obj):
    """Entries up to 2^21 - 1 (beyond any 16-bit fast path)."""
    say(f"2-opt N=64 obj={obj} costs up to COST_MAX")
    c = random_matrix(64, 4242 + obj, symmetric=not (obj & 2), lo=1, hi=COST_MAX)
    want = oracle.search(c, obj, 48, seed=5)
    assert_search_equal(gpu_search(c, obj, 48, seed=5), want)


@pytest.mark.parametrize("n", [4, 5, 6, 7, 9, 16, 33, 48, 63, 65, 96, 100, 127, 129, 150, 191, 193, 200, 255])
def test_sum_any_size_up_to_256_lds_kernel_and_its_fallback(n):
    """N not a multiple of 64: order and partner data in LDS, 16-bit matrix; fallback to the general kernel when an
    entry needs more than 16 bits; ties; caller-provided initial orders; one restart."""
    restarts = 21
    for hi, tag in ((5000, "16-bit path"), (65535, "largest entry 65535"), (65536, "fallback at 2^16"), (2, "ties")):
        say(f"2-opt N={n} sum, entries up to {hi} ({tag})")
        c = random_matrix(n, 7700 + n + hi % 97, symmetric=True, lo=1, hi=hi)
        c[1, 3] = c[3, 1] = hi
        want = oracle.search(c, 0, restarts, seed=13 + n)
        assert_search_equal(gpu_search(c, 0, restarts, seed=13 + n), want)
    c = random_matrix(n, 4321 + n, symmetric=True, lo=1, hi=9000)
    init = random_perms(n, 18, seed=n)
    assert_search_equal(gpu_search(c, 0, 18, seed=5, init=init), oracle.search(c, 0, 18, seed=0, init=init))
    assert_search_equal(gpu_search(c, 0, 1, seed=6), oracle.search(c, 0, 1, seed=6))


@pytest.mark.parametrize("n,restarts", [(128, 24), (192, 22), (256, 20)])
def test_n128_n256_sum_fast_path_and_its_fallback(n, restarts):
    """Several ranks per lane with a 16-bit LDS matrix when max(c) < 2^16; entries at or above 2^16 must
    take the general kernel (same results either way); and a matrix full of ties."""
    for hi, tag in ((6000, "16-bit path"), (65535, "16-bit path, largest entry 65535"), (65536, "fallback at 2^16"),
                    (COST_MAX, "fallback, COST_MAX"), (3, "ties")):
        say(f"2-opt N={n} sum, entries up to {hi} ({tag})")
        c = random_matrix(n, 7000 + n + hi % 97, symmetric=True, lo=1, hi=hi)
        c[3, 5] = c[5, 3] = hi
        want = oracle.search(c, 0, restarts, seed=11 + n)
        assert_search_equal(gpu_search(c, 0, restarts, seed=11 + n), want)
    say(f"2-opt N={n} sum, caller-provided initial tours, restarts not a multiple of 16")
    c = random_matrix(n, 1234 + n, symmetric=True, lo=1, hi=9000)
    init = random_perms(n, 19, seed=n)
    want = oracle.search(c, 0, 19, seed=0, init=init)
    assert_search_equal(gpu_search(c, 0, 19, seed=5, init=init), want)


@pytest.mark.parametrize("n,restarts", [(128, 24), (192, 22), (256, 20)])
@pytest.mark.parametrize("obj", [1, 3])
def test_n128_n256_max_hop_fast_path_and_its_fallback(n, restarts, obj):
    """Max-hop objective (undirected on a symmetric matrix, directed on an asymmetric one) with several ranks per lane
    and a 16-bit LDS matrix: hierarchy-like values, the largest 16-bit entry, the fallback at 2^16, plateaus of ties,
    caller-provided orders, a single restart, many restarts with a ragged last workgroup, and the orientation flip."""
    sym = obj == 1
    for hi, tag in ((6000, "16-bit path"), (65535, "16-bit path, largest entry 65535"), (65536, "fallback at 2^16"),
                    (3, "ties"), (40, "few distinct values")):
        say(f"2-opt N={n} objective {obj}, entries up to {hi} ({tag})")
        c = random_matrix(n, 7100 + n + hi % 97 + obj, symmetric=sym, lo=1, hi=hi)
        c[3, 5] = hi
        if sym:
            c[5, 3] = hi
        want = oracle.search(c, obj, restarts, seed=12 + n)
        assert_search_equal(gpu_search(c, obj, restarts, seed=12 + n), want)
    say(f"2-opt N={n} objective {obj}, caller-provided initial tours; one restart")
    c = random_matrix(n, 1334 + n + obj, symmetric=sym, lo=1, hi=9000)
    init = random_perms(n, 19, seed=n)
    assert_search_equal(gpu_search(c, obj, 19, seed=5, init=init), oracle.search(c, obj, 19, seed=0, init=init))
    assert_search_equal(gpu_search(c, obj, 1, seed=6), oracle.search(c, obj, 1, seed=6))
    say(f"2-opt N={n} objective {obj}, 2100 restarts (several wavefronts per workgroup, ragged end), sampled")
    got = gpu_search(c, obj, 2100, seed=8)
    rows = np.unique(np.concatenate([np.arange(0, 2100, 150), [2096, 2097, 2098, 2099]]))
    assert_search_equal(got, _oracle_rows(c, obj, 8, rows), rows=rows)
    if obj == 3:
        say(f"2-opt + orientation flip N={n}, directed max-hop")
        b = cc.cc_local_search_ex(dev(c), 3, cc.CC_MOVES_2OPT | cc.CC_MOVES_FLIP, restarts, 31)
        torch.cuda.synchronize()
        want = oracle.local_search(c, 3, cc.CC_MOVES_2OPT | cc.CC_MOVES_FLIP, restarts, 31)
        assert np.array_equal(b.restart_costs.cpu().numpy(), want["costs"])
        assert np.array_equal(b.restart_tours.cpu().numpy(), want["tours"])
        assert np.array_equal(b.restart_moves.cpu().numpy(), want["moves"])


@pytest.mark.parametrize("n,restarts", [(128, 24), (192, 22), (256, 20)])
def test_n128_n256_directed_sum_fast_path_and_its_fallback(n, restarts):
    """Directed ring sum with several ranks per lane and a 16-bit LDS matrix.  The fast path runs while
    max(c) * (N + 2) < 2^22 (its 32-bit keys then hold every partial delta); the first value beyond that, and larger
    ones, take the general kernel.  Also ties, caller-provided orders, one restart, many restarts, the flip."""
    limit = (1 << 22) // (n + 2)
    for hi, tag in ((6000, "fast path"), (limit - 1, "fast path, largest entry it takes"), (limit, "fallback at the limit"),
                    (65535, "fallback"), (COST_MAX, "fallback, COST_MAX"), (3, "ties")):
        say(f"2-opt N={n} directed sum, entries up to {hi} ({tag})")
        c = random_matrix(n, 7200 + n + hi % 97, symmetric=False, lo=max(1, hi - 4000), hi=hi)
        c[3, 5] = hi
        want = oracle.search(c, 2, restarts, seed=14 + n)
        assert_search_equal(gpu_search(c, 2, restarts, seed=14 + n), want)
    c = random_matrix(n, 1434 + n, symmetric=False, lo=1, hi=9000)
    say(f"2-opt N={n} directed sum, caller-provided initial tours; one restart; 2100 restarts sampled; flip")
    init = random_perms(n, 19, seed=n)
    assert_search_equal(gpu_search(c, 2, 19, seed=5, init=init), oracle.search(c, 2, 19, seed=0, init=init))
    assert_search_equal(gpu_search(c, 2, 1, seed=6), oracle.search(c, 2, 1, seed=6))
    got = gpu_search(c, 2, 2100, seed=8)
    rows = np.unique(np.concatenate([np.arange(0, 2100, 300), [2098, 2099]]))
    assert_search_equal(got, _oracle_rows(c, 2, 8, rows), rows=rows)
    b = cc.cc_local_search_ex(dev(c), 2, cc.CC_MOVES_2OPT | cc.CC_MOVES_FLIP, restarts, 31)
    torch.cuda.synchronize()
    want = oracle.local_search(c, 2, cc.CC_MOVES_2OPT | cc.CC_MOVES_FLIP, restarts, 31)
    assert np.array_equal(b.restart_costs.cpu().numpy(), want["costs"])
    assert np.array_equal(b.restart_tours.cpu().numpy(), want["tours"])
    assert np.array_equal(b.restart_moves.cpu().numpy(), want["moves"])


def test_workload4_matrix_max_hop_1024_restarts_full(capfd):
    """The N = 256 hierarchy of workload 4 under the max-hop objective, 1024 restarts, every restart replayed by the
    oracle."""
    c = make_matrix(4)
    seed = WORKLOADS[4].search_seed
    with capfd.disabled():
        say(f"matrix 4 (N=256), max-hop, 1024 restarts, all replayed by the oracle on {THREADS} threads")
    got = gpu_search(c, 1, 1024, seed)
    t0 = time.time()
    costs, tours, moves = oracle.restarts_parallel(c, 1, seed, 0, 1024, THREADS)
    report(f"matrix 4 max-hop (N=256): oracle replayed 1024 of 1024 restarts in {time.time() - t0:.1f} s")
    assert np.array_equal(got["costs"], costs) and np.array_equal(got["moves"], moves)
    assert np.array_equal(got["tours"], tours)
    k = int(np.lexsort((np.arange(1024), costs))[0])
    assert got["best_restart"] == k and np.array_equal(got["best_perm"], tours[k])


def test_n1024_sum_row_streaming_path_and_its_fallback():
    """N = 1024: rows streamed through LDS when max(c) < 2^16, general kernel otherwise; ties."""
    from concurrent.futures import ThreadPoolExecutor
    for hi, tag, restarts in ((3, "ties", 3), (65535, "16-bit path, largest entry 65535", 2), (65536, "fallback", 2)):
        say(f"2-opt N=1024 sum, entries up to {hi} ({tag})")
        c = random_matrix(1024, 8100 + hi % 89, symmetric=True, lo=1, hi=hi)
        c[3, 5] = c[5, 3] = hi
        with ThreadPoolExecutor(restarts) as ex:
            parts = list(ex.map(lambda r: oracle.restarts(c, 0, 21, r, r + 1), range(restarts)))
        got = gpu_search(c, 0, restarts, seed=21)
        assert np.array_equal(got["costs"], np.concatenate([p[0] for p in parts]))
        assert np.array_equal(got["tours"], np.concatenate([p[1] for p in parts]))
        assert np.array_equal(got["moves"], np.concatenate([p[2] for p in parts]))


def test_n512_sum_row_streaming_path_and_its_fallback():
    """N = 512 (the paper's large runs): the row-streaming kernel with four diagonals per lane; fallback; ties;
    a hierarchical matrix like workload 5's."""
    from concurrent.futures import ThreadPoolExecutor
    from gen import hierarchical_matrix
    w = WORKLOADS[5]
    cases = [(random_matrix(512, 8300, symmetric=True, lo=1, hi=3), "ties", 4),
             (random_matrix(512, 8301, symmetric=True, lo=1, hi=65535), "16-bit path, entries up to 65535", 3),
             (random_matrix(512, 8302, symmetric=True, lo=1, hi=65535), "fallback (one entry 2^16)", 2),
             (hierarchical_matrix(512, w.group_sizes, w.level_ranges, w.sigma, True, 8303), "hierarchical", 5)]
    cases[2][0][3, 5] = cases[2][0][5, 3] = 65536
    for c, tag, restarts in cases:
        say(f"2-opt N=512 sum ({tag})")
        with ThreadPoolExecutor(restarts) as ex:
            parts = list(ex.map(lambda r: oracle.restarts(c, 0, 22, r, r + 1), range(restarts)))
        got = gpu_search(c, 0, restarts, seed=22)
        assert np.array_equal(got["costs"], np.concatenate([p[0] for p in parts]))
        assert np.array_equal(got["tours"], np.concatenate([p[1] for p in parts]))
        assert np.array_equal(got["moves"], np.concatenate([p[2] for p in parts]))


def test_n64_sum_many_restarts():
    """Several wavefronts per SIMD and a ragged last workgroup: 4100 restarts on the workload matrix, a
    wide-entry matrix and a matrix full of ties, each checked on a spread of restarts."""
    for c, tag in ((make_matrix(2), "workload matrix"),
                   (random_matrix(64, 515, symmetric=True, lo=1, hi=COST_MAX), "entries up to COST_MAX"),
                   (random_matrix(64, 516, symmetric=True, lo=1, hi=3), "ties")):
        say(f"2-opt N=64 sum, 4100 restarts ({tag})")
        got = gpu_search(c, 0, 4100, seed=77)
        rows = np.unique(np.concatenate([np.arange(0, 4100, 41), [4096, 4097, 4098, 4099]]))
        want = _oracle_rows(c, 0, 77, rows)
        assert_search_equal(got, want, rows=rows)
        k = int(np.argmin(got["costs"]))
        assert got["best_restart"] == k and np.array_equal(got["best_perm"], got["tours"][k])


def test_many_ties_lowest_id_wins():
    """Few distinct cost values: most sweeps have tied best moves and restarts tie on final cost."""
    for n, obj in ((16, 0), (64, 0), (64, 1), (32, 3), (64, 2)):
        say(f"2-opt ties N={n} obj={obj}")
        c = random_matrix(n, 31 + n + obj, symmetric=not (obj & 2), lo=1, hi=3)
        want = oracle.search(c, obj, 64, seed=3)
        assert_search_equal(gpu_search(c, obj, 64, seed=3), want)


def test_explicit_initial_tours_and_single_restart():
    say("2-opt with caller-provided initial tours; R=1")
    c = make_matrix(2)
    init = random_perms(64, 17, seed=99)
    want = oracle.search(c, 0, 17, seed=0, init=init)
    assert_search_equal(gpu_search(c, 0, 17, seed=123, init=init), want)
    want1 = oracle.search(c, 0, 1, seed=8)
    assert_search_equal(gpu_search(c, 0, 1, seed=8), want1)


def test_simple_entry_point_matches_extended():
    say("cc_2opt_search (allocating form)")
    c = make_matrix(2)
    want = oracle.search(c, 0, 32, seed=WORKLOADS[2].search_seed)
    perm, cost = cc.cc_2opt_search(dev(c), 0, 32, WORKLOADS[2].search_seed)
    torch.cuda.synchronize()
    assert int(cost.item()) == want["best_cost"] and np.array_equal(perm.cpu().numpy(), want["best_perm"])


@pytest.mark.parametrize("n,obj", [(64, 0), (64, 3), (24, 1), (128, 0)])
def test_search_without_winner_then_best_of_restarts(n, obj):
    """The two-call form the benchmark times: per-restart results first, the winner picked by cc_best_of_restarts."""
    say(f"2-opt in two calls N={n} objective={obj}")
    c = random_matrix(n, 321 + n, symmetric=not (obj & 2), lo=1, hi=4000)
    restarts = 37
    want = oracle.search(c, obj, restarts, seed=11)
    bufs = cc.SearchBuffers(n, obj, restarts, "cuda")
    bufs.best_cost.fill_(-1)
    bufs.best_restart.fill_(-1)
    cc.cc_2opt_search_ex(dev(c), obj, restarts, 11, buffers=bufs, pick_best=False)
    torch.cuda.synchronize()
    assert int(bufs.best_cost.item()) == -1 and int(bufs.best_restart.item()) == -1     # untouched
    assert np.array_equal(bufs.restart_costs.cpu().numpy(), want["costs"])
    assert np.array_equal(bufs.restart_tours.cpu().numpy(), want["tours"])
    cc.cc_best_of_restarts(bufs)
    torch.cuda.synchronize()
    assert int(bufs.best_cost.item()) == want["best_cost"] and int(bufs.best_restart.item()) == want["best_restart"]
    assert np.array_equal(bufs.best_perm.cpu().numpy(), want["best_perm"])


def test_workload2_n64_sum_1024_restarts_full():
    say("C2: N=64 sum, 1024 restarts (all restarts compared)")
    c = make_matrix(2)
    seed = WORKLOADS[2].search_seed
    o = oracle.restarts_parallel(c, oracle.SUM, seed, 0, 1024, THREADS)
    k = int(np.argmin(o[0]))
    want = dict(costs=o[0], tours=o[1], moves=o[2], best_cost=int(o[0][k]), best_restart=k, best_perm=o[1][k])
    assert_search_equal(gpu_search(c, 0, 1024, seed), want)


def test_workload3_n64_max_directed_1024_restarts_full():
    say("C3: N=64 max directed, 1024 restarts (all restarts compared)")
    c = make_matrix(3)
    seed = WORKLOADS[3].search_seed
    o = oracle.restarts_parallel(c, oracle.MAX_DIRECTED, seed, 0, 1024, THREADS)
    k = int(np.argmin(o[0]))
    want = dict(costs=o[0], tours=o[1], moves=o[2], best_cost=int(o[0][k]), best_restart=k, best_perm=o[1][k])
    assert_search_equal(gpu_search(c, 3, 1024, seed), want)


def test_matrix3_n64_sum_directed_1024_restarts_full():
    say("N=64 directed sum on the asymmetric matrix, 1024 restarts (all restarts compared)")
    c = make_matrix(3)
    seed = WORKLOADS[3].search_seed
    o = oracle.restarts_parallel(c, oracle.SUM_DIRECTED, seed, 0, 1024, THREADS)
    k = int(np.argmin(o[0]))
    want = dict(costs=o[0], tours=o[1], moves=o[2], best_cost=int(o[0][k]), best_restart=k, best_perm=o[1][k])
    assert_search_equal(gpu_search(c, 2, 1024, seed), want)


@pytest.mark.parametrize("top", [(1 << 16) - 1, 1 << 16])
def test_n64_sum_directed_at_the_16_bit_boundary(top):
    """Largest entry one below / at 2^16: the last matrix the N = 64 kernel takes and the first it hands on."""
    say(f"2-opt N=64 obj=2, largest entry {top}")
    c = random_matrix(64, 8800 + (top & 1), symmetric=False, lo=top - 3000, hi=top)
    c[5, 9] = top
    want = oracle.search(c, 2, 40, seed=31)
    assert_search_equal(gpu_search(c, 2, 40, seed=31), want)


def _certify(c, obj, tour, cost):
    """Properties that hold at any size: a permutation anchored at rank 0's start node, its cost, and
    no improving move (checked with the oracle's move values)."""
    n = c.shape[0]
    assert sorted(tour) == list(range(n))
    assert oracle.ring_cost(c, tour, obj) == cost
    assert oracle.all_move_values(c, obj, tour).min() >= cost


def test_workload4_n256_sum_4096_restarts_full(capfd):
    """Full size on the GPU and in the oracle: every one of the 4096 restarts is replayed by the oracle (the same
    single-threaded routine over disjoint restart ranges on the host's cores) and compared - final order, cost,
    number of applied moves - and so is the winner."""
    with capfd.disabled():
        say(f"C4: N=256 sum, 4096 restarts, all replayed by the oracle on {THREADS} threads")
    c = make_matrix(4)
    seed = WORKLOADS[4].search_seed
    got = gpu_search(c, 0, 4096, seed)
    t0 = time.time()
    costs, tours, moves = oracle.restarts_parallel(c, 0, seed, 0, 4096, THREADS)
    report(f"C4 (N=256 sum): oracle replayed 4096 of 4096 restarts on {THREADS} threads in {time.time() - t0:.1f} s")
    assert np.array_equal(got["costs"], costs)
    assert np.array_equal(got["moves"], moves)
    assert np.array_equal(got["tours"], tours)
    k = int(np.lexsort((np.arange(4096), costs))[0])          # lowest cost, lowest restart among equals
    assert got["best_restart"] == k and got["best_cost"] == int(costs[k])
    assert np.array_equal(got["best_perm"], tours[k])
    for r in (k, 7, 4000):
        _certify(c, 0, got["tours"][r], int(got["costs"][r]))
    init = oracle.init_tours(seed, 256, 4096)
    assert (got["tours"][:, 0] == init[:, 0]).all()          # the anchor never moves


C5_MIN_RESTARTS = 64
C5_ORACLE_BUDGET_S = 420.0


def test_workload5_n1024_sum_256_restarts_full(capfd):
    """Full size on the GPU.  The oracle needs several core-seconds per restart at N = 1024, so it replays the
    restarts in rounds of one per host thread, in a fixed order that starts with a spread over the whole range, until
    all 256 are done; on a host too slow for that within the time allowed it stops after at least 64 and says how
    many were compared.  The winner is checked against the oracle when every restart was replayed."""
    c = make_matrix(5)
    seed = WORKLOADS[5].search_seed
    got = gpu_search(c, 0, 256, seed)
    spread = list(dict.fromkeys([0, 131, 255] + list(range(3, 256, 4))))
    order = spread + [r for r in range(256) if r not in set(spread)]
    assert sorted(order) == list(range(256))
    say(f"C5: N=1024 sum, 256 restarts, oracle on {THREADS} threads")
    from concurrent.futures import ThreadPoolExecutor
    done = []
    t0 = time.time()
    with ThreadPoolExecutor(THREADS) as ex:
        for lo in range(0, 256, THREADS):
            rows = order[lo:lo + THREADS]
            parts = list(ex.map(lambda r: _oracle_rows(c, 0, seed, [r]), rows))
            want = dict(costs=np.concatenate([p["costs"] for p in parts]),
                        tours=np.concatenate([p["tours"] for p in parts]),
                        moves=np.concatenate([p["moves"] for p in parts]))
            assert_search_equal(got, want, rows=rows)
            done += rows
            with capfd.disabled():          # a progress line per round, also when output is captured
                say(f"C5: {len(done)} restarts compared after {time.time() - t0:.0f} s")
            if len(done) >= C5_MIN_RESTARTS and time.time() - t0 > C5_ORACLE_BUDGET_S:
                break
    report(f"C5 (N=1024 sum): oracle replayed {len(done)} of 256 restarts on {THREADS} threads in {time.time() - t0:.1f} s")
    assert len(done) >= C5_MIN_RESTARTS
    k = int(np.lexsort((np.arange(256), got["costs"]))[0])
    if len(done) == 256:          # then got["costs"] is the oracle's, element for element
        assert got["best_restart"] == k and got["best_cost"] == int(got["costs"][k])
        assert np.array_equal(got["best_perm"], got["tours"][k])
    else:
        assert got["best_restart"] == k and np.array_equal(got["best_perm"], got["tours"][k])
    _certify(c, 0, got["tours"][k], int(got["costs"][k]))
    _certify(c, 0, got["tours"][17], int(got["costs"][17]))


def test_determinism_same_call_twice():
    say("2-opt determinism: two identical calls")
    c = make_matrix(3)
    a = gpu_search(c, 3, 256, 42)
    b = gpu_search(c, 3, 256, 42)
    assert_search_equal(a, b)


def test_largest_possible_costs_n1024():
    """N = 1024 with every entry 2^21 - 1: ring cost 1024 * (2^21 - 1) = 2^31 - 1024, the largest the contract allows
    and still inside int32; no move improves, so every restart returns its initial order with that cost."""
    say("extreme: N=1024, all entries COST_MAX")
    n = 1024
    c = np.full((n, n), COST_MAX, dtype=np.int32)
    np.fill_diagonal(c, 0)
    for obj in (0, 1, 2, 3):
        got = gpu_search(c, obj, 3, seed=9)
        want_cost = n * COST_MAX if not (obj & 1) else COST_MAX
        assert (got["costs"] == want_cost).all() and (got["moves"] == 0).all()
        assert np.array_equal(got["tours"], oracle.init_tours(9, n, 3))
    perms = random_perms(n, 5, seed=1)
    out = cc.cc_ring_cost_batch(dev(c), dev(perms), 0)
    rd = cc.cc_rd_cost_batch(dev(c), dev(perms))
    torch.cuda.synchronize()
    assert (out.cpu().numpy() == n * COST_MAX).all() and (rd.cpu().numpy() == 10 * COST_MAX).all()
    # one cheaper entry pair: exactly the moves that bring those two nodes together improve; compare with the oracle
    c[5, 9] = c[9, 5] = 1
    want = oracle.search(c, 0, 2, seed=9)
    assert_search_equal(gpu_search(c, 0, 2, seed=9), want)


@pytest.mark.parametrize("n", [13, 64, 100, 128, 512])
def test_sum_objective_reads_only_the_upper_triangle(n):
    """A matrix that is not symmetric breaks the contract of the undirected objectives; the ring-sum searches then
    see the matrix mirrored from its upper triangle, so their deltas stay exact and every descent ends.  Checked
    on matrices whose two triangles disagree completely, with entries on both sides of the 16-bit boundary."""
    restarts = 12 if n <= 128 else 3
    for hi in (3000, 70000):
        c = random_matrix(n, 9100 + n + hi % 7, symmetric=False, lo=0, hi=hi)
        mirrored = np.triu(c) + np.triu(c, 1).T
        assert not np.array_equal(c, c.T) and np.array_equal(mirrored, mirrored.T)
        say(f"2-opt N={n} sum on an asymmetric matrix, entries up to {hi}")
        want = oracle.search(mirrored, 0, restarts, seed=3 + n)
        assert_search_equal(gpu_search(c, 0, restarts, seed=3 + n), want)
        if n <= 128:
            both = cc.CC_MOVES_2OPT | cc.CC_MOVES_OROPT
            say(f"2-opt + segment insertion N={n} on the same matrix")
            b = cc.cc_local_search_ex(dev(c), 0, both, restarts, 3 + n)
            torch.cuda.synchronize()
            want = oracle.local_search(mirrored, 0, both, restarts, 3 + n)
            assert np.array_equal(b.restart_costs.cpu().numpy(), want["costs"])
            assert np.array_equal(b.restart_tours.cpu().numpy(), want["tours"])
            assert np.array_equal(b.restart_moves.cpu().numpy(), want["moves"])
