"""GPU parity, ring search over the wider move sets: cc_local_search / cc_local_search_ex (segment insertion, the
orientation flip) against the CPU oracle.  Deterministic search, all integers: per restart the final order, its cost
and the number of applied moves must be bit-exact, and so must the winner."""
import numpy as np
import pytest
import torch

import oracle
import paper_2105_14088_amd as cc
from gen import COST_MAX, WORKLOADS, make_matrix, random_matrix, random_perms
from gpu_util import assert_search_equal, dev, say

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("built_library")]
OROPT, BOTH, FLIP = cc.CC_MOVES_OROPT, cc.CC_MOVES_2OPT | cc.CC_MOVES_OROPT, cc.CC_MOVES_2OPT | cc.CC_MOVES_FLIP


def gpu_local(c, objective, classes, restarts, seed, init=None):
    b = cc.cc_local_search_ex(dev(c), objective, classes, restarts, seed, None if init is None else dev(init))
    torch.cuda.synchronize()
    return dict(best_perm=b.best_perm.cpu().numpy(), best_cost=int(b.best_cost.item()),
                best_restart=int(b.best_restart.item()), costs=b.restart_costs.cpu().numpy(),
                tours=b.restart_tours.cpu().numpy(), moves=b.restart_moves.cpu().numpy())


@pytest.mark.parametrize("n", [2, 3, 4, 5, 6, 7, 13, 31, 64, 65, 96, 97, 130])
@pytest.mark.parametrize("classes", [OROPT, BOTH])
def test_insertion_small_sizes(n, classes):
    """Every segment length limit (N = 4: single nodes only, N = 5: up to pairs), the LDS-matrix kernel (N <= 96)
    and the one that gathers through L2, workgroups of one to three waves; few ties and many."""
    restarts = 24 if n <= 65 else 10
    for hi, tag in ((4000, "few ties"), (3, "many ties")):
        say(f"local search N={n} classes={classes} R={restarts} entries up to {hi} ({tag})")
        c = random_matrix(n, 8100 + n + hi % 89, symmetric=True, lo=1, hi=hi)
        want = oracle.local_search(c, oracle.SUM, classes, restarts, seed=31 + n)
        assert_search_equal(gpu_local(c, oracle.SUM, classes, restarts, seed=31 + n), want)


@pytest.mark.parametrize("classes", [OROPT, BOTH])
def test_insertion_large_costs_and_given_starts(classes):
    say(f"local search N=64 classes={classes}, entries up to COST_MAX")
    c = random_matrix(64, 555, symmetric=True, lo=1, hi=COST_MAX)
    want = oracle.local_search(c, oracle.SUM, classes, 16, seed=9)
    assert_search_equal(gpu_local(c, oracle.SUM, classes, 16, seed=9), want)
    say(f"local search N=50 classes={classes}, caller-provided starts, one restart")
    c = random_matrix(50, 556, symmetric=True, lo=1, hi=7000)
    init = random_perms(50, 9, seed=3)
    assert_search_equal(gpu_local(c, oracle.SUM, classes, 9, seed=1, init=init),
                        oracle.local_search(c, oracle.SUM, classes, 9, seed=0, init=init))
    assert_search_equal(gpu_local(c, oracle.SUM, classes, 1, seed=4), oracle.local_search(c, oracle.SUM, classes, 1, 4))


@pytest.mark.parametrize("classes", [OROPT, BOTH])
def test_insertion_workload2_sampled_restarts(classes):
    """The N = 64 workload matrix at its 1024 restarts: every restart's cost against the oracle run on a sample of
    restarts, and properties that hold for all: orders are permutations with rank 0's node kept, the reported cost
    is the order's ring cost, the winner is the lexicographic minimum."""
    w = WORKLOADS[2]
    c = make_matrix(2)
    say(f"local search workload 2, classes={classes}, 1024 restarts")
    got = gpu_local(c, oracle.SUM, classes, 1024, w.search_seed)
    rows = np.arange(0, 1024, 37)
    for r in rows:
        costs, tours, moves = oracle.local_restarts(c, oracle.SUM, classes, w.search_seed, int(r), int(r) + 1)
        assert got["costs"][r] == costs[0] and got["moves"][r] == moves[0]
        assert np.array_equal(got["tours"][r], tours[0])
    starts = oracle.init_tours(w.search_seed, 64, 1024)
    assert np.array_equal(np.sort(got["tours"], axis=1), np.tile(np.arange(64, dtype=np.int32), (1024, 1)))
    assert np.array_equal(got["tours"][:, 0], starts[:, 0])
    assert np.array_equal(oracle.ring_cost_batch(c, got["tours"], oracle.SUM), got["costs"])
    arg = int(np.lexsort((np.arange(1024), got["costs"]))[0])
    assert got["best_restart"] == arg and got["best_cost"] == got["costs"][arg]
    assert np.array_equal(got["best_perm"], got["tours"][arg])
    if classes == BOTH:      # an optimum of the union is an optimum of 2-opt alone: sampled certificate
        for r in rows[:6]:
            assert oracle.all_move_values(c, oracle.SUM, got["tours"][r]).min() >= got["costs"][r]
            assert oracle.oropt_all_values(c, got["tours"][r]).min() >= got["costs"][r]


@pytest.mark.parametrize("n,restarts", [(256, 6), (1024, 2)])
def test_insertion_large_n(n, restarts):
    """Workgroups of 4 and 16 waves; the order-1024 case starts from a nearly sorted hierarchy so that the descent
    is short enough for the oracle."""
    c = make_matrix(4) if n == 256 else make_matrix(5)
    if n == 256:
        say("local search N=256, workload 4 matrix, 6 restarts, both classes")
        want = oracle.local_search(c, oracle.SUM, BOTH, restarts, seed=77)
        assert_search_equal(gpu_local(c, oracle.SUM, BOTH, restarts, seed=77), want)
        return
    say("local search N=1024, workload 5 matrix, starts = 2-opt optima with a few displaced nodes")
    base = cc.cc_2opt_search_ex(dev(c), oracle.SUM, restarts, 5)
    torch.cuda.synchronize()
    init = base.restart_tours.cpu().numpy().copy()
    rng = np.random.default_rng(1)
    for r in range(restarts):
        for _ in range(6):
            a, b = rng.integers(1, n, size=2)
            init[r, a], init[r, b] = init[r, b], init[r, a]
    want = oracle.local_search(c, oracle.SUM, BOTH, restarts, seed=0, init=init)
    assert_search_equal(gpu_local(c, oracle.SUM, BOTH, restarts, seed=0, init=init), want)


@pytest.mark.parametrize("n", [3, 4, 9, 64, 65, 100, 200])
@pytest.mark.parametrize("obj", [oracle.SUM_DIRECTED, oracle.MAX_DIRECTED])
def test_flip_with_directed_objectives(n, obj):
    restarts = 20 if n <= 100 else 8
    say(f"local search with the orientation flip, N={n} obj={obj} R={restarts}")
    c = random_matrix(n, 6100 + n + obj, symmetric=False, lo=1, hi=3000)
    want = oracle.local_search(c, obj, FLIP, restarts, seed=2 + n)
    assert_search_equal(gpu_local(c, obj, FLIP, restarts, seed=2 + n), want)


def test_flip_is_taken_on_a_one_way_ring():
    """c[a][a-1] = 1, all else 10, starts walking the expensive way: one flip each."""
    n = 40
    c = np.full((n, n), 10, dtype=np.int32)
    for a in range(n):
        c[a][(a - 1) % n] = 1
    np.fill_diagonal(c, 0)
    init = np.tile(np.array([0] + list(range(n - 1, 0, -1)), dtype=np.int32), (3, 1))
    for obj, end in ((oracle.SUM_DIRECTED, n), (oracle.MAX_DIRECTED, 1)):
        say(f"one-way ring, obj={obj}")
        got = gpu_local(c, obj, FLIP, 3, seed=0, init=init)
        assert got["costs"].tolist() == [end] * 3 and got["moves"].tolist() == [1] * 3
        assert np.array_equal(got["tours"], np.tile(np.arange(n, dtype=np.int32), (3, 1)))
        assert_search_equal(got, oracle.local_search(c, obj, FLIP, 3, seed=0, init=init))


@pytest.mark.parametrize("obj", [0, 1, 2, 3])
def test_class_2opt_alone_is_cc_2opt_search(obj):
    say(f"local search with 2-opt moves only, obj={obj}")
    c = random_matrix(64, 1000 + obj, symmetric=not (obj & 2), lo=1, hi=5000)
    a = gpu_local(c, obj, cc.CC_MOVES_2OPT, 32, seed=8)
    assert_search_equal(a, oracle.search(c, obj, 32, seed=8))
    perm, cost = cc.cc_local_search(dev(c), obj, cc.CC_MOVES_2OPT, 32, 8)
    torch.cuda.synchronize()
    assert int(cost.item()) == a["best_cost"] and np.array_equal(perm.cpu().numpy(), a["best_perm"])


def test_simple_entry_point_and_errors():
    c = random_matrix(48, 77, symmetric=True, lo=1, hi=900)
    say("cc_local_search, N=48, both classes")
    perm, cost = cc.cc_local_search(dev(c), oracle.SUM, BOTH, 12, 3)
    torch.cuda.synchronize()
    want = oracle.local_search(c, oracle.SUM, BOTH, 12, 3)
    assert int(cost.item()) == want["best_cost"] and np.array_equal(perm.cpu().numpy(), want["best_perm"])
    with pytest.raises(cc.CCError):
        cc.cc_local_search(dev(c), oracle.MAX, OROPT, 12, 3)
    with pytest.raises(cc.CCError):
        cc.cc_local_search(dev(c), oracle.SUM, FLIP, 12, 3)


@pytest.mark.parametrize("n,restarts", [(128, 18), (192, 14), (256, 13)])
@pytest.mark.parametrize("classes", [OROPT, BOTH])
def test_insertion_n128_n192_n256_wavefront_kernel_and_its_fallback(n, restarts, classes):
    """Several ranks per lane with a 16-bit LDS matrix when max(c) < 2^16; an entry at 2^16 takes the general kernel
    (same results either way); a matrix full of ties; caller-provided starts; restart counts that leave the last
    workgroup partly empty."""
    for hi, tag in ((5000, "16-bit path"), (65535, "largest entry 65535"), (65536, "fallback at 2^16"), (3, "ties")):
        if hi >= 65535 and classes == OROPT:
            continue
        say(f"local search N={n} classes={classes} entries up to {hi} ({tag})")
        c = random_matrix(n, 8800 + n + hi % 97, symmetric=True, lo=1, hi=hi)
        c[2, 7] = c[7, 2] = hi
        r = restarts if hi == 5000 else 4
        want = oracle.local_search(c, oracle.SUM, classes, r, seed=19 + n)
        assert_search_equal(gpu_local(c, oracle.SUM, classes, r, seed=19 + n), want)
    say(f"local search N={n} classes={classes}, caller-provided starts")
    c = random_matrix(n, 4444 + n, symmetric=True, lo=1, hi=9000)
    init = random_perms(n, 5, seed=n)
    assert_search_equal(gpu_local(c, oracle.SUM, classes, 5, seed=1, init=init),
                        oracle.local_search(c, oracle.SUM, classes, 5, seed=0, init=init))


@pytest.mark.parametrize("classes", [OROPT, BOTH])
def test_insertion_n64_at_the_16_bit_boundary(classes):
    """N = 64: entries up to 65535 still take the wavefront kernel (its 32-bit keys are then at their limit: two
    entries of 65535 shifted by 14 bits plus the gap word), one entry of 65536 sends the search to the general kernel."""
    for hi in (65535, 65536):
        say(f"local search N=64 classes={classes}, entries up to {hi}")
        c = random_matrix(64, 6060 + hi % 11, symmetric=True, lo=60000, hi=hi)
        c[5, 9] = c[9, 5] = hi
        c[11, 12] = c[12, 11] = 0
        np.fill_diagonal(c, 0)
        want = oracle.local_search(c, oracle.SUM, classes, 24, seed=hi)
        assert_search_equal(gpu_local(c, oracle.SUM, classes, 24, seed=hi), want)
