"""Seeded random sweep over sizes, objectives, value ranges and restart counts for the search calls: every case is
compared bit for bit with the oracle.  Sizes are drawn around the dispatch boundaries of the kernels (64, 96, 128,
192, 256 and their neighbours), value ranges around the 16-bit boundary and with many ties."""
import numpy as np
import pytest
import torch

import oracle
import paper_2105_14088_amd as cc
from gen import COST_MAX, random_matrix
from gpu_util import assert_search_equal, dev, gpu_search, say

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("built_library")]

SIZES = [4, 5, 7, 8, 15, 16, 17, 31, 32, 33, 47, 48, 63, 64, 65, 95, 96, 97, 100, 127, 128, 129, 160, 191, 192, 193, 200,
         255, 256]
HIS = [1, 2, 7, 300, 5000, 65535, 65536, 70000, COST_MAX]


def _cases(count, seed):
    rng = np.random.default_rng(seed)
    for k in range(count):
        n = int(rng.choice(SIZES))
        obj = int(rng.choice([0, 0, 1, 2, 3]))
        hi = int(rng.choice(HIS))
        restarts = int(rng.integers(1, 40 if n <= 128 else 12))
        yield k, n, obj, hi, restarts, int(rng.integers(0, 2**62))


@pytest.mark.parametrize("block", range(10))
def test_2opt_random_cases(block):
    for k, n, obj, hi, restarts, seed in _cases(20, 1000 + block):
        say(f"sweep {block}.{k}: 2-opt N={n} objective={obj} entries<={hi} restarts={restarts} seed={seed}")
        c = random_matrix(n, 31 * block + k, symmetric=not (obj & 2), lo=0 if hi > 2 else 1, hi=hi)
        assert_search_equal(gpu_search(c, obj, restarts, seed=seed), oracle.search(c, obj, restarts, seed=seed))


@pytest.mark.parametrize("block", range(3))
def test_swap_and_annealing_random_cases(block):
    rng = np.random.default_rng(500 + block)
    for k in range(10):
        n = int(rng.choice([2, 4, 8, 16, 32, 64, 128, 256]))
        hi = int(rng.choice(HIS))
        sym = bool(rng.integers(0, 2))
        restarts = int(rng.integers(1, 10 if n <= 64 else 4))
        seed = int(rng.integers(0, 2**62))
        c = random_matrix(n, 77 * block + k, symmetric=sym, lo=0, hi=hi)
        say(f"sweep {block}.{k}: pair swaps N={n} entries<={hi} symmetric={sym} restarts={restarts}")
        b = cc.cc_rd_swap_search_ex(dev(c), restarts, seed)
        torch.cuda.synchronize()
        want = oracle.rd_swap_search(c, restarts, seed)
        assert np.array_equal(b.restart_costs.cpu().numpy(), want["costs"])
        assert np.array_equal(b.restart_tours.cpu().numpy(), want["tours"])
        assert np.array_equal(b.restart_moves.cpu().numpy(), want["moves"])
        steps = int(rng.integers(0, 1500))
        ts, te = int(rng.integers(0, min(hi, 3000) + 1)), int(rng.integers(0, 50))
        say(f"sweep {block}.{k}: annealing (pairs) N={n} steps={steps} T={ts}->{te}")
        b = cc.cc_sa_rd_search_ex(dev(c), restarts, steps, ts, te, seed)
        torch.cuda.synchronize()
        want = oracle.sa_rd_search(c, restarts, steps, ts, te, seed)
        assert np.array_equal(b.restart_costs.cpu().numpy(), want["costs"])
        assert np.array_equal(b.restart_tours.cpu().numpy(), want["tours"])
        assert np.array_equal(b.restart_moves.cpu().numpy(), want["accepted"])
        m = int(rng.choice(SIZES))
        cs = random_matrix(m, 13 * block + k, symmetric=True, lo=0, hi=hi)
        say(f"sweep {block}.{k}: annealing (ring) N={m} steps={steps} T={ts}->{te}")
        b = cc.cc_sa_search_ex(dev(cs), restarts, steps, ts, te, seed)
        torch.cuda.synchronize()
        want = oracle.sa_search(cs, restarts, steps, ts, te, seed)
        assert np.array_equal(b.restart_costs.cpu().numpy(), want["costs"])
        assert np.array_equal(b.restart_tours.cpu().numpy(), want["tours"])
        assert np.array_equal(b.restart_moves.cpu().numpy(), want["accepted"])


@pytest.mark.parametrize("block", range(3))
def test_local_search_random_cases(block):
    """Wider move sets: segment insertion with or without 2-opt (ring sum), 2-opt with the orientation flip (directed
    objectives); N = 64 is drawn often because it has a kernel of its own with a fallback at the 16-bit boundary."""
    rng = np.random.default_rng(900 + block)
    both = cc.CC_MOVES_2OPT | cc.CC_MOVES_OROPT
    for k in range(16):
        n = int(rng.choice(SIZES + [64] * 8))
        hi = int(rng.choice(HIS))
        restarts = int(rng.integers(1, 30 if n <= 128 else 6))
        seed = int(rng.integers(0, 2**62))
        kind = int(rng.integers(0, 3))
        if kind < 2:
            classes, obj = (cc.CC_MOVES_OROPT, both)[kind], oracle.SUM
        else:
            classes, obj = cc.CC_MOVES_2OPT | cc.CC_MOVES_FLIP, int(rng.choice([oracle.SUM_DIRECTED, oracle.MAX_DIRECTED]))
        say(f"sweep {block}.{k}: local search N={n} classes={classes} objective={obj} entries<={hi} restarts={restarts}")
        c = random_matrix(n, 53 * block + k, symmetric=not (obj & 2), lo=0 if hi > 2 else 1, hi=hi)
        b = cc.cc_local_search_ex(dev(c), obj, classes, restarts, seed)
        torch.cuda.synchronize()
        got = dict(best_perm=b.best_perm.cpu().numpy(), best_cost=int(b.best_cost.item()),
                   best_restart=int(b.best_restart.item()), costs=b.restart_costs.cpu().numpy(),
                   tours=b.restart_tours.cpu().numpy(), moves=b.restart_moves.cpu().numpy())
        assert_search_equal(got, oracle.local_search(c, obj, classes, restarts, seed))
