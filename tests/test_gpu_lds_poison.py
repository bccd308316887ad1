"""Debug run with poisoned LDS: with CC_LDS_POISON=1 every library call first fills the LDS of all compute units with
0x7f bytes, so a kernel that reads LDS it has not written itself sees garbage, not what an earlier launch left there.
One case per kernel family, each compared bit for bit with the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2105_14088_amd as cc
from gen import random_matrix
from gpu_util import assert_search_equal, dev, gpu_search, say

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("built_library")]


@pytest.fixture(autouse=True)
def poisoned(monkeypatch):
    monkeypatch.setenv("CC_LDS_POISON", "1")


def _orders(n, count, seed):
    t = cc.cc_init_tours(n, count, seed)
    torch.cuda.synchronize()
    return t


@pytest.mark.parametrize("n", [8, 64, 100, 128, 256, 1024])
def test_batches_with_poisoned_lds(n):
    c = random_matrix(n, 5 + n, symmetric=False, lo=0, hi=60000)
    count = 40000 if n == 256 else 3000          # N = 256: large enough for the kernels with the matrix in LDS
    perms = _orders(n, count, 11)
    ph = perms.cpu().numpy()
    say(f"poisoned LDS: batches N={n} orders={count}")
    for obj in (0, 1):
        got = cc.cc_ring_cost_batch(dev(c), perms, obj)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), oracle.ring_cost_batch(c, ph, obj))
    if n <= 256:
        got = cc.cc_ring_cost_batch_u8(dev(c), perms.to(torch.uint8), 0)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), oracle.ring_cost_batch(c, ph, 0))
    if n & (n - 1) == 0:
        ws = torch.empty(cc.cc_rd_batch_workspace_bytes(n), dtype=torch.uint8, device="cuda")
        for w in (None, ws):
            got = cc.cc_rd_cost_batch(dev(c), perms, workspace=w)
            torch.cuda.synchronize()
            assert np.array_equal(got.cpu().numpy(), oracle.rd_cost_batch(c, ph))
        got = cc.cc_dbt_cost_batch(dev(c), perms)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), oracle.dbt_cost_batch(c, ph))
    if n in (64, 256, 1024):
        for w in (None, ws):
            got = cc.cc_bcube_cost_batch(dev(c), 4, perms, workspace=w)
            torch.cuda.synchronize()
            assert np.array_equal(got.cpu().numpy(), oracle.bcube_cost_batch(c, 4, ph))


@pytest.mark.parametrize("n,restarts", [(64, 9), (100, 5), (128, 5), (192, 4), (256, 18), (300, 2), (512, 2), (1024, 1)])
@pytest.mark.parametrize("hi", [3000, 70000])
def test_2opt_with_poisoned_lds(n, restarts, hi):
    for obj in (0, 1, 2, 3):
        if n > 256 and obj != 0 and hi > 3000:
            continue                                 # the general kernel at this size is covered by the smaller value range
        say(f"poisoned LDS: 2-opt N={n} objective={obj} entries<={hi} restarts={restarts}")
        c = random_matrix(n, 3 * n + obj, symmetric=not (obj & 2), lo=0, hi=hi)
        assert_search_equal(gpu_search(c, obj, restarts, seed=77 + n), oracle.search(c, obj, restarts, seed=77 + n))


@pytest.mark.parametrize("n,restarts", [(64, 6), (128, 3), (256, 3), (100, 3)])
def test_wider_move_sets_with_poisoned_lds(n, restarts):
    both = cc.CC_MOVES_2OPT | cc.CC_MOVES_OROPT
    for classes, obj in ((cc.CC_MOVES_OROPT, 0), (both, 0), (cc.CC_MOVES_2OPT | cc.CC_MOVES_FLIP, 3),
                         (cc.CC_MOVES_2OPT | cc.CC_MOVES_FLIP, 2)):
        say(f"poisoned LDS: local search N={n} classes={classes} objective={obj}")
        c = random_matrix(n, 7 * n + classes, symmetric=not (obj & 2), lo=0, hi=4000)
        b = cc.cc_local_search_ex(dev(c), obj, classes, restarts, 5)
        torch.cuda.synchronize()
        got = dict(best_perm=b.best_perm.cpu().numpy(), best_cost=int(b.best_cost.item()),
                   best_restart=int(b.best_restart.item()), costs=b.restart_costs.cpu().numpy(),
                   tours=b.restart_tours.cpu().numpy(), moves=b.restart_moves.cpu().numpy())
        assert_search_equal(got, oracle.local_search(c, obj, classes, restarts, 5))


@pytest.mark.parametrize("n,restarts", [(64, 6), (128, 2), (256, 2), (512, 1), (32, 3)])
def test_pair_swaps_and_annealing_with_poisoned_lds(n, restarts):
    c = random_matrix(n, 9 * n, symmetric=True, lo=0, hi=5000)
    say(f"poisoned LDS: pair swaps N={n}")
    b = cc.cc_rd_swap_search_ex(dev(c), restarts, 3)
    torch.cuda.synchronize()
    want = oracle.rd_swap_search(c, restarts, 3)
    assert np.array_equal(b.restart_costs.cpu().numpy(), want["costs"])
    assert np.array_equal(b.restart_tours.cpu().numpy(), want["tours"])
    assert np.array_equal(b.restart_moves.cpu().numpy(), want["moves"])
    if n <= 256:
        say(f"poisoned LDS: annealing N={n}")
        for call, ref in ((cc.cc_sa_search_ex, oracle.sa_search), (cc.cc_sa_rd_search_ex, oracle.sa_rd_search)):
            b = call(dev(c), restarts, 800, 300, 0, 3)
            torch.cuda.synchronize()
            want = ref(c, restarts, 800, 300, 0, 3)
            assert np.array_equal(b.restart_costs.cpu().numpy(), want["costs"])
            assert np.array_equal(b.restart_tours.cpu().numpy(), want["tours"])
            assert np.array_equal(b.restart_moves.cpu().numpy(), want["accepted"])


def test_probes_with_poisoned_lds():
    rng = np.random.default_rng(4)
    s = rng.integers(0, 30000, size=(12, 12, 500), dtype=np.int32)
    say("poisoned LDS: probes N=12 K=500")
    got = cc.cc_cost_matrix_from_probes(dev(s), 10, True)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), oracle.cost_matrix_from_probes(s, 10, True))
