"""GPU parity of the calls chained as the paper chains them (Sections 4.2 - 4.3): probes -> cost matrix -> annealing ->
descent from the annealed orders -> winner, and the four cost models of Section 4.1 on the winning order.  Every
stage is compared with the oracle's result for the same stage, computed from the oracle's own previous stage."""
import numpy as np
import pytest
import torch

import oracle
import paper_2105_14088_amd as cc
from gen import make_matrix, probe_samples
from gpu_util import dev, say

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("built_library")]


def test_probes_to_rank_order_n64():
    say("pipeline N=64: probes -> matrix -> annealing -> 2-opt -> cost models")
    base = make_matrix(2)
    samples = probe_samples(base, 300, seed=21)
    seed, chains = 0xC0FFEE99, 48

    c_dev = cc.cc_cost_matrix_from_probes(dev(samples), 10, True)
    assert cc.cc_validate_matrix(c_dev, True) == 0
    c_host = oracle.cost_matrix_from_probes(samples, 10, True)
    torch.cuda.synchronize()
    assert np.array_equal(c_dev.cpu().numpy(), c_host)

    sa = cc.cc_sa_search_ex(c_dev, chains, 8000, 300, 0, seed)
    sa_want = oracle.sa_search(c_host, chains, 8000, 300, 0, seed)
    torch.cuda.synchronize()
    assert np.array_equal(sa.restart_tours.cpu().numpy(), sa_want["tours"])

    polished = cc.cc_2opt_search_ex(c_dev, cc.CC_RING_SUM, chains, seed, init_tours=sa.restart_tours.clone())
    want = oracle.search(c_host, oracle.SUM, chains, seed, init=sa_want["tours"])
    torch.cuda.synchronize()
    assert np.array_equal(polished.restart_costs.cpu().numpy(), want["costs"])
    assert np.array_equal(polished.restart_tours.cpu().numpy(), want["tours"])
    best = polished.best_perm.cpu().numpy()
    assert np.array_equal(best, want["best_perm"]) and int(polished.best_cost.item()) == want["best_cost"]
    assert want["best_cost"] <= sa_want["best_cost"] <= oracle.ring_cost_batch(c_host, oracle.init_tours(seed, 64, chains)).min()

    one = polished.best_perm.view(1, 64)
    got = [int(cc.cc_ring_cost_batch(c_dev, one, cc.CC_RING_SUM).item()), int(cc.cc_ring_cost_batch(c_dev, one, cc.CC_RING_MAX).item()),
           int(cc.cc_rd_cost_batch(c_dev, one).item()), int(cc.cc_bcube_cost_batch(c_dev, 4, one).item()),
           int(cc.cc_dbt_cost_batch(c_dev, one).item()),
           int(cc.cc_ring_cost_batch_u8(c_dev, one.to(torch.uint8), cc.CC_RING_SUM).item())]
    torch.cuda.synchronize()
    assert got == [oracle.ring_cost(c_host, best, oracle.SUM), oracle.ring_cost(c_host, best, oracle.MAX),
                   oracle.rd_cost(c_host, best), oracle.bcube_cost(c_host, 4, best), oracle.dbt_cost(c_host, best),
                   oracle.ring_cost(c_host, best, oracle.SUM)]
    assert got[0] == want["best_cost"]


def test_probes_to_halving_doubling_order_n64():
    say("pipeline N=64, halving-doubling: probes -> matrix -> annealing (pairs) -> pair-swap descent")
    base = make_matrix(2)
    samples = probe_samples(base, 200, seed=22)
    seed, chains = 0xC0FFEE98, 24
    c_dev = cc.cc_cost_matrix_from_probes(dev(samples), 10, True)
    c_host = oracle.cost_matrix_from_probes(samples, 10, True)
    sa = cc.cc_sa_rd_search_ex(c_dev, chains, 3000, 300, 0, seed)
    sa_want = oracle.sa_rd_search(c_host, chains, 3000, 300, 0, seed)
    torch.cuda.synchronize()
    assert np.array_equal(sa.restart_tours.cpu().numpy(), sa_want["tours"])
    polished = cc.cc_rd_swap_search_ex(c_dev, chains, seed, init_tours=sa.restart_tours.clone())
    want = oracle.rd_swap_search(c_host, chains, seed, init=sa_want["tours"])
    torch.cuda.synchronize()
    assert np.array_equal(polished.restart_costs.cpu().numpy(), want["costs"])
    assert np.array_equal(polished.best_perm.cpu().numpy(), want["best_perm"])
    assert int(polished.best_cost.item()) == want["best_cost"] <= sa_want["best_cost"]
    assert int(cc.cc_rd_cost_batch(c_dev, polished.best_perm.view(1, 64)).item()) == want["best_cost"]
