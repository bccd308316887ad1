"""GPU parity, cost matrix from probes (Section 4.2 percentile + max-symmetrisation) against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2105_14088_amd as cc
from gen import COST_MAX, make_matrix, probe_samples
from gpu_util import dev, say

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("built_library")]


def check(s, q, sym):
    out = cc.cc_cost_matrix_from_probes(dev(s), q, sym)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), oracle.cost_matrix_from_probes(s, q, sym))


@pytest.mark.parametrize("n,k", [(1, 5), (2, 1), (3, 2), (5, 7), (8, 63), (8, 64), (8, 65), (7, 255), (7, 256), (6, 257),
                                 (5, 1023), (5, 1024), (5, 1025), (4, 4096), (3, 10000), (3, 16384), (33, 100)])
def test_sizes_and_percentiles(n, k):
    rng = np.random.default_rng(n * 100000 + k)
    s = rng.integers(0, 20000, size=(n, n, k)).astype(np.int32)
    for q in (0, 10, 50, 99, 100):
        for sym in (True, False):
            say(f"probes N={n} K={k} percentile={q} symmetrize={sym}")
            check(s, q, sym)


def test_value_extremes_and_ties():
    say("probes: constant samples, zeros, out-of-range values, full range")
    rng = np.random.default_rng(3)
    n, k = 6, 500
    s = np.full((n, n, k), 777, dtype=np.int32)
    check(s, 10, True)
    check(np.zeros((n, n, k), dtype=np.int32), 10, True)
    s = rng.integers(0, COST_MAX + 1, size=(n, n, k)).astype(np.int32)
    s[0, 1, ::2] = -5
    s[1, 0, ::3] = 1 << 30
    s[2, 3, :] = COST_MAX
    for q in (10, 50, 90):
        check(s, q, True)
        check(s, q, False)
    s = rng.integers(40, 44, size=(n, n, k)).astype(np.int32)     # four distinct values: ranks inside long runs of ties
    for q in (1, 10, 25, 26, 50, 75, 100):
        check(s, q, False)


def test_synthetic_probe_traces_n64():
    """The N = 64 hierarchical matrix as base RTT, 2000 probes per ordered pair with 20 % interference."""
    say("probes N=64 K=2000 synthetic traces")
    base = make_matrix(2)
    s = probe_samples(base, 2000, seed=5)
    out = cc.cc_cost_matrix_from_probes(dev(s), 10, True)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.array_equal(got, oracle.cost_matrix_from_probes(s, 10, True))
    assert cc.cc_validate_matrix(out, True) == 0
    off = ~np.eye(64, dtype=bool)
    assert (got[off] >= base[off]).all() and (got[off] / base[off]).max() < 1.06


def test_full_size_n64_10000_probes():
    """The paper's probe count: 10000 samples per ordered pair at N = 64 (164 MB of samples)."""
    say("probes N=64 K=10000")
    rng = np.random.default_rng(10)
    s = rng.integers(100, 30000, size=(64, 64, 10000), dtype=np.int32)
    check(s, 10, True)


def test_whole_pipeline_probes_to_order_stays_on_the_device():
    """The method end to end (Sections 4.2 and 4.3) without a host round trip: probes -> cost matrix -> annealing ->
    2-opt from the chains' orders -> the winner scored again by the batch call.  Every stage equals the oracle's, and
    the reported cost is the ring cost of the reported order."""
    say("pipeline N=64: probes -> matrix -> annealing -> 2-opt -> batch cost of the winner")
    samples = probe_samples(make_matrix(2), 300, seed=11)
    chains, steps, seed = 32, 4000, 2105
    c_dev = cc.cc_cost_matrix_from_probes(dev(samples), 10, True)
    annealed = cc.cc_sa_search_ex(c_dev, chains, steps, 300, 0, seed)
    polished = cc.cc_2opt_search_ex(c_dev, cc.CC_RING_SUM, chains, seed, init_tours=annealed.restart_tours.clone())
    again = cc.cc_ring_cost_batch(c_dev, polished.best_perm.view(1, 64), cc.CC_RING_SUM)
    hd = cc.cc_rd_cost_batch(c_dev, polished.best_perm.view(1, 64))
    torch.cuda.synchronize()
    c = oracle.cost_matrix_from_probes(samples, 10, True)
    sa = oracle.sa_search(c, chains, steps, 300, 0, seed)
    want = oracle.search(c, oracle.SUM, chains, seed, init=sa["tours"])
    assert np.array_equal(c_dev.cpu().numpy(), c)
    assert np.array_equal(annealed.restart_tours.cpu().numpy(), sa["tours"])
    assert np.array_equal(polished.restart_tours.cpu().numpy(), want["tours"])
    best = polished.best_perm.cpu().numpy()
    assert np.array_equal(best, want["best_perm"]) and int(polished.best_cost.item()) == want["best_cost"]
    assert int(again.item()) == want["best_cost"] == oracle.ring_cost(c, best, oracle.SUM)
    assert int(hd.item()) == int(oracle.rd_cost_batch(c, best.reshape(1, 64))[0])
