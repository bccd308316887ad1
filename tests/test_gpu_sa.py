"""GPU parity, simulated annealing over the ring: cc_sa_search / cc_sa_search_ex against the oracle's
sequential chain, bit for bit (best cost, best order and accepted count of every chain)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2105_14088_amd as cc
from gen import COST_MAX, WORKLOADS, make_matrix, random_matrix
from gpu_util import dev, say

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("built_library")]
SEED = 0xC0FFEE55


def run(c, chains, steps, ts, te, seed, init=None):
    bufs = cc.cc_sa_search_ex(dev(c), chains, steps, ts, te, seed, init_tours=None if init is None else dev(init))
    torch.cuda.synchronize()
    return (bufs.restart_costs.cpu().numpy(), bufs.restart_tours.cpu().numpy(), bufs.restart_moves.cpu().numpy(),
            int(bufs.best_cost.item()), bufs.best_perm.cpu().numpy(), int(bufs.best_restart.item()))


def check(c, chains, steps, ts, te, seed, init=None):
    costs, tours, acc, bc, bp, br = run(c, chains, steps, ts, te, seed, init)
    want = oracle.sa_search(c, chains, steps, ts, te, seed, init)
    assert np.array_equal(costs, want["costs"])
    assert np.array_equal(acc, want["accepted"])
    assert np.array_equal(tours, want["tours"])
    assert (bc, br) == (want["best_cost"], want["best_chain"]) and np.array_equal(bp, want["best_perm"])
    return acc


@pytest.mark.parametrize("n", [2, 3, 4, 5, 8, 13, 63, 64, 65, 100, 128, 129, 200, 256, 1000, 1024])
def test_chains_match_oracle(n):
    c = random_matrix(n, 70 + n, symmetric=True, lo=1, hi=3000)
    steps = 3000 if n <= 256 else 1500
    for chains, ts, te in ((1, 400, 0), (5, 150, 150), (9, 0, 0), (6, 2000, 5)):
        say(f"sa N={n} chains={chains} steps={steps} T={ts}->{te}")
        check(c, chains, steps, ts, te, SEED + n)


@pytest.mark.parametrize("steps", [0, 1, 2, 63, 64, 65, 127, 128, 129, 1000])
def test_step_counts_around_the_proposal_batch(steps):
    say(f"sa N=64 steps={steps}")
    c = make_matrix(2)
    check(c, 8, steps, 300, 30, SEED)


def test_extreme_costs_and_temperatures():
    """Entries up to 2^21 - 1, temperatures at the limits, the largest step count's arithmetic (few steps run)."""
    say("sa extreme values")
    c = random_matrix(64, 9, symmetric=True, lo=0, hi=COST_MAX)
    check(c, 8, 4000, COST_MAX, 0, SEED)
    check(c, 8, 4000, COST_MAX, COST_MAX, SEED)
    check(c, 4, 3000, 1, 1, SEED)


@pytest.mark.parametrize("n", [200, 256])
def test_ring_chains_at_the_16_bit_boundary_n_up_to_256(n):
    """128 < N <= 256: the matrix as 16-bit entries in LDS when every entry is below 2^16, through L2 otherwise."""
    for top in ((1 << 16) - 1, 1 << 16, COST_MAX):
        say(f"sa N={n} largest entry {top}")
        c = random_matrix(n, 300 + n + top % 5, symmetric=True, lo=max(1, top - 30000), hi=top)
        c[1, 4] = c[4, 1] = top
        check(c, 5, 2000, 20000, 50, SEED + top % 9)


def test_given_initial_orders_and_duplicates_in_cost():
    say("sa init tours / ties")
    n = 32
    c = np.full((n, n), 7, dtype=np.int32)          # every move is neutral: all accepted, cost never changes
    np.fill_diagonal(c, 0)
    init = oracle.init_tours(SEED, n, 6, first=100)
    acc = check(c, 6, 500, 0, 0, SEED, init)
    assert (acc == 500).all()
    c = random_matrix(n, 3, symmetric=True, lo=1, hi=5)   # tiny value range: many equal costs
    check(c, 6, 2000, 2, 0, SEED, init)


def test_workload2_matrix_1024_chains():
    """The N = 64 hierarchical matrix, 1024 chains of 20000 steps cooling from the intra-rack cost scale to zero;
    the oracle replays a sample of the chains."""
    say("sa C2 matrix, 1024 chains x 20000 steps")
    c = make_matrix(2)
    chains, steps, ts, te = 1024, 20000, 300, 0
    seed = WORKLOADS[2].search_seed
    costs, tours, acc, bc, bp, br = run(c, chains, steps, ts, te, seed)
    rows = np.unique(np.concatenate([np.arange(0, chains, 41), [chains - 1, br]]))
    for r in rows:
        wc, wt, wa = oracle.sa_chains(c, steps, ts, te, seed, int(r), int(r) + 1)
        assert costs[r] == wc[0] and acc[r] == wa[0] and np.array_equal(tours[r], wt[0])
    assert np.array_equal(costs, oracle.ring_cost_batch(c, tours))
    assert bc == costs.min() and br == int(np.flatnonzero(costs == costs.min())[0]) and np.array_equal(bp, tours[br])


def test_annealed_orders_feed_the_descent():
    """Chains' best orders passed to the 2-opt descent as starting orders: the combination matches the oracle's."""
    say("sa -> 2-opt")
    c = make_matrix(2)
    chains = 64
    bufs = cc.cc_sa_search_ex(dev(c), chains, 5000, 300, 0, SEED)
    polished = cc.cc_2opt_search_ex(dev(c), 0, chains, SEED, init_tours=bufs.restart_tours.clone())
    torch.cuda.synchronize()
    sa = oracle.sa_search(c, chains, 5000, 300, 0, SEED)
    want = oracle.search(c, 0, chains, SEED, init=sa["tours"])
    assert np.array_equal(polished.restart_costs.cpu().numpy(), want["costs"])
    assert int(polished.best_cost.item()) == want["best_cost"] <= sa["best_cost"]


def test_simple_entry_point():
    say("cc_sa_search")
    c = make_matrix(2)
    perm, cost = cc.cc_sa_search(dev(c), 16, 4000, 300, 0, SEED)
    torch.cuda.synchronize()
    want = oracle.sa_search(c, 16, 4000, 300, 0, SEED)
    assert int(cost.item()) == want["best_cost"] and np.array_equal(perm.cpu().numpy(), want["best_perm"])


# ------------------------------------------------------------------------- halving-doubling model, pair neighbour
def check_rd(c, chains, steps, ts, te, seed, init=None):
    bufs = cc.cc_sa_rd_search_ex(dev(c), chains, steps, ts, te, seed, init_tours=None if init is None else dev(init))
    torch.cuda.synchronize()
    want = oracle.sa_rd_search(c, chains, steps, ts, te, seed, init)
    assert np.array_equal(bufs.restart_costs.cpu().numpy(), want["costs"])
    assert np.array_equal(bufs.restart_moves.cpu().numpy(), want["accepted"])
    assert np.array_equal(bufs.restart_tours.cpu().numpy(), want["tours"])
    assert (int(bufs.best_cost.item()), int(bufs.best_restart.item())) == (want["best_cost"], want["best_chain"])
    assert np.array_equal(bufs.best_perm.cpu().numpy(), want["best_perm"])


@pytest.mark.parametrize("n", [2, 4, 8, 16, 32, 64, 128, 256, 512, 1024])
@pytest.mark.parametrize("symmetric", [True, False])
def test_rd_chains_match_oracle(n, symmetric):
    steps = 2000 if n <= 64 else (600 if n <= 256 else 250)
    for hi, tag in ((3000, "few ties"), (3, "many ties"), (COST_MAX, "entries up to COST_MAX")):
        c = random_matrix(n, 800 + n + hi % 13, symmetric=symmetric, lo=0, hi=hi)
        for chains, ts, te in ((5, min(hi, 400), 0), (3, 0, 0)):
            say(f"sa rd N={n} symmetric={symmetric} {tag} chains={chains} steps={steps} T={ts}->{te}")
            check_rd(c, chains, steps, ts, te, SEED + n)


@pytest.mark.parametrize("steps", [0, 1, 63, 64, 65, 129, 1000])
def test_rd_step_counts_around_the_proposal_batch(steps):
    say(f"sa rd N=64 steps={steps}")
    check_rd(make_matrix(2), 6, steps, 300, 30, SEED)


def test_rd_workload2_matrix_1024_chains_and_given_orders():
    say("sa rd C2 matrix, 1024 chains x 5000 steps (sampled); given initial orders; simple entry point")
    c = make_matrix(2)
    chains, steps, ts, te = 1024, 5000, 300, 0
    seed = WORKLOADS[2].search_seed
    bufs = cc.cc_sa_rd_search_ex(dev(c), chains, steps, ts, te, seed)
    torch.cuda.synchronize()
    costs, tours, acc = bufs.restart_costs.cpu().numpy(), bufs.restart_tours.cpu().numpy(), bufs.restart_moves.cpu().numpy()
    for r in np.unique(np.concatenate([np.arange(0, chains, 97), [chains - 1, int(bufs.best_restart.item())]])):
        wc, wt, wa = oracle.sa_rd_chains(c, steps, ts, te, seed, int(r), int(r) + 1)
        assert costs[r] == wc[0] and acc[r] == wa[0] and np.array_equal(tours[r], wt[0])
    assert np.array_equal(costs, oracle.rd_cost_batch(c, tours))
    assert int(bufs.best_cost.item()) == costs.min()
    init = oracle.init_tours(SEED, 64, 7, first=50)
    check_rd(c, 7, 1500, 200, 0, SEED, init)
    perm, cost = cc.cc_sa_rd_search(dev(c), 12, 2000, 300, 0, SEED)
    torch.cuda.synchronize()
    want = oracle.sa_rd_search(c, 12, 2000, 300, 0, SEED)
    assert int(cost.item()) == want["best_cost"] and np.array_equal(perm.cpu().numpy(), want["best_perm"])


def test_longest_chain_and_largest_values():
    """The documented limits together: 2^24 steps, temperatures and entries at 2^21 - 1 (the products of the
    acceptance test then come within a factor of two of 2^63)."""
    say("sa ring: 2 chains x 2^24 steps, entries and temperatures up to 2^21 - 1")
    c = random_matrix(16, 5, symmetric=True, lo=0, hi=COST_MAX)
    check(c, 2, 1 << 24, COST_MAX, COST_MAX // 2, SEED)
    say("sa rd: 1 chain x 2^22 steps, entries and temperatures up to 2^21 - 1")
    c = random_matrix(8, 6, symmetric=False, lo=0, hi=COST_MAX)
    check_rd(c, 1, 1 << 22, COST_MAX, COST_MAX // 3, SEED)
