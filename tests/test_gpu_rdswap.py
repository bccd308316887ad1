"""GPU parity, pair-swap search under the halving-doubling model: cc_rd_swap_search[_ex] against the CPU
oracle - per restart the final order, its cost and the number of applied swaps; over restarts the winner.
All integers: bit-exact."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2105_14088_amd as cc
from gen import COST_MAX, WORKLOADS, make_matrix, random_matrix, random_perms
from gpu_util import assert_search_equal, dev, say

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("built_library")]
THREADS = min(16, os.cpu_count() or 1)


def gpu_swap_search(c, restarts, seed, init=None):
    b = cc.cc_rd_swap_search_ex(dev(c), restarts, seed, None if init is None else dev(init))
    torch.cuda.synchronize()
    return dict(best_perm=b.best_perm.cpu().numpy(), best_cost=int(b.best_cost.item()),
                best_restart=int(b.best_restart.item()), costs=b.restart_costs.cpu().numpy(),
                tours=b.restart_tours.cpu().numpy(), moves=b.restart_moves.cpu().numpy())


@pytest.mark.parametrize("n", [2, 4, 8, 16, 32, 64, 128])
@pytest.mark.parametrize("symmetric", [True, False])
def test_swap_search_sizes(n, symmetric):
    for hi, tag in ((4000, "few ties"), (3, "many ties"), (COST_MAX, "entries up to COST_MAX")):
        restarts = 40 if n <= 64 else 6
        say(f"rd swap search N={n} symmetric={symmetric} {tag} R={restarts}")
        c = random_matrix(n, 4400 + n + hi % 101, symmetric=symmetric, lo=0, hi=hi)
        want = oracle.rd_swap_search(c, restarts, seed=31 + n)
        assert_search_equal(gpu_swap_search(c, restarts, seed=31 + n), want)


def test_swap_search_initial_tours_single_restart_and_simple_entry_point():
    say("rd swap search: caller-provided initial tours; R=1; allocating entry point")
    c = make_matrix(2)
    init = random_perms(64, 9, seed=4)
    want = oracle.rd_swap_search(c, 9, seed=0, init=init)
    assert_search_equal(gpu_swap_search(c, 9, seed=77, init=init), want)
    assert_search_equal(gpu_swap_search(c, 1, seed=5), oracle.rd_swap_search(c, 1, seed=5))
    want = oracle.rd_swap_search(c, 16, seed=WORKLOADS[2].search_seed)
    perm, cost = cc.cc_rd_swap_search(dev(c), 16, WORKLOADS[2].search_seed)
    torch.cuda.synchronize()
    assert int(cost.item()) == want["best_cost"] and np.array_equal(perm.cpu().numpy(), want["best_perm"])


@pytest.mark.parametrize("top", [(1 << 16) - 1, 1 << 16])
@pytest.mark.parametrize("symmetric", [True, False])
def test_swap_search_n64_at_the_16_bit_boundary(top, symmetric):
    """Largest entry one below / at 2^16: the N = 64 kernel's last matrix with 32-bit keys and its first with 64-bit
    ones; all entries close to the top, so that round costs add up to the largest totals."""
    say(f"rd swap search N=64, largest entry {top}, symmetric={symmetric}")
    c = random_matrix(64, 7100 + (top & 1), symmetric=symmetric, lo=top - 2000, hi=top)
    c[3, 11] = top
    if symmetric:
        c[11, 3] = top
    want = oracle.rd_swap_search(c, 24, seed=13)
    assert_search_equal(gpu_swap_search(c, 24, seed=13), want)


def test_swap_search_n64_1024_restarts_full():
    say("rd swap search: N=64 hierarchical matrix, 1024 restarts (all restarts compared)")
    c = make_matrix(2)
    seed = WORKLOADS[2].search_seed
    from concurrent.futures import ThreadPoolExecutor
    edges = np.linspace(0, 1024, THREADS * 2 + 1).astype(int)
    with ThreadPoolExecutor(THREADS) as ex:
        parts = list(ex.map(lambda s: oracle.rd_swap_restarts(c, seed, int(s[0]), int(s[1])), zip(edges[:-1], edges[1:])))
    costs = np.concatenate([p[0] for p in parts]); tours = np.concatenate([p[1] for p in parts])
    moves = np.concatenate([p[2] for p in parts])
    k = int(np.argmin(costs))
    want = dict(costs=costs, tours=tours, moves=moves, best_cost=int(costs[k]), best_restart=k, best_perm=tours[k])
    got = gpu_swap_search(c, 1024, seed)
    assert_search_equal(got, want)
    # properties: every result is a permutation, its cost is its halving-doubling cost, no swap improves it
    for r in (0, k, 1023):
        assert sorted(got["tours"][r]) == list(range(64))
        assert oracle.rd_cost(c, got["tours"][r]) == got["costs"][r]
        assert oracle.rd_swap_all_values(c, got["tours"][r]).min() >= got["costs"][r]


@pytest.mark.parametrize("n", [128, 256])
def test_swap_search_workgroup_kernel_and_its_fallback(n):
    """N = 128 / 256: 16-bit workgroup kernel when max(c) < 2^16, general kernel otherwise (decided on the device)."""
    for hi, sym, tag in ((65535, True, "entries up to 2^16 - 1 (16-bit kernel)"), (3, False, "many ties (16-bit kernel)"),
                         (65536, True, "one entry 2^16 (general kernel)")):
        say(f"rd swap search N={n} {tag}")
        c = random_matrix(n, 5100 + n + hi % 7, symmetric=sym, lo=0, hi=min(hi, 65535))
        if hi == 65536:
            c[3, 5] = c[5, 3] = 65536
        want = oracle.rd_swap_search(c, 5, seed=77 + n)
        assert_search_equal(gpu_swap_search(c, 5, seed=77 + n), want)


def test_swap_search_n256_and_n1024():
    say("rd swap search: N=256 hierarchical matrix, 6 restarts (16-bit workgroup kernel)")
    c = make_matrix(4)
    with __import__("concurrent.futures").futures.ThreadPoolExecutor(6) as ex:
        parts = list(ex.map(lambda r: oracle.rd_swap_restarts(c, 3, r, r + 1), range(6)))
    got = gpu_swap_search(c, 6, seed=3)
    assert np.array_equal(got["costs"], np.concatenate([p[0] for p in parts]))
    assert np.array_equal(got["tours"], np.concatenate([p[1] for p in parts]))
    assert np.array_equal(got["moves"], np.concatenate([p[2] for p in parts]))
    k = int(np.argmin(got["costs"]))
    assert got["best_restart"] == k and got["best_cost"] == got["costs"][k]
    say("rd swap search: N=1024, asymmetric, 3 % large entries, 2 restarts (workgroup kernel on the folded 16-bit copy)")
    c = random_matrix(1024, 999, symmetric=False, lo=1, hi=40)
    mask = np.random.default_rng(1).random((1024, 1024)) < 0.97
    c = np.where(mask, 1, c).astype(np.int32)
    np.fill_diagonal(c, 0)
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(2) as ex:
        parts = list(ex.map(lambda r: oracle.rd_swap_restarts(c, 3, r, r + 1), range(2)))
    got = gpu_swap_search(c, 2, seed=3)
    assert np.array_equal(got["costs"], np.concatenate([p[0] for p in parts]))
    assert np.array_equal(got["tours"], np.concatenate([p[1] for p in parts]))
    assert np.array_equal(got["moves"], np.concatenate([p[2] for p in parts]))
    assert (got["moves"] > 10).all()


@pytest.mark.parametrize("n", [512, 1024])
def test_swap_search_n512_n1024_folded_copy_and_fallback(n):
    """N = 512 / 1024: one workgroup per restart reading the folded 16-bit copy of the matrix from the workspace;
    one entry of 2^16 sends the same search to the general kernel.  Sparse large entries keep the descents short."""
    from concurrent.futures import ThreadPoolExecutor
    for top, tag in ((40, "folded 16-bit copy"), (65536, "general kernel")):
        say(f"rd swap search: N={n}, asymmetric, 3 % large entries, 2 restarts ({tag})")
        c = random_matrix(n, 500 + n, symmetric=False, lo=1, hi=40)
        mask = np.random.default_rng(n).random((n, n)) < 0.97
        c = np.where(mask, 1, c).astype(np.int32)
        np.fill_diagonal(c, 0)
        c[7, 3] = top
        with ThreadPoolExecutor(2) as ex:
            parts = list(ex.map(lambda r: oracle.rd_swap_restarts(c, 9, r, r + 1), range(2)))
        got = gpu_swap_search(c, 2, seed=9)
        assert np.array_equal(got["costs"], np.concatenate([p[0] for p in parts]))
        assert np.array_equal(got["tours"], np.concatenate([p[1] for p in parts]))
        assert np.array_equal(got["moves"], np.concatenate([p[2] for p in parts]))
        assert (got["moves"] > 5).all()
