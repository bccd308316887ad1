"""GPU test of cc_2opt_search_noalloc, the form of cc_2opt_search whose per-restart results live in the library's
static device array: through the C ABI, its best order and cost must equal those of cc_2opt_search bit for bit, on
two calls in a row, the second one smaller than the first (the array then still holds the first call's contents).
The CPU oracle is checked beside it.  The size limit is a host-side check that launches nothing."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2105_14088_amd as cc
from gen import WORKLOADS, make_matrix, random_matrix
from gpu_util import dev, say

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("built_library")]


def _both(c, obj, restarts, seed):
    cd = dev(c)
    n = c.shape[0]
    best_perm = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    best_cost = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    cc.cc_2opt_search_noalloc(cd, obj, restarts, seed, best_perm, best_cost)
    torch.cuda.synchronize()
    ref_perm, ref_cost = cc.cc_2opt_search(cd, obj, restarts, seed)
    torch.cuda.synchronize()
    return best_perm.cpu().numpy(), int(best_cost.item()), ref_perm.cpu().numpy(), int(ref_cost.item())


def test_two_calls_in_a_row_second_smaller():
    cases = [("matrix 2, N=64 ring sum, 1024 restarts", make_matrix(2), cc.CC_RING_SUM, 1024, WORKLOADS[2].search_seed),
             ("N=16 ring sum, 37 restarts", random_matrix(16, 991, symmetric=True, lo=1, hi=3000), cc.CC_RING_SUM, 37, 5)]
    for tag, c, obj, restarts, seed in cases:
        say(f"cc_2opt_search_noalloc: {tag}")
        perm, cost, ref_perm, ref_cost = _both(c, obj, restarts, seed)
        assert cost == ref_cost
        assert np.array_equal(perm, ref_perm)
        want = oracle.search(c, obj, restarts, seed)
        assert cost == want["best_cost"] and np.array_equal(perm, want["best_perm"])


def test_larger_sizes_then_smaller_every_kernel_family():
    """N = 256 (16-bit LDS matrix), N = 512 (matrix copy inside the static array), a directed max-hop search at
    N = 64 and a general-kernel size, each call smaller than the one before it."""
    cases = [("N=512 sum, 6 restarts", random_matrix(512, 12, symmetric=True, lo=1, hi=5000), cc.CC_RING_SUM, 6, 3),
             ("N=256 sum, 40 restarts", random_matrix(256, 13, symmetric=True, lo=1, hi=5000), cc.CC_RING_SUM, 40, 4),
             ("N=64 max directed, 200 restarts", make_matrix(3), cc.CC_RING_MAX_DIRECTED, 200, 9),
             ("N=33 sum directed, 11 restarts", random_matrix(33, 14, symmetric=False, lo=1, hi=70000),
              cc.CC_RING_SUM_DIRECTED, 11, 2)]
    for tag, c, obj, restarts, seed in cases:
        say(f"cc_2opt_search_noalloc: {tag}")
        perm, cost, ref_perm, ref_cost = _both(c, obj, restarts, seed)
        assert cost == ref_cost
        assert np.array_equal(perm, ref_perm)


def test_size_limit_is_an_error_and_launches_nothing():
    L = cc.lib()
    c = dev(make_matrix(2))
    best_perm = torch.full((64,), -7, dtype=torch.int32, device="cuda")
    best_cost = torch.full((1,), -7, dtype=torch.int64, device="cuda")
    limit = 8 << 20
    restarts = 1
    while cc.cc_2opt_workspace_bytes(64, 0, restarts * 2) <= limit:
        restarts *= 2
    while cc.cc_2opt_workspace_bytes(64, 0, restarts + 1) <= limit:
        restarts += 1
    say(f"cc_2opt_search_noalloc: limit at N=64 is {restarts} restarts")
    args = (ctypes.c_void_p(c.data_ptr()), 64, 0)
    tail = (ctypes.c_uint64(1), ctypes.c_void_p(best_perm.data_ptr()), ctypes.c_void_p(best_cost.data_ptr()),
            ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert L.cc_2opt_search_noalloc(*args, restarts + 1, *tail) == -7
    torch.cuda.synchronize()
    assert int(best_cost.item()) == -7 and bool((best_perm == -7).all())
    assert "scratch" in cc.cc_status_string(-7)
    assert L.cc_2opt_search_noalloc(*args, restarts, *tail) == 0          # the largest search that fits runs
    torch.cuda.synchronize()
    ref_perm, ref_cost = cc.cc_2opt_search(c, 0, restarts, 1)
    torch.cuda.synchronize()
    assert int(best_cost.item()) == int(ref_cost.item()) and torch.equal(best_perm, ref_perm)
