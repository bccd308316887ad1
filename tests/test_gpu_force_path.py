"""CC_FORCE_PATH=general pins every search call to its general kernel.  Full-size A/B of the specialised kernels
against the general ones on the workload matrices (the general kernels are otherwise reached only through matrix
entries of 2^16 and more, or sizes without a specialised kernel), and parity of the general kernels with the oracle."""
import os
import time

import numpy as np
import pytest
import torch

import oracle
import paper_2105_14088_amd as cc
from gen import WORKLOADS, make_matrix
from gpu_util import assert_search_equal, dev, gpu_search, report, say

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("built_library")]
THREADS = min(16, os.cpu_count() or 1)


@pytest.fixture
def pinned():
    old = os.environ.get("CC_FORCE_PATH")
    os.environ["CC_FORCE_PATH"] = "general"
    yield
    if old is None:
        del os.environ["CC_FORCE_PATH"]
    else:
        os.environ["CC_FORCE_PATH"] = old


def _timed_search(c, obj, restarts, seed):
    cd = dev(c)
    bufs = cc.SearchBuffers(c.shape[0], obj, restarts, cd.device)
    cc.cc_2opt_search_ex(cd, obj, restarts, seed, buffers=bufs)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    cc.cc_2opt_search_ex(cd, obj, restarts, seed, buffers=bufs)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1)


@pytest.mark.parametrize("wid,obj", [(2, 0), (3, 3), (3, 2), (3, 1), (4, 0)])
def test_general_kernel_equals_fast_path_and_oracle_at_full_size(wid, obj, pinned):
    w = WORKLOADS[wid]
    c = make_matrix(wid)
    if obj == 1:
        c = np.maximum(c, c.T)          # the undirected max-hop objective wants a symmetric matrix
    restarts, seed = w.restarts, w.search_seed
    say(f"pinned general kernel: matrix {wid} objective {obj}, {restarts} restarts")
    got = gpu_search(c, obj, restarts, seed)
    ms_general = _timed_search(c, obj, restarts, seed)
    del os.environ["CC_FORCE_PATH"]
    fast = gpu_search(c, obj, restarts, seed)
    ms_fast = _timed_search(c, obj, restarts, seed)
    os.environ["CC_FORCE_PATH"] = "general"
    assert_search_equal(got, fast)
    t0 = time.time()
    costs, tours, moves = oracle.restarts_parallel(c, obj, seed, 0, restarts, THREADS)
    assert np.array_equal(got["costs"], costs) and np.array_equal(got["moves"], moves)
    assert np.array_equal(got["tours"], tours)
    report(f"matrix {wid} objective {obj}: general kernel {ms_general:.3f} ms, specialised path {ms_fast:.3f} ms, "
           f"all {restarts} restarts equal to the oracle ({time.time() - t0:.1f} s on {THREADS} threads)")


def test_wider_move_sets_and_pair_swaps_pinned(pinned):
    c = make_matrix(2)
    seed = WORKLOADS[2].search_seed
    both = cc.CC_MOVES_2OPT | cc.CC_MOVES_OROPT
    say("pinned general kernels: 2-opt + insertion and pair swaps on matrix 2, 128 restarts")
    b = cc.cc_local_search_ex(dev(c), 0, both, 128, seed)
    torch.cuda.synchronize()
    want = oracle.local_search(c, 0, both, 128, seed)
    assert np.array_equal(b.restart_costs.cpu().numpy(), want["costs"])
    assert np.array_equal(b.restart_tours.cpu().numpy(), want["tours"])
    s = cc.cc_rd_swap_search_ex(dev(c), 128, seed)
    torch.cuda.synchronize()
    want = oracle.rd_swap_search(c, 128, seed)
    assert np.array_equal(s.restart_costs.cpu().numpy(), want["costs"])
    assert np.array_equal(s.restart_tours.cpu().numpy(), want["tours"])
    c3 = make_matrix(3)
    f = cc.cc_local_search_ex(dev(c3), 3, cc.CC_MOVES_2OPT | cc.CC_MOVES_FLIP, 128, 7)
    torch.cuda.synchronize()
    want = oracle.local_search(c3, 3, cc.CC_MOVES_2OPT | cc.CC_MOVES_FLIP, 128, 7)
    assert np.array_equal(f.restart_costs.cpu().numpy(), want["costs"])
    assert np.array_equal(f.restart_tours.cpu().numpy(), want["tours"])
