"""The workspace forms of the calls enqueue kernels only (no allocation, no memset), so a step can be captured in a
HIP graph and replayed: every replay must reproduce the eager results, with eager work in between."""
import numpy as np
import pytest
import torch

import oracle
import paper_2105_14088_amd as cc
from gen import WORKLOADS, make_matrix
from gpu_util import say

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("built_library")]


def test_search_and_batch_calls_replay_in_a_graph():
    say("HIP graph: capture cc_2opt_search_ex + cc_best_of_restarts + ring / halving-doubling batches, replay 4 times")
    c_host = make_matrix(2)
    c = torch.from_numpy(c_host).cuda()
    seed, restarts, batch = WORKLOADS[2].search_seed, 64, 4096
    orders = cc.cc_init_tours(64, batch, seed)
    bufs = cc.SearchBuffers(64, cc.CC_RING_SUM, restarts, c.device)
    out_ring = torch.empty(batch, dtype=torch.int64, device="cuda")
    out_rd = torch.empty(batch, dtype=torch.int64, device="cuda")

    def step():
        cc.cc_2opt_search_ex(c, cc.CC_RING_SUM, restarts, seed, buffers=bufs, pick_best=False)
        cc.cc_best_of_restarts(bufs)
        cc.cc_ring_cost_batch(c, orders, cc.CC_RING_SUM, out=out_ring)
        cc.cc_rd_cost_batch(c, orders, out=out_rd)

    step()                                   # eager reference (also loads the kernels before capture)
    torch.cuda.synchronize()
    want = [t.clone() for t in (bufs.restart_costs, bufs.restart_tours, bufs.restart_moves, bufs.best_perm,
                                bufs.best_cost, out_ring, out_rd)]
    ref = oracle.search(c_host, oracle.SUM, restarts, seed)
    assert np.array_equal(want[0].cpu().numpy(), ref["costs"]) and int(want[4].item()) == ref["best_cost"]

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for replay in range(4):
        for t in (bufs.restart_costs, bufs.restart_tours, bufs.restart_moves, bufs.best_perm, bufs.best_cost, out_ring,
                  out_rd):
            t.fill_(-1)                       # eager work between replays; also proves the replay rewrites everything
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (bufs.restart_costs, bufs.restart_tours, bufs.restart_moves, bufs.best_perm, bufs.best_cost, out_ring,
               out_rd)
        for g, w in zip(got, want):
            assert torch.equal(g, w), f"replay {replay}"


def test_local_search_replays_in_a_graph():
    """cc_local_search_ex: seeded starts, the matrix-maximum kernel, the wavefront kernel and the skipped general
    kernel (N = 64), and the general kernel alone (N = 100), all inside one captured step."""
    say("HIP graph: capture cc_local_search_ex at N = 64 and N = 100, replay 3 times")
    both = cc.CC_MOVES_2OPT | cc.CC_MOVES_OROPT
    c64_host = make_matrix(2)
    c64 = torch.from_numpy(c64_host).cuda()
    from gen import random_matrix
    c100_host = random_matrix(100, 5, symmetric=True, lo=1, hi=3000)
    c100 = torch.from_numpy(c100_host).cuda()
    b64 = cc.SearchBuffers(64, cc.CC_RING_SUM, 48, c64.device)
    b100 = cc.SearchBuffers(100, cc.CC_RING_SUM, 12, c64.device)

    def step():
        cc.cc_local_search_ex(c64, cc.CC_RING_SUM, both, 48, 11, buffers=b64)
        cc.cc_local_search_ex(c100, cc.CC_RING_SUM, cc.CC_MOVES_OROPT, 12, 12, buffers=b100)

    step()
    torch.cuda.synchronize()
    outs = (b64.restart_costs, b64.restart_tours, b64.restart_moves, b64.best_perm, b64.best_cost, b64.best_restart,
            b100.restart_costs, b100.restart_tours, b100.restart_moves, b100.best_perm, b100.best_cost)
    want = [t.clone() for t in outs]
    ref64 = oracle.local_search(c64_host, oracle.SUM, both, 48, 11)
    ref100 = oracle.local_search(c100_host, oracle.SUM, oracle.MOVES_OROPT, 12, 12)
    assert np.array_equal(want[1].cpu().numpy(), ref64["tours"]) and np.array_equal(want[7].cpu().numpy(), ref100["tours"])

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for replay in range(3):
        for t in outs:
            t.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for g, w in zip(outs, want):
            assert torch.equal(g, w), f"replay {replay}"


def test_other_searches_replay_in_a_graph():
    """The remaining search calls and the workspace forms of the batch calls inside one captured step: pair swaps at N = 64 (wavefront kernel) and N = 256
    (workgroup kernel with its 128 KiB of LDS, folded matrix, skipped general kernel), the directed ring sum at
    N = 64 (seeded starts, matrix maximum, wavefront kernel, skipped general kernel), and both annealing calls."""
    say("HIP graph: capture pair-swap searches, a directed-sum search and annealing, replay 3 times")
    from gen import random_matrix
    c64_host = make_matrix(2)
    c3_host = make_matrix(3)
    c256_host = random_matrix(256, 17, symmetric=False, lo=1, hi=9000)
    c64, c3, c256 = (torch.from_numpy(x).cuda() for x in (c64_host, c3_host, c256_host))
    dev = c64.device
    b_swap64 = cc.SearchBuffers(64, 0, 40, dev)
    b_swap256 = cc.SearchBuffers(256, 0, 2, dev)
    b_dsum = cc.SearchBuffers(64, cc.CC_RING_SUM_DIRECTED, 40, dev)
    b_sa = cc.SearchBuffers(64, 0, 8, dev)
    b_sard = cc.SearchBuffers(64, 0, 8, dev)

    orders = cc.cc_init_tours(256, 300, 26)
    ws_batch = torch.empty(cc.cc_rd_batch_workspace_bytes(256), dtype=torch.uint8, device=dev)
    out_rd = torch.empty(300, dtype=torch.int64, device=dev)
    out_bcube = torch.empty(300, dtype=torch.int64, device=dev)

    def step():
        cc.cc_rd_cost_batch(c256, orders, out=out_rd, workspace=ws_batch)          # folded-matrix forms
        cc.cc_bcube_cost_batch(c256, 4, orders, out=out_bcube, workspace=ws_batch)
        cc.cc_rd_swap_search_ex(c64, 40, 21, buffers=b_swap64)
        cc.cc_rd_swap_search_ex(c256, 2, 22, buffers=b_swap256)
        cc.cc_2opt_search_ex(c3, cc.CC_RING_SUM_DIRECTED, 40, 23, buffers=b_dsum)
        cc.cc_sa_search_ex(c64, 8, 3000, 300, 0, 24, buffers=b_sa)
        cc.cc_sa_rd_search_ex(c64, 8, 2000, 300, 0, 25, buffers=b_sard)

    step()
    torch.cuda.synchronize()
    bufs = (b_swap64, b_swap256, b_dsum, b_sa, b_sard)
    outs = [t for b in bufs for t in (b.restart_costs, b.restart_tours, b.restart_moves, b.best_perm, b.best_cost,
                                       b.best_restart)]
    outs += [out_rd, out_bcube]
    want = [t.clone() for t in outs]
    orders_host = orders.cpu().numpy()
    assert np.array_equal(out_rd.cpu().numpy(), oracle.rd_cost_batch(c256_host, orders_host))
    assert np.array_equal(out_bcube.cpu().numpy(), oracle.bcube_cost_batch(c256_host, 4, orders_host))
    refs = (oracle.rd_swap_search(c64_host, 40, 21), oracle.rd_swap_search(c256_host, 2, 22),
            oracle.search(c3_host, oracle.SUM_DIRECTED, 40, 23), oracle.sa_search(c64_host, 8, 3000, 300, 0, 24),
            oracle.sa_rd_search(c64_host, 8, 2000, 300, 0, 25))
    for b, ref in zip(bufs, refs):
        assert np.array_equal(b.restart_tours.cpu().numpy(), ref["tours"])
        assert int(b.best_cost.item()) == ref["best_cost"]

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for replay in range(3):
        for t in outs:
            t.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for g, w in zip(outs, want):
            assert torch.equal(g, w), f"replay {replay}"


def test_searches_at_128_to_512_replay_in_a_graph():
    """The kernels for the larger sizes inside one captured step: max-hop (directed and not) at N = 256, the directed
    ring sum at N = 128 (each with its matrix maximum, the multi-rank kernel and the skipped general kernel), pair swaps at
    N = 512 (folded copy, LDS tiles), and the 2-opt search on the library's static scratch array."""
    say("HIP graph: capture max-hop and directed-sum searches at N = 128 / 256, pair swaps at N = 512, the no-allocation search")
    from gen import random_matrix
    c256_host = random_matrix(256, 61, symmetric=True, lo=1, hi=9000)
    a256_host = random_matrix(256, 62, symmetric=False, lo=1, hi=9000)
    a128_host = random_matrix(128, 63, symmetric=False, lo=1, hi=9000)
    c512_host = random_matrix(512, 64, symmetric=True, lo=1, hi=9000)
    c64_host = make_matrix(2)
    c256, a256, a128, c512, c64 = (torch.from_numpy(x).cuda() for x in (c256_host, a256_host, a128_host, c512_host, c64_host))
    dev = c256.device
    b_max = cc.SearchBuffers(256, cc.CC_RING_MAX, 6, dev)
    b_maxd = cc.SearchBuffers(256, cc.CC_RING_MAX_DIRECTED, 5, dev)
    b_dsum = cc.SearchBuffers(128, cc.CC_RING_SUM_DIRECTED, 7, dev)
    b_swap = cc.SearchBuffers(512, 0, 1, dev)
    na_perm = torch.empty(64, dtype=torch.int32, device=dev)
    na_cost = torch.empty(1, dtype=torch.int64, device=dev)

    def step():
        cc.cc_2opt_search_ex(c256, cc.CC_RING_MAX, 6, 31, buffers=b_max)
        cc.cc_2opt_search_ex(a256, cc.CC_RING_MAX_DIRECTED, 5, 32, buffers=b_maxd)
        cc.cc_2opt_search_ex(a128, cc.CC_RING_SUM_DIRECTED, 7, 33, buffers=b_dsum)
        cc.cc_rd_swap_search_ex(c512, 1, 34, buffers=b_swap)
        cc.cc_2opt_search_noalloc(c64, cc.CC_RING_SUM, 50, 35, na_perm, na_cost)

    step()                                   # also the first call of the no-allocation entry on this device
    torch.cuda.synchronize()
    bufs = (b_max, b_maxd, b_dsum, b_swap)
    outs = [t for b in bufs for t in (b.restart_costs, b.restart_tours, b.restart_moves, b.best_perm, b.best_cost,
                                       b.best_restart)]
    outs += [na_perm, na_cost]
    want = [t.clone() for t in outs]
    refs = (oracle.search(c256_host, oracle.MAX, 6, 31), oracle.search(a256_host, oracle.MAX_DIRECTED, 5, 32),
            oracle.search(a128_host, oracle.SUM_DIRECTED, 7, 33), oracle.rd_swap_search(c512_host, 1, 34))
    for b, ref in zip(bufs, refs):
        assert np.array_equal(b.restart_tours.cpu().numpy(), ref["tours"])
        assert int(b.best_cost.item()) == ref["best_cost"]
    ref = oracle.search(c64_host, oracle.SUM, 50, 35)
    assert np.array_equal(na_perm.cpu().numpy(), ref["best_perm"]) and int(na_cost.item()) == ref["best_cost"]

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for replay in range(3):
        for t in outs:
            t.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for g, w in zip(outs, want):
            assert torch.equal(g, w), f"replay {replay}"
