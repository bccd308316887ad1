"""The workspace forms of the calls enqueue kernels only (no allocation, no memset), so a step can be captured in a
HIP graph and replayed: every replay must reproduce the eager results, with eager work in between."""
import numpy as np
import pytest
import torch

import oracle
import paper_2105_14088_amd as cc
from gen import WORKLOADS, make_matrix
from gpu_util import say

pytestmark = pytest.mark.gpu


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
