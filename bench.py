#!/usr/bin/env python3
"""Benchmark of the rank-order search hot path on one MI355X.

One step = one pass of the whole path on the N=64 workload, inputs resident in HBM:
  (1) cc_2opt_search_ex: 1024 seeded restarts of best-improvement 2-opt, ring sum objective, on the
      hierarchical 64-node RTT matrix (initial orders, staging, sweeps, argmin, moves), then
      cc_best_of_restarts (the search's last step, called on its own so that the search kernel's
      duration can be read from HIP events);
  (2) cc_ring_cost_batch, sum and max objectives, on 2^20 resident seeded orders;
  (3) cc_rd_cost_batch on 2^16 of the same orders.
`value` is 2-opt move evaluations per second over segment (1) (both calls) of the timed steps; the batch
throughput (orders per second, segments (2)) is reported beside it as `perm_evals_per_s`.  Segment
times come from HIP events recorded on the launch stream inside the timed region.

After the timed steps the same search kernel is also timed on 64 times the restarts (`roofline_saturated`: several
wavefronts per SIMD instead of one; --no-saturated skips it).

Prints ONE JSON line.  --gpus above 1 is refused: the search needs no second GPU (restarts are
independent) and this library runs on one.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

N_CU = 256
CLOCK_GHZ = 2.4
LDS_BYTES_PER_CLK_PER_CU = 128          # nominal ds_read_b32 rate: 64 lanes x 4 B every 2 clocks
LDS_PEAK_GBS = N_CU * LDS_BYTES_PER_CLK_PER_CU * CLOCK_GHZ          # 78643 GB/s
VALU_PEAK_GOPS = N_CU * 64 * CLOCK_GHZ                               # 39322 G int32 lane-ops/s
HBM_PEAK_GBS = 8000.0
LDS_MEASURED_B32_GBS = 72600.0          # conflict-free ds_read_b32 micro-kernel on this chip (92 % of nominal)
LDS_BYTES_PER_MOVE = 8                  # two int32 new-hop gathers per undirected move
VALU_OPS_PER_MOVE = 3                   # combine two gathers with the removed hops, form key, min
# HBM bytes per launch from rocprofv3 FETCH_SIZE (x 2.000) + WRITE_SIZE (x 1.000), calibrated on a 256 MiB copy
# (profiles/bench_n64_pmc_counters.md).  Set to None whenever the kernel changes after the counters were taken.
TRAFFIC_SEARCH_KERNEL_BYTES = (292.0 + 272.0) * 1024
TRAFFIC_RING_BATCH_BYTES = (262317.6 + 8196.2) * 1024


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-saturated", action="store_true",
                    help="skip the extra measurement after the timed steps (the same search kernel on 64x the "
                         "restarts, reported as roofline_saturated)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy before the steps (a dispatch of known HBM "
                         "traffic that scales rocprofv3's FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py runs on one GPU only: restarts and orders are independent, nothing is exchanged "
              "between devices, and this library has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2105_14088_amd as cc
    from paper_2105_14088_amd.build import build as build_library
    if not os.path.exists(cc.LIB_PATH):           # built in-tree beforehand as a rule; built here only when nothing is
        build_library(force=True)
    from gen import WORKLOADS, make_matrix

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = WORKLOADS[2]
    n, restarts, seed = w.n, w.restarts, w.search_seed
    batch = w.batch
    rd_batch = 1 << 16
    c_host = make_matrix(2)
    c = torch.from_numpy(c_host).cuda()
    orders = cc.cc_init_tours(n, batch, seed)
    out_sum = torch.empty(batch, dtype=torch.int64, device="cuda")
    out_max = torch.empty(batch, dtype=torch.int64, device="cuda")
    out_rd = torch.empty(rd_batch, dtype=torch.int64, device="cuda")
    bufs = cc.SearchBuffers(n, cc.CC_RING_SUM, restarts, c.device)
    torch.cuda.synchronize()

    def step(ev=None):
        if ev:
            ev[0].record()
        cc.cc_2opt_search_ex(c, cc.CC_RING_SUM, restarts, seed, buffers=bufs, pick_best=False)
        if ev:
            ev[1].record()
        cc.cc_best_of_restarts(bufs)
        if ev:
            ev[2].record()
        cc.cc_ring_cost_batch(c, orders, cc.CC_RING_SUM, out=out_sum)
        if ev:
            ev[3].record()
        cc.cc_ring_cost_batch(c, orders, cc.CC_RING_MAX, out=out_max)
        if ev:
            ev[4].record()
        cc.cc_rd_cost_batch(c, orders[:rd_batch], out=out_rd)
        if ev:
            ev[5].record()

    if args.pmc_calibration:
        cal_src = torch.zeros(64 << 20, dtype=torch.int32, device="cuda")
        cal_dst = torch.empty_like(cal_src)
        cal_dst.copy_(cal_src)
        torch.cuda.synchronize()
        del cal_src, cal_dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(events[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    seg = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(5)] for e in events])   # ms
    t_kernel, t_best, t_sum, t_max, t_rd = seg.mean(axis=0)
    t_search = t_kernel + t_best
    moves = bufs.restart_moves.cpu().numpy().astype(np.int64)
    nbhd = n * (n - 3) // 2
    move_evals = int(((moves + 1) * nbhd).sum())
    move_rate = move_evals / (t_search * 1e-3)
    perm_rate = 2 * batch / ((t_sum + t_max) * 1e-3)
    kernel_move_rate = move_evals / (t_kernel * 1e-3)      # the search kernel alone (roofline)
    lds_gbs = kernel_move_rate * LDS_BYTES_PER_MOVE / 1e9
    hbm_gbs = perm_rate * (4 * n + 8) / 1e9

    result = {
        "metric": "2-opt move evals/sec at N=64 (ring sum, 1024 restarts); permutation evals/sec beside it",
        "value": move_rate,
        "unit": "move evals/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32",
        "data": "synthetic",
        "config": {"workload": "C2: N=64 hierarchical symmetric RTT matrix (8 racks x 8), 1024 seeded 2-opt restarts, "
                               "ring sum; plus ring sum/max batch on 2^20 seeded orders and halving-doubling batch "
                               "on 2^16", "N": n, "restarts": restarts, "batch": batch, "rd_batch": rd_batch},
        "move_evals_per_step": move_evals,
        "applied_moves_per_step": int(moves.sum()),
        "best_cost": int(bufs.best_cost.item()),
        "segments_ms": {"search_2opt_kernel": t_kernel, "best_of_restarts": t_best, "ring_sum_batch": t_sum,
                        "ring_max_batch": t_max, "rd_batch": t_rd},
        "perm_evals_per_s": perm_rate,
        "rd_perm_evals_per_s": rd_batch / (t_rd * 1e-3),
        "roofline": {"kernel": "twoopt_sum_n64_kernel (2-opt search: neighbourhood sweep, argmin, apply)",
                     "kernel_ms": t_kernel, "bound": "lds", "achieved": lds_gbs,
                     "peak": LDS_PEAK_GBS, "unit": "GB/s", "frac": lds_gbs / LDS_PEAK_GBS,
                     "traffic": TRAFFIC_SEARCH_KERNEL_BYTES, "bytes_per_move": LDS_BYTES_PER_MOVE,
                     "frac_of_measured_b32_peak": lds_gbs / LDS_MEASURED_B32_GBS,
                     "valu": {"achieved": kernel_move_rate * VALU_OPS_PER_MOVE / 1e9, "peak": VALU_PEAK_GOPS,
                              "unit": "G lane-ops/s",
                              "frac": kernel_move_rate * VALU_OPS_PER_MOVE / 1e9 / VALU_PEAK_GOPS,
                              "ops_per_move": VALU_OPS_PER_MOVE}},
        "roofline_batch": {"kernel": "ring cost batch", "bound": "hbm", "achieved": hbm_gbs, "peak": HBM_PEAK_GBS,
                           "unit": "GB/s", "frac": hbm_gbs / HBM_PEAK_GBS, "traffic": TRAFFIC_RING_BATCH_BYTES,
                           "bytes_per_perm": 4 * n + 8},
    }

    if not args.no_saturated:
        # The same kernel with every SIMD holding several wavefronts (outside the timed steps): 64 times the restarts.
        sat_restarts = 64 * restarts
        sat_bufs = cc.SearchBuffers(n, cc.CC_RING_SUM, sat_restarts, c.device)
        cc.cc_2opt_search_ex(c, cc.CC_RING_SUM, sat_restarts, seed, buffers=sat_bufs, pick_best=False)
        torch.cuda.synchronize()
        sat_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(5)]
        for e0, e1 in sat_ev:
            e0.record()
            cc.cc_2opt_search_ex(c, cc.CC_RING_SUM, sat_restarts, seed, buffers=sat_bufs, pick_best=False)
            e1.record()
        torch.cuda.synchronize()
        sat_ms = float(np.median([e0.elapsed_time(e1) for e0, e1 in sat_ev]))
        sat_evals = int(((sat_bufs.restart_moves.cpu().numpy().astype(np.int64) + 1) * nbhd).sum())
        sat_gbs = sat_evals / (sat_ms * 1e-3) * LDS_BYTES_PER_MOVE / 1e9
        result["roofline_saturated"] = {"kernel": "2-opt search (neighbourhood sweep), same kernel", "restarts": sat_restarts,
                                        "ms": sat_ms, "move_evals_per_s": sat_evals / (sat_ms * 1e-3), "bound": "lds",
                                        "achieved": sat_gbs, "peak": LDS_PEAK_GBS, "unit": "GB/s",
                                        "frac": sat_gbs / LDS_PEAK_GBS,
                                        "note": "not the metric's configuration: 1024 restarts put one wavefront on each "
                                                "of the 1024 SIMDs, where instruction issue latency bounds the kernel"}
        del sat_bufs

    if not args.no_cpu_baseline:
        import oracle
        t1 = time.perf_counter()
        oc, ot, om = oracle.restarts(c_host, oracle.SUM, seed, 0, restarts)
        dt = time.perf_counter() - t1
        assert np.array_equal(om, moves) and np.array_equal(oc, bufs.restart_costs.cpu().numpy())
        sample = orders[:1 << 16].cpu().numpy()
        t2 = time.perf_counter()
        oracle.ring_cost_batch(c_host, sample, oracle.SUM)
        dt2 = time.perf_counter() - t2
        result["cpu_baseline"] = {"value": move_evals / dt, "unit": "move evals/s", "cores": 1, "kind": "oracle",
                                  "sample": f"all {restarts} restarts of the same search, single thread, {dt:.2f} s; "
                                            f"ring batch on 65536 orders: {(1 << 16) / dt2:.3e} perm evals/s",
                                  "perm_evals_per_s": (1 << 16) / dt2}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
