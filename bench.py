#!/usr/bin/env python3
"""Benchmark of the rank-order search hot path on one MI355X.

One step = one pass of the whole path on the N=64 workloads, inputs resident in HBM:
  (1) cc_2opt_search_ex, one call as the library's users issue it: 1024 seeded restarts of best-improvement 2-opt,
      ring sum objective, on the hierarchical symmetric 64-node RTT matrix (initial orders, staging, sweeps, argmin,
      moves, winner selection);
  (2) the same call on the asymmetric 64-node bandwidth-cost matrix under the directed max-hop objective
      (1024 restarts, every move scored for both walking directions);
  (3) cc_ring_cost_batch, sum and max objectives, on 2^20 resident seeded orders;
  (4) cc_rd_cost_batch on 2^16 of the same orders.
`value` is 2-opt move evaluations per second of segment (1), the configuration the metric is quoted on; the
directed max-hop rate (`move_evals_per_s_c3`) and the batch rate (`perm_evals_per_s`, segments (3)) stand beside
it.  Segment times come from HIP events recorded on the launch stream inside the timed region.

After the timed steps, each of its own and evented launch by launch on the same stream:
  - the two search kernels alone (the search calls without winner selection), the launches back to back between one
    pair of events (`kernel_ms` = the average launch duration that `frac` is computed from; it is the figure the
    profiler reports for the kernel) and every launch between a pair of its own (`kernel_ms_with_own_events`, 2 us
    more: the events' own cost): `roofline`, `roofline_c3`;
  - the ring-sum search kernel on 64 times the restarts (`roofline_saturated`; --no-saturated skips it);
  - the ring batch on 2^22 orders, a 1 GiB stream that cannot sit in the 256 MB last-level cache
    (`roofline_batch.cold`; --no-cold skips it);
  - the CPU oracle on the host's cores (`cpu_baseline`; --no-cpu-baseline skips it).

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
# Algorithmic LDS bytes per move evaluation: the two new hops of a 2-opt move as int32 matrix entries (undirected),
# four for a directed move (both walking directions); half of that where the kernel keeps 16-bit entries.
LDS_BYTES_PER_MOVE = 8
LDS_BYTES_PER_DIRECTED_MOVE = 16
LDS_BYTES_PER_DIRECTED_MOVE_PACKED = 8
VALU_OPS_PER_MOVE = 3                   # combine two gathers with the removed hops, form key, min
# rocprofv3 counter readings per launch (profiles/bench_n64_pmc_counters.md), valid for the kernels as they stood
# when the counters were taken; None once a kernel has changed since.
#   LDS: SQ_INSTS_LDS wave instructions per launch x 256 B (64 lanes x 4 B) = bytes the kernel moved through LDS
#   HBM: FETCH_SIZE (x 2.000) + WRITE_SIZE (x 1.000) KiB, scale factors from a plain 256 MiB device copy
COUNTERS = {
    "search_sum_lds_insts": 2263348,                       # twoopt_sum_n64_kernel, 1024 restarts of workload 2
    "search_sum_hbm_bytes": (120.0 * 2 + 272.0) * 1024,
    "search_max_lds_insts": 840968,                        # twoopt_max_n64_kernel, 1024 restarts of workload 3
    "search_max_hbm_bytes": (148.5 * 2 + 272.0) * 1024,
    "ring_batch_hbm_bytes": (131158.5 * 2 + 8195.9) * 1024,        # 2^20 orders
    "ring_batch_cold_hbm_bytes": (524374.5 * 2 + 32779.3) * 1024,  # 2^22 orders
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-saturated", action="store_true",
                    help="skip the extra measurement after the timed steps (the same search kernel on 64x the "
                         "restarts, reported as roofline_saturated)")
    ap.add_argument("--no-cold", action="store_true",
                    help="skip the ring batch on 2^22 orders (1 GiB stream, roofline_batch.cold)")
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
    w3 = WORKLOADS[3]
    assert (w3.n, w3.restarts) == (n, restarts)
    seed3 = w3.search_seed
    batch = w.batch
    rd_batch = 1 << 16
    c_host = make_matrix(2)
    c3_host = make_matrix(3)
    c = torch.from_numpy(c_host).cuda()
    c3 = torch.from_numpy(c3_host).cuda()
    orders = cc.cc_init_tours(n, batch, seed)
    out_sum = torch.empty(batch, dtype=torch.int64, device="cuda")
    out_max = torch.empty(batch, dtype=torch.int64, device="cuda")
    out_rd = torch.empty(rd_batch, dtype=torch.int64, device="cuda")
    bufs = cc.SearchBuffers(n, cc.CC_RING_SUM, restarts, c.device)
    bufs3 = cc.SearchBuffers(n, cc.CC_RING_MAX_DIRECTED, restarts, c.device)
    torch.cuda.synchronize()

    def step(ev=None):
        if ev:
            ev[0].record()
        cc.cc_2opt_search_ex(c, cc.CC_RING_SUM, restarts, seed, buffers=bufs)
        if ev:
            ev[1].record()
        cc.cc_2opt_search_ex(c3, cc.CC_RING_MAX_DIRECTED, restarts, seed3, buffers=bufs3)
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

    def evented(fn, reps):
        """Mean duration in ms of `reps` calls of fn, each bracketed by its own pair of HIP events."""
        fn()
        torch.cuda.synchronize()
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for e0, e1 in pairs:
            e0.record()
            fn()
            e1.record()
        torch.cuda.synchronize()
        return float(np.mean([e0.elapsed_time(e1) for e0, e1 in pairs]))

    def back_to_back(fn, reps):
        """Mean duration in ms of `reps` calls of fn issued back to back between ONE pair of HIP events: without the
        few microseconds that an event of its own adds to every launch."""
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

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
    t_search, t_search3, t_sum, t_max, t_rd = seg.mean(axis=0)
    moves = bufs.restart_moves.cpu().numpy().astype(np.int64)
    moves3 = bufs3.restart_moves.cpu().numpy().astype(np.int64)
    nbhd = n * (n - 3) // 2
    move_evals = int(((moves + 1) * nbhd).sum())
    move_evals3 = int(((moves3 + 1) * 2 * nbhd).sum())
    move_rate = move_evals / (t_search * 1e-3)
    move_rate3 = move_evals3 / (t_search3 * 1e-3)
    perm_rate = 2 * batch / ((t_sum + t_max) * 1e-3)
    hbm_gbs = perm_rate * (4 * n + 8) / 1e9

    # the search kernels alone: the same calls without winner selection, one kernel launch each
    reps = max(args.steps, 10)
    t_kernel_own = evented(lambda: cc.cc_2opt_search_ex(c, cc.CC_RING_SUM, restarts, seed, buffers=bufs,
                                                        pick_best=False), reps)
    t_kernel3_own = evented(lambda: cc.cc_2opt_search_ex(c3, cc.CC_RING_MAX_DIRECTED, restarts, seed3, buffers=bufs3,
                                                         pick_best=False), reps)
    t_kernel = back_to_back(lambda: cc.cc_2opt_search_ex(c, cc.CC_RING_SUM, restarts, seed, buffers=bufs,
                                                             pick_best=False), reps)
    t_kernel3 = back_to_back(lambda: cc.cc_2opt_search_ex(c3, cc.CC_RING_MAX_DIRECTED, restarts, seed3,
                                                              buffers=bufs3, pick_best=False), reps)
    kernel_move_rate = move_evals / (t_kernel * 1e-3)
    kernel_move_rate3 = move_evals3 / (t_kernel3 * 1e-3)
    lds_gbs = kernel_move_rate * LDS_BYTES_PER_MOVE / 1e9
    lds_gbs3 = kernel_move_rate3 * LDS_BYTES_PER_DIRECTED_MOVE / 1e9
    lds_gbs3_packed = kernel_move_rate3 * LDS_BYTES_PER_DIRECTED_MOVE_PACKED / 1e9
    sweeps = int((moves + 1).sum())
    sweeps3 = int((moves3 + 1).sum())

    def lds_traffic(key):
        return None if COUNTERS[key] is None else COUNTERS[key] * 256.0

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
                               "ring sum (the metric's configuration); in the same step C3: N=64 asymmetric "
                               "bandwidth-cost matrix, directed max-hop, 1024 restarts; ring sum/max batch on 2^20 "
                               "seeded orders; halving-doubling batch on 2^16",
                   "N": n, "restarts": restarts, "batch": batch, "rd_batch": rd_batch},
        "move_evals_per_step": move_evals,
        "applied_moves_per_step": int(moves.sum()),
        "sweeps_per_restart": {"mean": float((moves + 1).mean()), "max": int((moves + 1).max())},
        "best_cost": int(bufs.best_cost.item()),
        "move_evals_per_s_c3": move_rate3,
        "move_evals_per_step_c3": move_evals3,
        "best_cost_c3": int(bufs3.best_cost.item()),
        "segments_ms": {"search_2opt_sum": t_search, "search_2opt_max_directed": t_search3, "ring_sum_batch": t_sum,
                        "ring_max_batch": t_max, "rd_batch": t_rd},
        "perm_evals_per_s": perm_rate,
        "rd_perm_evals_per_s": rd_batch / (t_rd * 1e-3),
        "roofline": {"kernel": "twoopt_sum_n64_kernel (2-opt search: neighbourhood sweep, argmin, apply)",
                     "kernel_ms": t_kernel, "launches": reps,
                     "kernel_ms_with_own_events": t_kernel_own,
                     "frac_with_own_events": move_evals / (t_kernel_own * 1e-3) * LDS_BYTES_PER_MOVE / 1e9 / LDS_PEAK_GBS,
                     "bound": "lds", "achieved": lds_gbs,
                     "peak": LDS_PEAK_GBS, "unit": "GB/s", "frac": lds_gbs / LDS_PEAK_GBS,
                     "bytes_per_move": LDS_BYTES_PER_MOVE,
                     "traffic": lds_traffic("search_sum_lds_insts"),
                     "traffic_kind": "bytes moved through LDS per launch: SQ_INSTS_LDS x 256 B (the kernel issues one "
                                     "4-byte gather per move; the second new hop of a move is the neighbouring "
                                     "lane's gather)",
                     "hbm_traffic": COUNTERS["search_sum_hbm_bytes"],
                     "issued_lds_bytes_per_move": 4,
                     "frac_issued": kernel_move_rate * 4 / 1e9 / LDS_PEAK_GBS,
                     "frac_of_measured_b32_peak": lds_gbs / LDS_MEASURED_B32_GBS,
                     "ns_per_sweep_longest_restart": t_kernel * 1e6 / int((moves + 1).max()),
                     "sweeps_per_launch": sweeps,
                     "valu": {"achieved": kernel_move_rate * VALU_OPS_PER_MOVE / 1e9, "peak": VALU_PEAK_GOPS,
                              "unit": "G lane-ops/s",
                              "frac": kernel_move_rate * VALU_OPS_PER_MOVE / 1e9 / VALU_PEAK_GOPS,
                              "ops_per_move": VALU_OPS_PER_MOVE}},
        "roofline_c3": {"kernel": "twoopt_max_n64_kernel (directed max-hop 2-opt search, packed 16-bit entries)",
                        "kernel_ms": t_kernel3, "launches": reps, "kernel_ms_with_own_events": t_kernel3_own,
                        "move_evals_per_s": kernel_move_rate3,
                        "bound": "lds", "achieved": lds_gbs3, "peak": LDS_PEAK_GBS, "unit": "GB/s",
                        "frac": lds_gbs3 / LDS_PEAK_GBS, "bytes_per_move": LDS_BYTES_PER_DIRECTED_MOVE,
                        "frac_at_storage_width": lds_gbs3_packed / LDS_PEAK_GBS,
                        "bytes_per_move_at_storage_width": LDS_BYTES_PER_DIRECTED_MOVE_PACKED,
                        "traffic": lds_traffic("search_max_lds_insts"),
                        "traffic_kind": "bytes moved through LDS per launch: SQ_INSTS_LDS x 256 B (one packed gather "
                                        "per move delivers both directions of a pair)",
                        "hbm_traffic": COUNTERS["search_max_hbm_bytes"],
                        "sweeps_per_launch": sweeps3,
                        "sweeps_per_restart": {"mean": float((moves3 + 1).mean()), "max": int((moves3 + 1).max())},
                        "ns_per_sweep_longest_restart": t_kernel3 * 1e6 / int((moves3 + 1).max())},
        "roofline_batch": {"kernel": "ring cost batch (ring_batch_lds_kernel<64>)", "bound": "hbm", "achieved": hbm_gbs,
                           "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": hbm_gbs / HBM_PEAK_GBS,
                           "traffic": COUNTERS["ring_batch_hbm_bytes"], "bytes_per_perm": 4 * n + 8,
                           "note": "sum and max calls back to back on one 268 MB order buffer: part of the stream "
                                   "can come from the 256 MB last-level cache; `cold` cannot"},
    }

    if not args.no_cold:
        # 2^22 orders = 1 GiB of int32 ranks: four times the last-level cache, so every pass streams from HBM
        cold_batch = 1 << 22
        cold_orders = cc.cc_init_tours(n, cold_batch, seed + 1)
        cold_out = torch.empty(cold_batch, dtype=torch.int64, device="cuda")
        cold_ms = evented(lambda: cc.cc_ring_cost_batch(c, cold_orders, cc.CC_RING_SUM, out=cold_out), 5)
        cold_gbs = cold_batch * (4 * n + 8) / (cold_ms * 1e-3) / 1e9
        result["roofline_batch"]["cold"] = {"batch": cold_batch, "ms": cold_ms, "achieved": cold_gbs,
                                            "frac": cold_gbs / HBM_PEAK_GBS,
                                            "perm_evals_per_s": cold_batch / (cold_ms * 1e-3),
                                            "traffic": COUNTERS["ring_batch_cold_hbm_bytes"]}
        result["roofline_batch"]["frac_cold"] = cold_gbs / HBM_PEAK_GBS
        del cold_orders, cold_out

    if not args.no_saturated:
        # The same kernel with every SIMD holding several wavefronts (outside the timed steps): 64 times the restarts.
        sat_restarts = 64 * restarts
        sat_bufs = cc.SearchBuffers(n, cc.CC_RING_SUM, sat_restarts, c.device)
        sat_ms = evented(lambda: cc.cc_2opt_search_ex(c, cc.CC_RING_SUM, sat_restarts, seed, buffers=sat_bufs,
                                                      pick_best=False), 5)
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
