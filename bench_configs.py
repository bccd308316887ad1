#!/usr/bin/env python3
"""Times every workload of the rank-order search on one MI355X and prints one JSON line per workload.

Cases: C1-C5 the parity-test configurations (matrix shapes and work amounts in gen/workloads.py); M64* the
batch-evaluation headline case (ring sum / max on 2^20 seeded orders at N=64, also with orders stored one byte
per rank); R/B/T* halving-doubling, BCube and double-binary-tree batches; S* pair-swap searches under the
halving-doubling model; L* ring searches over the wider move sets (segment insertion, orientation flip); A* / AR* simulated-annealing runs (ring / halving-doubling); P* cost matrices from
probes.  Times are HIP-event times around the library call on the launch stream, median of `--reps` after one
warm-up.  `bench.py` remains the single-line benchmark of the N=64 workload.  Pass --oracle to time the CPU
oracle beside each case (a bounded sample, one core) and compare the sample bit for bit; --only takes a
comma-separated list of case keys.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def timed(fn, reps):
    import torch
    fn()
    torch.cuda.synchronize()
    ts = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1))
    ts.sort()
    return ts[len(ts) // 2]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--oracle", action="store_true")
    ap.add_argument("--only", type=str, default="")
    args = ap.parse_args()

    import numpy as np
    import torch

    import paper_2105_14088_amd as cc
    from gen import WORKLOADS, make_matrix

    torch.cuda.set_device(0)
    only = set(args.only.split(",")) if args.only else None

    def emit(d):
        print(json.dumps(d), flush=True)

    def search_case(wid, n=None, restarts=None, name=None, objective=None):
        w = WORKLOADS[wid]
        if objective is not None:  # the workload's matrix and restarts under another objective
            import dataclasses
            w = dataclasses.replace(w, objective=objective, name=name, restarts=restarts or w.restarts)
        obj = cc.OBJECTIVES[w.objective]
        c_host = make_matrix(wid)
        if n is not None:         # the workload's hierarchy and value ranges at another size
            from gen import hierarchical_matrix
            import dataclasses
            c_host = hierarchical_matrix(n, w.group_sizes, w.level_ranges, w.sigma, True, w.matrix_seed + n)
            w = dataclasses.replace(w, n=n, restarts=restarts, name=name)
        c = torch.from_numpy(c_host).cuda()
        bufs = cc.SearchBuffers(w.n, obj, w.restarts, c.device)
        ms = timed(lambda: cc.cc_2opt_search_ex(c, obj, w.restarts, w.search_seed, buffers=bufs), args.reps)
        moves = bufs.restart_moves.cpu().numpy().astype(np.int64)
        nbhd = w.n * (w.n - 3) // 2 * (2 if obj & 2 else 1)
        evals = int(((moves + 1) * nbhd).sum())
        d = {"workload": w.name, "call": "cc_2opt_search_ex", "N": w.n, "objective": w.objective,
             "restarts": w.restarts, "ms": ms, "move_evals": evals, "move_evals_per_s": evals / (ms * 1e-3),
             "applied_moves_mean": float(moves.mean()), "applied_moves_max": int(moves.max()),
             "best_cost": int(bufs.best_cost.item())}
        if args.oracle:
            import oracle
            sample = min(w.restarts, 256 if w.n <= 64 else 16 if w.n <= 256 else 4 if w.n <= 512 else 1)
            t0 = time.perf_counter()
            oc, ot, om = oracle.restarts(c_host, obj, w.search_seed, 0, sample)
            dt = time.perf_counter() - t0
            ok = bool(np.array_equal(om, moves[:sample]) and np.array_equal(ot, bufs.restart_tours.cpu().numpy()[:sample]))
            d.update({"oracle_1core_move_evals_per_s": float(((om.astype(np.int64) + 1) * nbhd).sum() / dt),
                      "oracle_sample_restarts": sample, "oracle_sample_s": dt, "bit_exact_on_sample": ok})
        emit(d)

    def local_case(name, wid, classes, restarts=None):
        """Ring search over a wider move set (segment insertion with or without the 2-opt moves; the flip)."""
        w = WORKLOADS[wid]
        obj = cc.OBJECTIVES[w.objective]
        restarts = restarts or w.restarts
        c_host = make_matrix(wid)
        c = torch.from_numpy(c_host).cuda()
        bufs = cc.SearchBuffers(w.n, obj, restarts, c.device)
        ms = timed(lambda: cc.cc_local_search_ex(c, obj, classes, restarts, w.search_seed, buffers=bufs), args.reps)
        moves = bufs.restart_moves.cpu().numpy().astype(np.int64)
        n = w.n
        nbhd = 0
        if classes & cc.CC_MOVES_2OPT:
            nbhd += n * (n - 3) // 2 * (2 if obj & 2 else 1)
        if classes & cc.CC_MOVES_OROPT:
            nbhd += sum((n - L) * (n - L - 1) * (1 if L == 1 else 2) for L in (1, 2, 3))
        if classes & cc.CC_MOVES_FLIP:
            nbhd += 1
        evals = int(((moves + 1) * nbhd).sum())
        d = {"workload": name, "call": "cc_local_search_ex", "N": n, "objective": w.objective, "move_classes": classes,
             "restarts": restarts, "ms": ms, "move_evals": evals, "move_evals_per_s": evals / (ms * 1e-3),
             "applied_moves_mean": float(moves.mean()), "applied_moves_max": int(moves.max()),
             "best_cost": int(bufs.best_cost.item()), "mean_cost": float(bufs.restart_costs.double().mean().item())}
        if args.oracle:
            import oracle
            sample = min(restarts, 64 if n <= 64 else 4 if n <= 256 else 1)
            t0 = time.perf_counter()
            oc, ot, om = oracle.local_restarts(c_host, obj, classes, w.search_seed, 0, sample)
            dt = time.perf_counter() - t0
            ok = bool(np.array_equal(om, moves[:sample]) and np.array_equal(ot, bufs.restart_tours.cpu().numpy()[:sample]))
            d.update({"oracle_1core_move_evals_per_s": float(((om.astype(np.int64) + 1) * nbhd).sum() / dt),
                      "oracle_sample_restarts": sample, "bit_exact_on_sample": ok})
        emit(d)

    def swap_case(name, wid, restarts, n=None):
        w = WORKLOADS[wid]
        c_host = make_matrix(wid)
        if n is not None:         # the workload's hierarchy and value ranges at another size
            from gen import hierarchical_matrix
            import dataclasses
            c_host = hierarchical_matrix(n, w.group_sizes, w.level_ranges, w.sigma, True, w.matrix_seed + n)
            w = dataclasses.replace(w, n=n)
        c = torch.from_numpy(c_host).cuda()
        bufs = cc.SearchBuffers(w.n, 0, restarts, c.device)
        ms = timed(lambda: cc.cc_rd_swap_search_ex(c, restarts, w.search_seed, buffers=bufs), args.reps)
        moves = bufs.restart_moves.cpu().numpy().astype(np.int64)
        nbhd = w.n * (w.n - 1) // 2
        evals = int(((moves + 1) * nbhd).sum())
        d = {"workload": name, "call": "cc_rd_swap_search_ex", "N": w.n, "restarts": restarts, "ms": ms,
             "move_evals": evals, "move_evals_per_s": evals / (ms * 1e-3), "applied_moves_mean": float(moves.mean()),
             "applied_moves_max": int(moves.max()), "best_cost": int(bufs.best_cost.item())}
        if args.oracle:
            import oracle
            sample = min(restarts, 64 if w.n <= 64 else 2 if w.n <= 256 else 1)
            t0 = time.perf_counter()
            oc, ot, om = oracle.rd_swap_restarts(c_host, w.search_seed, 0, sample)
            dt = time.perf_counter() - t0
            ok = bool(np.array_equal(om, moves[:sample]) and np.array_equal(ot, bufs.restart_tours.cpu().numpy()[:sample]))
            d.update({"oracle_1core_move_evals_per_s": float(((om.astype(np.int64) + 1) * nbhd).sum() / dt),
                      "oracle_sample_restarts": sample, "bit_exact_on_sample": ok})
        emit(d)

    def sa_case(name, wid, chains, steps, t_start, t_end, rd=False):
        call = cc.cc_sa_rd_search_ex if rd else cc.cc_sa_search_ex
        w = WORKLOADS[wid]
        c_host = make_matrix(wid)
        c = torch.from_numpy(c_host).cuda()
        bufs = cc.SearchBuffers(w.n, 0, chains, c.device)
        ms = timed(lambda: call(c, chains, steps, t_start, t_end, w.search_seed, buffers=bufs), args.reps)
        acc = bufs.restart_moves.cpu().numpy().astype(np.int64)
        d = {"workload": name, "call": "cc_sa_rd_search_ex" if rd else "cc_sa_search_ex", "N": w.n, "chains": chains, "steps": steps,
             "t_start": t_start, "t_end": t_end, "ms": ms, "chain_steps_per_s": chains * steps / (ms * 1e-3),
             "accepted_fraction": float(acc.mean() / steps), "best_cost": int(bufs.best_cost.item()),
             "mean_chain_best": float(bufs.restart_costs.double().mean().item())}
        if args.oracle:
            import oracle
            sample = min(chains, 8)
            t0 = time.perf_counter()
            sample = min(sample, 2) if rd else sample
            run = oracle.sa_rd_chains if rd else oracle.sa_chains
            oc, ot, oa = run(c_host, steps, t_start, t_end, w.search_seed, 0, sample)
            dt = time.perf_counter() - t0
            ok = bool(np.array_equal(oc, bufs.restart_costs.cpu().numpy()[:sample]) and
                      np.array_equal(ot, bufs.restart_tours.cpu().numpy()[:sample]) and np.array_equal(oa, acc[:sample]))
            d.update({"oracle_1core_chain_steps_per_s": sample * steps / dt, "oracle_sample_chains": sample,
                      "bit_exact_on_sample": ok})
        emit(d)

    def probes_case(name, n, k):
        rng = np.random.default_rng(n + k)
        s_host = rng.integers(100, 30000, size=(n, n, k), dtype=np.int32)
        s = torch.from_numpy(s_host).cuda()
        out = torch.empty((n, n), dtype=torch.int32, device="cuda")
        ms = timed(lambda: cc.cc_cost_matrix_from_probes(s, 10, True, out=out), args.reps)
        nbytes = n * (n - 1) * k * 4
        d = {"workload": name, "call": "cc_cost_matrix_from_probes", "N": n, "K": k, "ms": ms,
             "samples_per_s": n * (n - 1) * k / (ms * 1e-3), "hbm_GBps": nbytes / (ms * 1e-3) / 1e9}
        if args.oracle:
            import oracle
            sub = min(n, 16)
            t0 = time.perf_counter()
            want = oracle.cost_matrix_from_probes(s_host[:sub, :sub], 10, True)
            dt = time.perf_counter() - t0
            got = cc.cc_cost_matrix_from_probes(s[:sub, :sub].contiguous(), 10, True).cpu().numpy()
            d.update({"oracle_1core_samples_per_s": sub * (sub - 1) * k / dt, "bit_exact_on_sample": bool(np.array_equal(got, want))})
        emit(d)

    def batch_case(name, wid, kind, objective, batch):
        w = WORKLOADS[wid]
        c_host = make_matrix(wid)
        c = torch.from_numpy(c_host).cuda()
        orders = cc.cc_init_tours(w.n, batch, w.search_seed)
        out = torch.empty(batch, dtype=torch.int64, device="cuda")
        bytes_per_order = 4 * w.n + 8
        if kind == "ring":
            fn = lambda: cc.cc_ring_cost_batch(c, orders, objective, out=out)  # noqa: E731
        elif kind == "ring_u8":
            orders8 = orders.to(torch.uint8)
            bytes_per_order = w.n + 8
            fn = lambda: cc.cc_ring_cost_batch_u8(c, orders8, objective, out=out)  # noqa: E731
        elif kind == "bcube":
            fn = lambda: cc.cc_bcube_cost_batch(c, 4, orders, out=out)  # noqa: E731
        elif kind == "dbt":
            fn = lambda: cc.cc_dbt_cost_batch(c, orders, out=out)  # noqa: E731
        else:
            fn = lambda: cc.cc_rd_cost_batch(c, orders, out=out)  # noqa: E731
        ms = timed(fn, args.reps)
        d = {"workload": name, "call": "cc_ring_cost_batch_u8" if kind == "ring_u8" else f"cc_{kind}_cost_batch", "N": w.n, "objective": objective, "batch": batch,
             "ms": ms, "perm_evals_per_s": batch / (ms * 1e-3), "hbm_GBps": batch * bytes_per_order / (ms * 1e-3) / 1e9}
        if args.oracle:
            import oracle
            sample = min(batch, 1 << 14 if w.n <= 64 else 256)
            sub = orders[:sample].cpu().numpy()
            t0 = time.perf_counter()
            want = {"ring": lambda: oracle.ring_cost_batch(c_host, sub, objective),
                    "ring_u8": lambda: oracle.ring_cost_batch(c_host, sub, objective),
                    "rd": lambda: oracle.rd_cost_batch(c_host, sub),
                    "bcube": lambda: oracle.bcube_cost_batch(c_host, 4, sub),
                    "dbt": lambda: oracle.dbt_cost_batch(c_host, sub)}[kind]()
            dt = time.perf_counter() - t0
            d.update({"oracle_1core_perm_evals_per_s": sample / dt,
                      "bit_exact_on_sample": bool(np.array_equal(want, out[:sample].cpu().numpy()))})
        emit(d)

    cases = [
        ("C1", lambda: batch_case("C1_n8_ring_sum_4096", 1, "ring", 0, 4096)),
        ("C2", lambda: search_case(2)),
        ("C3", lambda: search_case(3)),
        ("D64", lambda: search_case(3, objective="sum_directed", name="D64_n64_sum_directed_1024")),
        ("C4", lambda: search_case(4)),
        ("X256", lambda: search_case(4, objective="max", name="X256_n256_max_1024", restarts=1024)),
        ("X256big", lambda: search_case(4, objective="max", name="X256_n256_max_4096")),
        ("X256d", lambda: search_case(4, objective="max_directed", name="X256_n256_max_directed_1024", restarts=1024)),
        ("D256", lambda: search_case(4, objective="sum_directed", name="D256_n256_sum_directed_1024", restarts=1024)),
        ("X128", lambda: search_case(4, n=128, restarts=1024, name="X128_n128_max_1024", objective="max")),
        ("C5rd", lambda: batch_case("C5_n1024_rd_65536", 5, "rd", 0, 65536)),
        ("C5", lambda: search_case(5)),
        ("C512", lambda: search_case(5, n=512, restarts=768, name="C512_n512_sum_768_restarts")),
        ("L64", lambda: local_case("L64_n64_2opt+insertion_1024", 2, 3)),
        ("L64or", lambda: local_case("L64_n64_insertion_1024", 2, 2)),
        ("L64flip", lambda: local_case("L64_n64_max_directed_2opt+flip_1024", 3, 5)),
        ("L256", lambda: local_case("L256_n256_2opt+insertion_4096", 4, 3)),
        ("S64", lambda: swap_case("S64_n64_rd_swap_1024", 2, 1024)),
        ("S256", lambda: swap_case("S256_n256_rd_swap_256", 4, 256)),
        ("S512", lambda: swap_case("S512_n512_rd_swap_64", 5, 64, n=512)),
        ("S1024", lambda: swap_case("S1024_n1024_rd_swap_32", 5, 32)),
        ("A64", lambda: sa_case("A64_n64_sa_1024x100000", 2, 1024, 100000, 300, 0)),
        ("A64big", lambda: sa_case("A64_n64_sa_8192x100000", 2, 8192, 100000, 300, 0)),
        ("A256", lambda: sa_case("A256_n256_sa_1024x200000", 4, 1024, 200000, 300, 0)),
        ("A1024", lambda: sa_case("A1024_n1024_sa_1024x200000", 5, 1024, 200000, 300, 0)),
        ("P64", lambda: probes_case("P64_n64_probes_10000", 64, 10000)),
        ("P256", lambda: probes_case("P256_n256_probes_2000", 256, 2000)),
        ("B64", lambda: batch_case("B64_n64_bcube4_2^20", 2, "bcube", 0, 1 << 20)),
        ("B1024", lambda: batch_case("B1024_n1024_bcube4_65536", 5, "bcube", 0, 65536)),
        ("T64", lambda: batch_case("T64_n64_dbt_2^20", 2, "dbt", 0, 1 << 20)),
        ("T1024", lambda: batch_case("T1024_n1024_dbt_65536", 5, "dbt", 0, 65536)),
        ("R64", lambda: batch_case("R64_n64_rd_2^20", 2, "rd", 0, 1 << 20)),
        ("AR64", lambda: sa_case("AR64_n64_sa_rd_1024x20000", 2, 1024, 20000, 300, 0, rd=True)),
        ("AR1024", lambda: sa_case("AR1024_n1024_sa_rd_256x20000", 5, 256, 20000, 300, 0, rd=True)),
        ("R256", lambda: batch_case("R256_n256_rd_2^18", 4, "rd", 0, 1 << 18)),
        ("B256", lambda: batch_case("B256_n256_bcube4_2^18", 4, "bcube", 0, 1 << 18)),
        ("M256", lambda: batch_case("M256_n256_ring_sum_2^18", 4, "ring", 0, 1 << 18)),
        ("M1024", lambda: batch_case("M1024_n1024_ring_sum_65536", 5, "ring", 0, 65536)),
        ("M64sum", lambda: batch_case("M64_ring_sum_2^20", 2, "ring", 0, 1 << 20)),
        ("M64max", lambda: batch_case("M64_ring_max_2^20", 3, "ring", 1, 1 << 20)),
        ("M64u8", lambda: batch_case("M64_ring_sum_2^20_byte_orders", 2, "ring_u8", 0, 1 << 20)),
        ("M64u8big", lambda: batch_case("M64_ring_sum_2^24_byte_orders", 2, "ring_u8", 0, 1 << 24)),
    ]
    for key, fn in cases:
        if only is None or key in only:
            fn()


if __name__ == "__main__":
    main()
