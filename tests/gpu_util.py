"""Helpers for the GPU parity tests: run a case through the C ABI, compare with the CPU oracle."""
import sys

import numpy as np
import torch

import paper_2105_14088_amd as cc


def say(msg: str):
    """Name the case before the GPU step runs (flushed, so it survives a lost box)."""
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


SUMMARY = []


def report(msg: str):
    """A line for the end of the test run (how much of a full-size case the oracle replayed), printed now as well."""
    SUMMARY.append(msg)
    say(msg)


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def gpu_ring(c: np.ndarray, perms: np.ndarray, objective: int) -> np.ndarray:
    out = cc.cc_ring_cost_batch(dev(c), dev(perms), objective)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def gpu_rd(c: np.ndarray, perms: np.ndarray) -> np.ndarray:
    out = cc.cc_rd_cost_batch(dev(c), dev(perms))
    torch.cuda.synchronize()
    return out.cpu().numpy()


def gpu_search(c: np.ndarray, objective: int, restarts: int, seed: int, init=None):
    b = cc.cc_2opt_search_ex(dev(c), objective, restarts, seed, None if init is None else dev(init))
    torch.cuda.synchronize()
    return dict(best_perm=b.best_perm.cpu().numpy(), best_cost=int(b.best_cost.item()),
                best_restart=int(b.best_restart.item()), costs=b.restart_costs.cpu().numpy(),
                tours=b.restart_tours.cpu().numpy(), moves=b.restart_moves.cpu().numpy())


def assert_search_equal(got: dict, want: dict, rows=None):
    """Bit-exact comparison of per-restart results (optionally only the restart ids in `rows`,
    with `want` holding just those rows) and, when all rows are present, of the winner."""
    if rows is None:
        assert np.array_equal(got["costs"], want["costs"])
        assert np.array_equal(got["moves"], want["moves"])
        assert np.array_equal(got["tours"], want["tours"])
        assert got["best_cost"] == want["best_cost"] and got["best_restart"] == want["best_restart"]
        assert np.array_equal(got["best_perm"], want["best_perm"])
    else:
        rows = np.asarray(rows)
        assert np.array_equal(got["costs"][rows], want["costs"])
        assert np.array_equal(got["moves"][rows], want["moves"])
        assert np.array_equal(got["tours"][rows], want["tours"])
