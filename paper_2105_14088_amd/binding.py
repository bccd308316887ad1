"""ctypes binding of libcc.so (C ABI in include/cc.h).  Argument marshalling only: every step of the
computation runs in the library's HIP kernels.  torch supplies device memory and streams.

There is no CPU fallback: if the shared library is missing or a tensor is not on the GPU the call
raises."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcc.so")

CC_RING_SUM, CC_RING_MAX, CC_RING_SUM_DIRECTED, CC_RING_MAX_DIRECTED = 0, 1, 2, 3
OBJECTIVES = {"sum": 0, "max": 1, "sum_directed": 2, "max_directed": 3}
CC_MOVES_2OPT, CC_MOVES_OROPT, CC_MOVES_FLIP = 1, 2, 4
CC_MAX_N = 1024
CC_COST_MAX = (1 << 21) - 1

# every symbol include/cc.h declares
EXPORTS = ["cc_ring_cost_batch", "cc_ring_cost_batch_u8", "cc_ring_cost_batch_u16", "cc_rd_cost_batch",
           "cc_rd_cost_batch_ex", "cc_rd_batch_workspace_bytes", "cc_bcube_cost_batch", "cc_bcube_cost_batch_ex",
           "cc_bcube_cost_batch_weighted", "cc_dbt_cost_batch", "cc_2opt_search", "cc_2opt_search_ex", "cc_2opt_search_noalloc",
           "cc_2opt_workspace_bytes", "cc_local_search", "cc_local_search_ex", "cc_best_of_restarts", "cc_rd_swap_search", "cc_rd_swap_search_ex",
           "cc_rd_swap_workspace_bytes", "cc_sa_search", "cc_sa_search_ex", "cc_sa_workspace_bytes", "cc_sa_rd_search",
           "cc_sa_rd_search_ex", "cc_init_tours", "cc_cost_matrix_from_probes", "cc_validate_matrix",
           "cc_status_string", "cc_last_hip_error", "cc_version"]


class CCError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().cc_status_string(status).decode()
        if status == -4:
            msg += f" (hipError {lib().cc_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{status}]")


_lib = None


def lib() -> ctypes.CDLL:
    """Loads libcc.so built in-tree (python -m paper_2105_14088_amd.build); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not built: run `python __graft_entry__.py build` "
                                    "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        i32, i64, u64, p, sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_size_t
        L.cc_ring_cost_batch.restype = ctypes.c_int
        L.cc_ring_cost_batch.argtypes = [p, i32, i32, p, i64, p, p]
        L.cc_ring_cost_batch_u8.restype = ctypes.c_int
        L.cc_ring_cost_batch_u8.argtypes = [p, i32, i32, p, i64, p, p]
        L.cc_ring_cost_batch_u16.restype = ctypes.c_int
        L.cc_ring_cost_batch_u16.argtypes = [p, i32, i32, p, i64, p, p]
        L.cc_rd_cost_batch.restype = ctypes.c_int
        L.cc_rd_cost_batch.argtypes = [p, i32, p, i64, p, p]
        L.cc_rd_cost_batch_ex.restype = ctypes.c_int
        L.cc_rd_cost_batch_ex.argtypes = [p, i32, p, i64, p, p, sz, p]
        L.cc_rd_batch_workspace_bytes.restype = sz
        L.cc_rd_batch_workspace_bytes.argtypes = [i32]
        L.cc_bcube_cost_batch_ex.restype = ctypes.c_int
        L.cc_bcube_cost_batch_ex.argtypes = [p, i32, i32, p, p, i64, p, p, sz, p]
        L.cc_bcube_cost_batch.restype = ctypes.c_int
        L.cc_bcube_cost_batch.argtypes = [p, i32, i32, p, i64, p, p]
        L.cc_bcube_cost_batch_weighted.restype = ctypes.c_int
        L.cc_bcube_cost_batch_weighted.argtypes = [p, i32, i32, p, p, i64, p, p]
        L.cc_dbt_cost_batch.restype = ctypes.c_int
        L.cc_dbt_cost_batch.argtypes = [p, i32, p, i64, p, p]
        L.cc_2opt_search.restype = ctypes.c_int
        L.cc_2opt_search.argtypes = [p, i32, i32, i32, u64, p, p, p]
        L.cc_2opt_search_noalloc.restype = ctypes.c_int
        L.cc_2opt_search_noalloc.argtypes = [p, i32, i32, i32, u64, p, p, p]
        L.cc_2opt_search_ex.restype = ctypes.c_int
        L.cc_2opt_search_ex.argtypes = [p, i32, i32, i32, u64, p, p, p, p, p, p, p, p, sz, p]
        L.cc_local_search.restype = ctypes.c_int
        L.cc_local_search.argtypes = [p, i32, i32, i32, i32, u64, p, p, p]
        L.cc_local_search_ex.restype = ctypes.c_int
        L.cc_local_search_ex.argtypes = [p, i32, i32, i32, i32, u64, p, p, p, p, p, p, p, p, sz, p]
        L.cc_best_of_restarts.restype = ctypes.c_int
        L.cc_best_of_restarts.argtypes = [p, p, i32, i32, p, p, p, p]
        L.cc_2opt_workspace_bytes.restype = sz
        L.cc_2opt_workspace_bytes.argtypes = [i32, i32, i32]
        L.cc_rd_swap_search.restype = ctypes.c_int
        L.cc_rd_swap_search.argtypes = [p, i32, i32, u64, p, p, p]
        L.cc_rd_swap_search_ex.restype = ctypes.c_int
        L.cc_rd_swap_search_ex.argtypes = [p, i32, i32, u64, p, p, p, p, p, p, p, p, sz, p]
        L.cc_rd_swap_workspace_bytes.restype = sz
        L.cc_rd_swap_workspace_bytes.argtypes = [i32, i32]
        L.cc_sa_search.restype = ctypes.c_int
        L.cc_sa_search.argtypes = [p, i32, i32, i64, i32, i32, u64, p, p, p]
        L.cc_sa_search_ex.restype = ctypes.c_int
        L.cc_sa_search_ex.argtypes = [p, i32, i32, i64, i32, i32, u64, p, p, p, p, p, p, p, p, sz, p]
        L.cc_sa_rd_search.restype = ctypes.c_int
        L.cc_sa_rd_search.argtypes = [p, i32, i32, i64, i32, i32, u64, p, p, p]
        L.cc_sa_rd_search_ex.restype = ctypes.c_int
        L.cc_sa_rd_search_ex.argtypes = [p, i32, i32, i64, i32, i32, u64, p, p, p, p, p, p, p, p, sz, p]
        L.cc_sa_workspace_bytes.restype = sz
        L.cc_sa_workspace_bytes.argtypes = [i32, i32]
        L.cc_init_tours.restype = ctypes.c_int
        L.cc_init_tours.argtypes = [i32, i64, i64, u64, p, p]
        L.cc_cost_matrix_from_probes.restype = ctypes.c_int
        L.cc_cost_matrix_from_probes.argtypes = [p, i32, i32, i32, i32, p, p]
        L.cc_validate_matrix.restype = ctypes.c_int
        L.cc_validate_matrix.argtypes = [p, i32, i32, p]
        L.cc_status_string.restype = ctypes.c_char_p
        L.cc_status_string.argtypes = [ctypes.c_int]
        L.cc_last_hip_error.restype = ctypes.c_int
        L.cc_last_hip_error.argtypes = []
        L.cc_version.restype = ctypes.c_int
        L.cc_version.argtypes = []
        _lib = L
    return _lib


def _dev(t: Optional[torch.Tensor], dtype, name: str):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor")
    if t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous {dtype} tensor")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _new(shape, dtype, device, stream=None) -> torch.Tensor:
    """A tensor this binding allocates for a call.  The call only enqueues kernels, so with an explicit stream that
    is not torch's current one the caching allocator must learn that the block is in use on that stream: otherwise
    a tensor dropped by the caller (or a workspace dropped here on return) could be handed to other work while the
    kernels still read or write it."""
    t = torch.empty(shape, dtype=dtype, device=device)
    if stream is not None:
        t.record_stream(stream)
    return t


def _matrix(c: torch.Tensor) -> int:
    if c.dim() != 2 or c.shape[0] != c.shape[1]:
        raise ValueError("cost_matrix must be square")
    return int(c.shape[0])


def _check(rc: int, where: str):
    if rc != 0:
        raise CCError(rc, where)


def cc_ring_cost_batch(cost_matrix: torch.Tensor, perms: torch.Tensor, objective: int = CC_RING_SUM,
                       out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    n = _matrix(cost_matrix)
    if perms.dim() != 2 or perms.shape[1] != n:
        raise ValueError("perms must be [B, N]")
    b = int(perms.shape[0])
    if out is None:
        out = _new(b, torch.int64, cost_matrix.device, stream)
    _check(lib().cc_ring_cost_batch(_dev(cost_matrix, torch.int32, "cost_matrix"), n, objective,
                                    _dev(perms, torch.int32, "perms"), b, _dev(out, torch.int64, "out"),
                                    _stream(stream)), "cc_ring_cost_batch")
    return out


def cc_ring_cost_batch_u8(cost_matrix: torch.Tensor, perms: torch.Tensor, objective: int,
                          out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    n = _matrix(cost_matrix)
    if perms.dim() != 2 or perms.shape[1] != n:
        raise ValueError("perms must be [B, N]")
    b = int(perms.shape[0])
    if out is None:
        out = _new(b, torch.int64, cost_matrix.device, stream)
    _check(lib().cc_ring_cost_batch_u8(_dev(cost_matrix, torch.int32, "cost_matrix"), n, objective,
                                       _dev(perms, torch.uint8, "perms"), b, _dev(out, torch.int64, "out"),
                                       _stream(stream)), "cc_ring_cost_batch_u8")
    return out


def cc_ring_cost_batch_u16(cost_matrix: torch.Tensor, perms: torch.Tensor, objective: int,
                           out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """perms: int16 or uint16 [B, N] (ranks are below 1024, so the two read the same)."""
    n = _matrix(cost_matrix)
    if perms.dim() != 2 or perms.shape[1] != n:
        raise ValueError("perms must be [B, N]")
    if perms.dtype not in (torch.int16, torch.uint16):
        raise ValueError("perms must be a 16-bit integer tensor")
    b = int(perms.shape[0])
    if out is None:
        out = _new(b, torch.int64, cost_matrix.device, stream)
    _check(lib().cc_ring_cost_batch_u16(_dev(cost_matrix, torch.int32, "cost_matrix"), n, objective,
                                        _dev(perms, perms.dtype, "perms"), b, _dev(out, torch.int64, "out"),
                                        _stream(stream)), "cc_ring_cost_batch_u16")
    return out


def cc_rd_batch_workspace_bytes(n: int) -> int:
    return int(lib().cc_rd_batch_workspace_bytes(n))


def cc_rd_cost_batch(cost_matrix: torch.Tensor, perms: torch.Tensor, out: Optional[torch.Tensor] = None,
                     stream=None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Calls cc_rd_cost_batch_ex when N >= 128 (with `workspace`, a uint8 device tensor of at least
    cc_rd_batch_workspace_bytes(N) bytes, or one allocated here), cc_rd_cost_batch otherwise."""
    n = _matrix(cost_matrix)
    if perms.dim() != 2 or perms.shape[1] != n:
        raise ValueError("perms must be [B, N]")
    b = int(perms.shape[0])
    if out is None:
        out = _new(b, torch.int64, cost_matrix.device, stream)
    if n < 128 and workspace is None:
        _check(lib().cc_rd_cost_batch(_dev(cost_matrix, torch.int32, "cost_matrix"), n,
                                      _dev(perms, torch.int32, "perms"), b, _dev(out, torch.int64, "out"),
                                      _stream(stream)), "cc_rd_cost_batch")
        return out
    if workspace is None:
        workspace = _new(cc_rd_batch_workspace_bytes(n), torch.uint8, cost_matrix.device, stream)
    _check(lib().cc_rd_cost_batch_ex(_dev(cost_matrix, torch.int32, "cost_matrix"), n, _dev(perms, torch.int32, "perms"),
                                     b, _dev(out, torch.int64, "out"), _dev(workspace, torch.uint8, "workspace"),
                                     workspace.numel(), _stream(stream)), "cc_rd_cost_batch_ex")
    return out


def _bcube(cost_matrix, base, round_weights, perms, out, stream, workspace, where):
    n = _matrix(cost_matrix)
    if perms.dim() != 2 or perms.shape[1] != n:
        raise ValueError("perms must be [B, N]")
    b = int(perms.shape[0])
    if out is None:
        out = _new(b, torch.int64, cost_matrix.device, stream)
    folded_form = (base == 2 and n >= 128) or (base == 4 and n in (256, 1024))      # the sizes the workspace serves
    if workspace is None and folded_form:
        workspace = _new(cc_rd_batch_workspace_bytes(n), torch.uint8, cost_matrix.device, stream)
    c, pm, o = _dev(cost_matrix, torch.int32, "cost_matrix"), _dev(perms, torch.int32, "perms"), _dev(out, torch.int64, "out")
    w = _dev(round_weights, torch.int32, "round_weights")
    if workspace is not None:
        _check(lib().cc_bcube_cost_batch_ex(c, n, base, w, pm, b, o, _dev(workspace, torch.uint8, "workspace"),
                                            workspace.numel(), _stream(stream)), "cc_bcube_cost_batch_ex")
    elif round_weights is None:
        _check(lib().cc_bcube_cost_batch(c, n, base, pm, b, o, _stream(stream)), where)
    else:
        _check(lib().cc_bcube_cost_batch_weighted(c, n, base, w, pm, b, o, _stream(stream)), where)
    return out


def cc_bcube_cost_batch(cost_matrix: torch.Tensor, base: int, perms: torch.Tensor, out: Optional[torch.Tensor] = None,
                        stream=None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Calls cc_bcube_cost_batch_ex where its workspace pays (base 2 from N = 128, base 4 at N = 256 and 1024; with
    `workspace`, a uint8 device tensor of cc_rd_batch_workspace_bytes(N) bytes, or one allocated here) and
    cc_bcube_cost_batch otherwise."""
    return _bcube(cost_matrix, base, None, perms, out, stream, workspace, "cc_bcube_cost_batch")


def cc_bcube_cost_batch_weighted(cost_matrix: torch.Tensor, base: int, round_weights: torch.Tensor, perms: torch.Tensor,
                                 out: Optional[torch.Tensor] = None, stream=None,
                                 workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    n = _matrix(cost_matrix)
    rounds, power = 0, 1
    while power < n:
        power *= base
        rounds += 1
    if round_weights.dim() != 1 or round_weights.shape[0] != rounds:
        raise ValueError("round_weights must be [log_base N]")
    return _bcube(cost_matrix, base, round_weights, perms, out, stream, workspace, "cc_bcube_cost_batch_weighted")


def cc_dbt_cost_batch(cost_matrix: torch.Tensor, perms: torch.Tensor, out: Optional[torch.Tensor] = None,
                      stream=None) -> torch.Tensor:
    n = _matrix(cost_matrix)
    if perms.dim() != 2 or perms.shape[1] != n:
        raise ValueError("perms must be [B, N]")
    b = int(perms.shape[0])
    if out is None:
        out = _new(b, torch.int64, cost_matrix.device, stream)
    _check(lib().cc_dbt_cost_batch(_dev(cost_matrix, torch.int32, "cost_matrix"), n, _dev(perms, torch.int32, "perms"),
                                   b, _dev(out, torch.int64, "out"), _stream(stream)), "cc_dbt_cost_batch")
    return out


def cc_2opt_workspace_bytes(n: int, objective: int, restarts: int) -> int:
    return int(lib().cc_2opt_workspace_bytes(n, objective, restarts))


def cc_2opt_search(cost_matrix: torch.Tensor, objective: int, restarts: int, seed: int, stream=None):
    """Returns (best_perm int32[N], best_cost int64[1]) device tensors (valid after stream sync)."""
    n = _matrix(cost_matrix)
    best_perm = _new(n, torch.int32, cost_matrix.device, stream)
    best_cost = _new(1, torch.int64, cost_matrix.device, stream)
    _check(lib().cc_2opt_search(_dev(cost_matrix, torch.int32, "cost_matrix"), n, objective, restarts,
                                seed & (2**64 - 1), _dev(best_perm, torch.int32, "best_perm"),
                                _dev(best_cost, torch.int64, "best_cost"), _stream(stream)), "cc_2opt_search")
    return best_perm, best_cost


def cc_2opt_search_noalloc(cost_matrix: torch.Tensor, objective: int, restarts: int, seed: int,
                           best_perm: torch.Tensor, best_cost: torch.Tensor, stream=None) -> None:
    """cc_2opt_search with the library's static device scratch array; writes into the caller's best_perm (int32 [N])
    and best_cost (int64 [1]).  Nothing is allocated, here or in the library."""
    n = _matrix(cost_matrix)
    if best_perm.numel() != n or best_cost.numel() != 1:
        raise ValueError("best_perm must be [N], best_cost [1]")
    _check(lib().cc_2opt_search_noalloc(_dev(cost_matrix, torch.int32, "cost_matrix"), n, objective, restarts,
                                        seed & (2**64 - 1), _dev(best_perm, torch.int32, "best_perm"),
                                        _dev(best_cost, torch.int64, "best_cost"), _stream(stream)),
           "cc_2opt_search_noalloc")


class SearchBuffers:
    """Device buffers for cc_2opt_search_ex, allocated once and reusable across calls."""

    def __init__(self, n: int, objective: int, restarts: int, device, per_restart: bool = True, stream=None):
        self.n, self.objective, self.restarts = n, objective, restarts
        self.best_perm = _new(n, torch.int32, device, stream)
        self.best_cost = _new(1, torch.int64, device, stream)
        self.best_restart = _new(1, torch.int32, device, stream)
        self.restart_costs = _new(restarts, torch.int64, device, stream) if per_restart else None
        self.restart_tours = _new((restarts, n), torch.int32, device, stream) if per_restart else None
        self.restart_moves = _new(restarts, torch.int32, device, stream) if per_restart else None
        nbytes = cc_2opt_workspace_bytes(n, objective, restarts)
        if nbytes == 0:
            raise ValueError("invalid (N, objective, restarts)")
        self.workspace = _new(nbytes + 256, torch.uint8, device, stream)
        off = (-self.workspace.data_ptr()) % 256
        self.ws_ptr = self.workspace.data_ptr() + off
        self.ws_bytes = nbytes


def cc_2opt_search_ex(cost_matrix: torch.Tensor, objective: int, restarts: int, seed: int,
                      init_tours: Optional[torch.Tensor] = None, buffers: Optional[SearchBuffers] = None,
                      stream=None, pick_best: bool = True) -> SearchBuffers:
    """pick_best=False stops after the per-restart results (cc_best_of_restarts picks the winner later)."""
    n = _matrix(cost_matrix)
    if buffers is None:
        buffers = SearchBuffers(n, objective, restarts, cost_matrix.device, stream=stream)
    if (buffers.n, buffers.restarts) != (n, restarts):
        raise ValueError("buffers were sized for a different search")
    if init_tours is not None and tuple(init_tours.shape) != (restarts, n):
        raise ValueError("init_tours must be [restarts, N]")
    b = buffers
    _check(lib().cc_2opt_search_ex(_dev(cost_matrix, torch.int32, "cost_matrix"), n, objective, restarts,
                                   seed & (2**64 - 1), _dev(init_tours, torch.int32, "init_tours"),
                                   _dev(b.best_perm, torch.int32, "best_perm") if pick_best else None,
                                   _dev(b.best_cost, torch.int64, "best_cost") if pick_best else None,
                                   _dev(b.best_restart, torch.int32, "best_restart") if pick_best else None,
                                   _dev(b.restart_costs, torch.int64, "restart_costs"),
                                   _dev(b.restart_tours, torch.int32, "restart_tours"),
                                   _dev(b.restart_moves, torch.int32, "restart_moves"),
                                   ctypes.c_void_p(b.ws_ptr), b.ws_bytes, _stream(stream)), "cc_2opt_search_ex")
    return b


def cc_local_search(cost_matrix: torch.Tensor, objective: int, move_classes: int, restarts: int, seed: int,
                    stream=None):
    """Returns (best_perm int32[N], best_cost int64[1]) device tensors (valid after stream sync)."""
    n = _matrix(cost_matrix)
    best_perm = _new(n, torch.int32, cost_matrix.device, stream)
    best_cost = _new(1, torch.int64, cost_matrix.device, stream)
    _check(lib().cc_local_search(_dev(cost_matrix, torch.int32, "cost_matrix"), n, objective, move_classes, restarts,
                                 seed & (2**64 - 1), _dev(best_perm, torch.int32, "best_perm"),
                                 _dev(best_cost, torch.int64, "best_cost"), _stream(stream)), "cc_local_search")
    return best_perm, best_cost


def cc_local_search_ex(cost_matrix: torch.Tensor, objective: int, move_classes: int, restarts: int, seed: int,
                       init_tours: Optional[torch.Tensor] = None, buffers: Optional[SearchBuffers] = None,
                       stream=None, pick_best: bool = True) -> SearchBuffers:
    """cc_2opt_search_ex over the move classes `move_classes` (CC_MOVES_*)."""
    n = _matrix(cost_matrix)
    if buffers is None:
        buffers = SearchBuffers(n, objective, restarts, cost_matrix.device, stream=stream)
    if (buffers.n, buffers.restarts) != (n, restarts):
        raise ValueError("buffers were sized for a different search")
    if init_tours is not None and tuple(init_tours.shape) != (restarts, n):
        raise ValueError("init_tours must be [restarts, N]")
    b = buffers
    _check(lib().cc_local_search_ex(_dev(cost_matrix, torch.int32, "cost_matrix"), n, objective, move_classes,
                                    restarts, seed & (2**64 - 1), _dev(init_tours, torch.int32, "init_tours"),
                                    _dev(b.best_perm, torch.int32, "best_perm") if pick_best else None,
                                    _dev(b.best_cost, torch.int64, "best_cost") if pick_best else None,
                                    _dev(b.best_restart, torch.int32, "best_restart") if pick_best else None,
                                    _dev(b.restart_costs, torch.int64, "restart_costs"),
                                    _dev(b.restart_tours, torch.int32, "restart_tours"),
                                    _dev(b.restart_moves, torch.int32, "restart_moves"),
                                    ctypes.c_void_p(b.ws_ptr), b.ws_bytes, _stream(stream)), "cc_local_search_ex")
    return b


def cc_best_of_restarts(buffers: SearchBuffers, stream=None) -> SearchBuffers:
    """Fills best_perm / best_cost / best_restart of `buffers` from its per-restart costs and orders."""
    b = buffers
    _check(lib().cc_best_of_restarts(_dev(b.restart_costs, torch.int64, "restart_costs"),
                                     _dev(b.restart_tours, torch.int32, "restart_tours"), b.n, b.restarts,
                                     _dev(b.best_perm, torch.int32, "best_perm"),
                                     _dev(b.best_cost, torch.int64, "best_cost"),
                                     _dev(b.best_restart, torch.int32, "best_restart"), _stream(stream)),
           "cc_best_of_restarts")
    return b


def cc_rd_swap_search(cost_matrix: torch.Tensor, restarts: int, seed: int, stream=None):
    """Returns (best_perm int32[N], best_cost int64[1]) device tensors (valid after stream sync)."""
    n = _matrix(cost_matrix)
    best_perm = _new(n, torch.int32, cost_matrix.device, stream)
    best_cost = _new(1, torch.int64, cost_matrix.device, stream)
    _check(lib().cc_rd_swap_search(_dev(cost_matrix, torch.int32, "cost_matrix"), n, restarts, seed & (2**64 - 1),
                                   _dev(best_perm, torch.int32, "best_perm"),
                                   _dev(best_cost, torch.int64, "best_cost"), _stream(stream)), "cc_rd_swap_search")
    return best_perm, best_cost


def cc_rd_swap_search_ex(cost_matrix: torch.Tensor, restarts: int, seed: int,
                         init_tours: Optional[torch.Tensor] = None, buffers: Optional[SearchBuffers] = None,
                         stream=None) -> SearchBuffers:
    n = _matrix(cost_matrix)
    if buffers is None:
        buffers = SearchBuffers(n, 0, restarts, cost_matrix.device, stream=stream)
    if (buffers.n, buffers.restarts) != (n, restarts):
        raise ValueError("buffers were sized for a different search")
    if init_tours is not None and tuple(init_tours.shape) != (restarts, n):
        raise ValueError("init_tours must be [restarts, N]")
    b = buffers
    _check(lib().cc_rd_swap_search_ex(_dev(cost_matrix, torch.int32, "cost_matrix"), n, restarts, seed & (2**64 - 1),
                                      _dev(init_tours, torch.int32, "init_tours"),
                                      _dev(b.best_perm, torch.int32, "best_perm"),
                                      _dev(b.best_cost, torch.int64, "best_cost"),
                                      _dev(b.best_restart, torch.int32, "best_restart"),
                                      _dev(b.restart_costs, torch.int64, "restart_costs"),
                                      _dev(b.restart_tours, torch.int32, "restart_tours"),
                                      _dev(b.restart_moves, torch.int32, "restart_moves"),
                                      ctypes.c_void_p(b.ws_ptr), b.ws_bytes, _stream(stream)), "cc_rd_swap_search_ex")
    return b


def _sa_search(fn_name: str, cost_matrix: torch.Tensor, chains: int, steps: int, t_start: int, t_end: int, seed: int,
               stream=None):
    """Returns (best_perm int32[N], best_cost int64[1]) device tensors (valid after stream sync)."""
    n = _matrix(cost_matrix)
    best_perm = _new(n, torch.int32, cost_matrix.device, stream)
    best_cost = _new(1, torch.int64, cost_matrix.device, stream)
    _check(getattr(lib(), fn_name)(_dev(cost_matrix, torch.int32, "cost_matrix"), n, chains, steps, t_start, t_end,
                                   seed & (2**64 - 1), _dev(best_perm, torch.int32, "best_perm"),
                                   _dev(best_cost, torch.int64, "best_cost"), _stream(stream)), fn_name)
    return best_perm, best_cost


def _sa_search_ex(fn_name: str, cost_matrix: torch.Tensor, chains: int, steps: int, t_start: int, t_end: int,
                  seed: int, init_tours: Optional[torch.Tensor] = None, buffers: Optional[SearchBuffers] = None,
                  stream=None) -> SearchBuffers:
    """Per-chain results land in the buffers' restart_costs / restart_tours (best cost and order of every chain)
    and restart_moves (accepted proposals); best_restart is the winning chain."""
    n = _matrix(cost_matrix)
    if buffers is None:
        buffers = SearchBuffers(n, 0, chains, cost_matrix.device, stream=stream)
    if (buffers.n, buffers.restarts) != (n, chains):
        raise ValueError("buffers were sized for a different search")
    if init_tours is not None and tuple(init_tours.shape) != (chains, n):
        raise ValueError("init_tours must be [chains, N]")
    b = buffers
    _check(getattr(lib(), fn_name)(_dev(cost_matrix, torch.int32, "cost_matrix"), n, chains, steps, t_start, t_end,
                                   seed & (2**64 - 1), _dev(init_tours, torch.int32, "init_tours"),
                                   _dev(b.best_perm, torch.int32, "best_perm"),
                                   _dev(b.best_cost, torch.int64, "best_cost"),
                                   _dev(b.best_restart, torch.int32, "best_restart"),
                                   _dev(b.restart_costs, torch.int64, "restart_costs"),
                                   _dev(b.restart_tours, torch.int32, "restart_tours"),
                                   _dev(b.restart_moves, torch.int32, "restart_moves"),
                                   ctypes.c_void_p(b.ws_ptr), b.ws_bytes, _stream(stream)), fn_name)
    return b


def cc_sa_search(cost_matrix, chains, steps, t_start, t_end, seed, stream=None):
    """Ring sum, sub-array reversals.  Returns (best_perm int32[N], best_cost int64[1]) device tensors."""
    return _sa_search("cc_sa_search", cost_matrix, chains, steps, t_start, t_end, seed, stream)


def cc_sa_search_ex(cost_matrix, chains, steps, t_start, t_end, seed, init_tours=None, buffers=None, stream=None):
    return _sa_search_ex("cc_sa_search_ex", cost_matrix, chains, steps, t_start, t_end, seed, init_tours, buffers, stream)


def cc_sa_rd_search(cost_matrix, chains, steps, t_start, t_end, seed, stream=None):
    """Halving-doubling model, pair exchanges.  Returns (best_perm int32[N], best_cost int64[1]) device tensors."""
    return _sa_search("cc_sa_rd_search", cost_matrix, chains, steps, t_start, t_end, seed, stream)


def cc_sa_rd_search_ex(cost_matrix, chains, steps, t_start, t_end, seed, init_tours=None, buffers=None, stream=None):
    return _sa_search_ex("cc_sa_rd_search_ex", cost_matrix, chains, steps, t_start, t_end, seed, init_tours, buffers,
                         stream)


def cc_init_tours(n: int, count: int, seed: int, first: int = 0, device="cuda", out: Optional[torch.Tensor] = None,
                  stream=None) -> torch.Tensor:
    if out is None:
        out = _new((count, n), torch.int32, device, stream)
    _check(lib().cc_init_tours(n, first, count, seed & (2**64 - 1), _dev(out, torch.int32, "tours"), _stream(stream)),
           "cc_init_tours")
    return out


def cc_cost_matrix_from_probes(samples: torch.Tensor, percentile: int = 10, symmetrize: bool = True,
                               out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    if samples.dim() != 3 or samples.shape[0] != samples.shape[1]:
        raise ValueError("samples must be [N, N, K]")
    n, k = int(samples.shape[0]), int(samples.shape[2])
    if out is None:
        out = _new((n, n), torch.int32, samples.device, stream)
    _check(lib().cc_cost_matrix_from_probes(_dev(samples, torch.int32, "samples"), n, k, percentile,
                                            1 if symmetrize else 0, _dev(out, torch.int32, "cost_matrix"),
                                            _stream(stream)), "cc_cost_matrix_from_probes")
    return out


def cc_validate_matrix(cost_matrix: torch.Tensor, require_symmetric: bool = True, stream=None) -> int:
    """Returns the status code (0 ok, -5 not symmetric, -6 out of range); raises on other errors."""
    n = _matrix(cost_matrix)
    rc = lib().cc_validate_matrix(_dev(cost_matrix, torch.int32, "cost_matrix"), n, 1 if require_symmetric else 0,
                                  _stream(stream))
    if rc not in (0, -5, -6):
        raise CCError(rc, "cc_validate_matrix")
    return rc


def cc_status_string(status: int) -> str:
    return lib().cc_status_string(status).decode()


def cc_version() -> int:
    return int(lib().cc_version())
