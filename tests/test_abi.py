"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares, and
rejects bad arguments before touching the GPU.  No compute call is made here."""
import ctypes
import os
import re

import pytest

import paper_2105_14088_amd as cc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
pytestmark = pytest.mark.usefixtures("built_library")


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "cc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cc_[a-z0-9_]+)\s*\(", text)))


def test_header_and_binding_agree():
    assert _declared_symbols() == sorted(cc.EXPORTS)


def test_library_exports_every_declared_symbol():
    L = cc.lib()
    for name in _declared_symbols():
        assert hasattr(L, name), name


def test_version_and_status_strings():
    assert cc.cc_version() >= 100
    seen = set()
    for s in range(0, -8, -1):
        txt = cc.cc_status_string(s)
        assert txt and txt != "unknown status" and txt not in seen
        seen.add(txt)
    assert cc.cc_status_string(-99) == "unknown status"


def test_workspace_bytes_host_only():
    assert cc.cc_2opt_workspace_bytes(64, 0, 1024) >= 1024 * 64 * 4 + 1024 * 12
    assert cc.cc_2opt_workspace_bytes(64, 0, 1024) % 256 == 0
    assert cc.cc_2opt_workspace_bytes(1, 0, 1) == 0
    assert cc.cc_2opt_workspace_bytes(1025, 0, 1) == 0
    assert cc.cc_2opt_workspace_bytes(64, 4, 1) == 0
    assert cc.cc_2opt_workspace_bytes(64, 0, 0) == 0


def test_argument_errors_are_returned_before_any_launch():
    L = cc.lib()
    fake = ctypes.c_void_p(0x1000)        # never dereferenced: every call below fails its host checks
    null = ctypes.c_void_p(0)
    INVALID, UNSUPPORTED, WORKSPACE = -1, -2, -3
    assert L.cc_ring_cost_batch(null, 64, 0, fake, 1, fake, null) == INVALID
    assert L.cc_ring_cost_batch(fake, 1, 0, fake, 1, fake, null) == UNSUPPORTED
    assert L.cc_ring_cost_batch(fake, 1025, 0, fake, 1, fake, null) == UNSUPPORTED
    assert L.cc_ring_cost_batch(fake, 64, 7, fake, 1, fake, null) == INVALID
    assert L.cc_ring_cost_batch(fake, 64, 0, fake, -1, fake, null) == INVALID
    assert L.cc_ring_cost_batch(fake, 64, 0, null, 1, fake, null) == INVALID
    assert L.cc_ring_cost_batch(fake, 64, 0, fake, 1, null, null) == INVALID
    assert L.cc_ring_cost_batch(fake, 64, 0, null, 0, null, null) == 0          # B = 0 is a no-op
    assert L.cc_ring_cost_batch_u8(fake, 257, 0, fake, 1, fake, null) == UNSUPPORTED   # ranks do not fit a byte
    assert L.cc_ring_cost_batch_u8(fake, 64, 0, null, 1, fake, null) == INVALID
    assert L.cc_ring_cost_batch_u8(fake, 64, 0, null, 0, null, null) == 0
    assert L.cc_ring_cost_batch_u16(fake, 1025, 0, fake, 1, fake, null) == UNSUPPORTED
    assert L.cc_ring_cost_batch_u16(fake, 512, 0, null, 1, fake, null) == INVALID
    assert L.cc_ring_cost_batch_u16(fake, 512, 0, ctypes.c_void_p(0x1001), 1, fake, null) == INVALID   # misaligned
    assert L.cc_ring_cost_batch_u16(fake, 512, 4, fake, 1, fake, null) == INVALID
    assert L.cc_ring_cost_batch_u16(fake, 512, 0, null, 0, null, null) == 0
    assert L.cc_rd_cost_batch(fake, 48, fake, 1, fake, null) == UNSUPPORTED      # not a power of two
    assert L.cc_rd_cost_batch(fake, 64, fake, -5, fake, null) == INVALID
    assert L.cc_rd_cost_batch(fake, 64, null, 0, null, null) == 0
    ws256 = ctypes.c_void_p(0x10000)
    need = L.cc_rd_batch_workspace_bytes(1024)
    assert need >= 2 * 1024 * 1024 and need % 256 == 0
    assert L.cc_rd_batch_workspace_bytes(1) == 0 and L.cc_rd_batch_workspace_bytes(2048) == 0
    assert L.cc_rd_batch_workspace_bytes(27) == 256 + 1536          # 2 * 27 * 27 = 1458 bytes, rounded up
    assert L.cc_rd_cost_batch_ex(fake, 48, fake, 1, fake, ws256, need, null) == UNSUPPORTED
    assert L.cc_rd_cost_batch_ex(fake, 1024, fake, 1, fake, null, need, null) == WORKSPACE
    assert L.cc_rd_cost_batch_ex(fake, 1024, fake, 1, fake, ws256, need - 1, null) == WORKSPACE
    assert L.cc_rd_cost_batch_ex(fake, 1024, fake, 1, fake, ctypes.c_void_p(0x10010), need, null) == WORKSPACE   # misaligned
    assert L.cc_rd_cost_batch_ex(fake, 1024, fake, -1, fake, ws256, need, null) == INVALID
    assert L.cc_rd_cost_batch_ex(fake, 1024, null, 1, fake, ws256, need, null) == INVALID
    assert L.cc_rd_cost_batch_ex(fake, 1024, null, 0, null, ws256, need, null) == 0
    assert L.cc_bcube_cost_batch(fake, 32, 4, fake, 1, fake, null) == UNSUPPORTED   # not a power of the base
    assert L.cc_bcube_cost_batch_ex(fake, 32, 4, null, fake, 1, fake, ws256, need, null) == UNSUPPORTED
    assert L.cc_bcube_cost_batch_ex(fake, 1024, 4, null, fake, 1, fake, ws256, need - 1, null) == WORKSPACE
    assert L.cc_bcube_cost_batch_ex(fake, 1024, 4, null, fake, 1, fake, null, need, null) == WORKSPACE
    assert L.cc_bcube_cost_batch_ex(fake, 1024, 4, ctypes.c_void_p(0x1002), fake, 1, fake, ws256, need, null) == INVALID
    assert L.cc_bcube_cost_batch_ex(fake, 1024, 1, null, fake, 1, fake, ws256, need, null) == INVALID
    assert L.cc_bcube_cost_batch_ex(fake, 1024, 4, null, null, 0, null, ws256, need, null) == 0
    assert L.cc_bcube_cost_batch(fake, 64, 1, fake, 1, fake, null) == INVALID
    assert L.cc_bcube_cost_batch(fake, 64, 4, fake, -1, fake, null) == INVALID
    assert L.cc_bcube_cost_batch(fake, 64, 4, null, 1, fake, null) == INVALID
    assert L.cc_bcube_cost_batch(fake, 64, 4, null, 0, null, null) == 0
    assert L.cc_bcube_cost_batch_weighted(fake, 64, 4, null, fake, 1, fake, null) == INVALID   # weights required
    assert L.cc_bcube_cost_batch_weighted(fake, 48, 2, fake, fake, 1, fake, null) == UNSUPPORTED
    assert L.cc_bcube_cost_batch_weighted(fake, 64, 2, fake, null, 0, null, null) == 0
    assert L.cc_cost_matrix_from_probes(null, 8, 10, 10, 1, fake, null) == INVALID
    assert L.cc_cost_matrix_from_probes(fake, 8, 0, 10, 1, fake, null) == INVALID
    assert L.cc_cost_matrix_from_probes(fake, 8, 16385, 10, 1, fake, null) == INVALID
    assert L.cc_cost_matrix_from_probes(fake, 8, 10, 101, 1, fake, null) == INVALID
    assert L.cc_cost_matrix_from_probes(fake, 1025, 10, 10, 1, fake, null) == UNSUPPORTED
    assert L.cc_dbt_cost_batch(fake, 1, fake, 1, fake, null) == UNSUPPORTED
    assert L.cc_dbt_cost_batch(fake, 48, fake, -1, fake, null) == INVALID
    assert L.cc_dbt_cost_batch(fake, 48, fake, 1, null, null) == INVALID
    assert L.cc_dbt_cost_batch(fake, 48, null, 0, null, null) == 0
    assert L.cc_sa_search(null, 64, 1, 10, 1, 1, 1, fake, fake, null) == INVALID
    assert L.cc_sa_search(fake, 64, 0, 10, 1, 1, 1, fake, fake, null) == INVALID          # no chains
    assert L.cc_sa_search(fake, 2000, 1, 10, 1, 1, 1, fake, fake, null) == UNSUPPORTED
    sa = [fake, 64, 4, 10, 1, 1, 1, null, fake, fake, null, null, null, null]
    assert L.cc_sa_search_ex(*sa, null, 0, null) == WORKSPACE
    sa[3] = (1 << 24) + 1
    assert L.cc_sa_search_ex(*sa, fake, 1 << 30, null) == INVALID                        # too many steps
    sa[3], sa[4] = 10, 1 << 21
    assert L.cc_sa_search_ex(*sa, fake, 1 << 30, null) == INVALID                        # temperature out of range
    sa[4], sa[5] = 1, -1
    assert L.cc_sa_search_ex(*sa, fake, 1 << 30, null) == INVALID
    assert L.cc_sa_rd_search(fake, 48, 1, 10, 1, 1, 1, fake, fake, null) == UNSUPPORTED      # not a power of two
    assert L.cc_sa_rd_search(fake, 64, 0, 10, 1, 1, 1, fake, fake, null) == INVALID
    assert L.cc_sa_rd_search_ex(fake, 64, 4, 10, 1, 1, 1, null, fake, fake, null, null, null, null, null, 0, null) == WORKSPACE
    assert L.cc_sa_workspace_bytes(64, 0) == 0 and L.cc_sa_workspace_bytes(64, 4) >= 4 * 64 * 4
    assert L.cc_2opt_search(null, 64, 0, 1, 1, fake, fake, null) == INVALID
    assert L.cc_2opt_search(fake, 64, 0, 0, 1, fake, fake, null) == INVALID
    assert L.cc_2opt_search(fake, 64, 9, 1, 1, fake, fake, null) == INVALID
    assert L.cc_2opt_search(fake, 64, 0, 1, 1, null, fake, null) == INVALID
    assert L.cc_2opt_search(fake, 2048, 0, 1, 1, fake, fake, null) == UNSUPPORTED
    args = [fake, 64, 0, 4, 1, null, fake, fake, null, null, null, null]
    assert L.cc_2opt_search_ex(*args, null, 0, null) == WORKSPACE
    assert L.cc_2opt_search_ex(*args, fake, 16, null) == WORKSPACE               # too small
    assert L.cc_2opt_search_ex(*args, ctypes.c_void_p(0x1004), 1 << 30, null) == WORKSPACE   # misaligned
    ws = ctypes.c_void_p(0x1000)
    assert L.cc_2opt_search_ex(fake, 64, 0, 4, 1, null, fake, null, null, fake, fake, null, ws, 1 << 30, null) == INVALID
    assert L.cc_2opt_search_ex(fake, 64, 0, 4, 1, null, null, null, null, null, fake, null, ws, 1 << 30, null) == INVALID
    assert L.cc_2opt_search_ex(fake, 64, 0, 4, 1, null, null, null, fake, fake, fake, null, ws, 1 << 30, null) == INVALID
    # move classes: only the documented (objective, classes) pairs are accepted
    for objective in range(4):
        for classes in range(0, 9):
            ok = (classes == 1 or (classes in (2, 3) and objective == 0) or (classes == 5 and objective in (2, 3)))
            rc = L.cc_local_search_ex(fake, 64, objective, classes, 4, 1, null, fake, fake, null, null, null, null,
                                      null, 0, null)
            assert rc == (WORKSPACE if ok else INVALID), (objective, classes)     # the workspace check comes last
            if not ok:
                assert L.cc_local_search(fake, 64, objective, classes, 4, 1, fake, fake, null) == INVALID
    assert L.cc_local_search(null, 64, 0, 3, 4, 1, fake, fake, null) == INVALID
    assert L.cc_local_search(fake, 64, 0, 3, 0, 1, fake, fake, null) == INVALID
    assert L.cc_local_search(fake, 1025, 0, 3, 1, 1, fake, fake, null) == UNSUPPORTED
    assert L.cc_best_of_restarts(null, fake, 64, 4, fake, fake, null, null) == INVALID
    assert L.cc_best_of_restarts(fake, fake, 64, 0, fake, fake, null, null) == INVALID
    assert L.cc_best_of_restarts(fake, fake, 1, 4, fake, fake, null, null) == UNSUPPORTED
    assert L.cc_rd_swap_search(null, 64, 1, 1, fake, fake, null) == INVALID
    assert L.cc_rd_swap_search(fake, 48, 1, 1, fake, fake, null) == UNSUPPORTED      # not a power of two
    assert L.cc_rd_swap_search(fake, 64, 0, 1, fake, fake, null) == INVALID
    assert L.cc_rd_swap_search(fake, 64, 1, 1, fake, null, null) == INVALID
    sargs = [fake, 64, 4, 1, null, fake, fake, null, null, null, null]
    assert L.cc_rd_swap_search_ex(*sargs, null, 0, null) == WORKSPACE
    assert L.cc_rd_swap_search_ex(*sargs, fake, 16, null) == WORKSPACE
    assert L.cc_rd_swap_workspace_bytes(64, 4) > 0 and L.cc_rd_swap_workspace_bytes(48, 4) == 0
    assert L.cc_init_tours(1, 0, 1, 1, fake, null) == UNSUPPORTED
    assert L.cc_init_tours(64, -1, 1, 1, fake, null) == INVALID
    assert L.cc_init_tours(64, 0, 1, 1, null, null) == INVALID
    assert L.cc_init_tours(64, 0, 0, 1, null, null) == 0
    assert L.cc_validate_matrix(null, 64, 1, null) == INVALID


def test_binding_refuses_cpu_tensors():
    import torch
    c = torch.zeros((8, 8), dtype=torch.int32)
    p = torch.zeros((1, 8), dtype=torch.int32)
    with pytest.raises(ValueError):
        cc.cc_ring_cost_batch(c, p, 0, out=torch.zeros(1, dtype=torch.int64), stream=_FakeStream())


class _FakeStream:
    cuda_stream = 0


def test_build_refuses_operand_reversed_dpp(tmp_path):
    """The build's check of the device assembly: a reversed-operand DPP form is refused, the forms the kernels rely
    on (plain rotates, add / sub / min / max with a DPP operand) pass."""
    from paper_2105_14088_amd import build as b
    good = tmp_path / "good-hip-amdgcn-amd-amdhsa-gfx950.s"
    good.write_text("\tv_mov_b32_dpp v1, v1 wave_rol:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n"
                    "\tv_sub_u32_dpp v3, v29, v3 wave_ror:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n"
                    "\tv_lshlrev_b32_e32 v2, 2, v1\n\tv_subrev_u32_e32 v2, v3, v1\n")
    b.check_device_isa(str(tmp_path))
    bad = tmp_path / "bad-hip-amdgcn-amd-amdhsa-gfx950.s"
    bad.write_text("\tv_add_u32_e32 v1, v2, v3\n"
                   "\tv_subrev_u32_dpp v75, v75, v74 wave_rol:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n")
    with pytest.raises(RuntimeError, match="v_subrev_u32_dpp"):
        b.check_device_isa(str(tmp_path))
