"""The C-ABI library loads, exports every function include/psk.h declares, and its host-side
argument checks answer without touching a GPU."""
import ctypes
import os
import re

import pytest

import paper_2001_00532_amd as psk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "psk.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(psk_[a-z0-9_]+)\s*\(", text)))


def test_header_and_library_agree():
    names = declared_functions()
    assert set(names) == set(psk.EXPORTS)
    L = psk.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_sizes_and_strings():
    assert psk.psk_version() >= 100
    assert psk.psk_num_tiles(0, 1024) == 0 and psk.psk_num_tiles(1, 1024) == 1
    assert psk.psk_num_tiles(1024, 1024) == 1 and psk.psk_num_tiles(1025, 1024) == 2
    assert psk.psk_num_tiles(10, 0) == -1
    for op in range(6):
        assert psk.psk_default_tile(op) > 0
    assert psk.psk_default_tile(9) == -1
    assert psk.psk_default_tile_bcsr(psk.PSK_OP_SPMV_BCSR, 4) == psk.psk_default_tile(psk.PSK_OP_SPMV_BCSR)
    assert psk.psk_default_tile_bcsr(psk.PSK_OP_SPMV_BCSR, 2) > 0 and psk.psk_default_tile_bcsr(psk.PSK_OP_SPMV_BCSR, 8) > 0
    assert psk.psk_default_tile_bcsr(psk.PSK_OP_SPMV_BCSR, 3) == -1 and psk.psk_default_tile_bcsr(psk.PSK_OP_SPMV_CSR, 4) == -1
    w = psk.psk_workspace_bytes(psk.PSK_OP_SPMV_CSR, 100, 10_000, tile=1024)
    assert w >= 256 and w % 256 == 0
    assert psk.psk_workspace_bytes(psk.PSK_OP_SPMM_CSR, 100, 10_000, k=128, tile=1024) > w
    assert psk.psk_workspace_bytes(psk.PSK_OP_SPMM_CSR, 100, 10_000, k=0, tile=1024) == 0
    assert psk.psk_workspace_bytes(7, 100, 10_000) == 0
    # fp64 carries are doubles: twice the record space of the fp32 SpMV
    assert psk.psk_workspace_bytes(psk.PSK_OP_SPMV_CSR_F64, 100, 10_000_000, tile=1024) > \
        psk.psk_workspace_bytes(psk.PSK_OP_SPMV_CSR, 100, 10_000_000, tile=1024)
    assert psk.psk_workspace_bytes(psk.PSK_OP_MTTKRP_CSF3, 100, 10_000, k=64) > w
    assert psk.psk_workspace_bytes(psk.PSK_OP_SPMV_CSR, 0, 0) >= 256
    assert psk.status_string(0) == "ok" and "tile" in psk.status_string(3)
    assert psk.status_string(99) == "unknown status"


def test_argument_errors_are_reported_before_any_launch():
    """All of these return on the host-side checks; no HIP call is made."""
    L = psk.lib()
    one = ctypes.c_void_p(256)        # a non-NULL, 256-byte aligned dummy address, never dereferenced
    null = ctypes.c_void_p(0)
    big = 1 << 20
    # SIZE
    assert L.psk_spmv_csr(-1, 4, 0, one, one, one, one, one, 0, 1, 7, one, big, null) == 2
    assert L.psk_spmv_csr(4, 4, 2 ** 31, one, one, one, one, one, 0, 1, 7, one, big, null) == 2
    assert L.psk_spmv_csr(0, 4, 5, one, one, one, one, one, 0, 1, 7, one, big, null) == 2
    assert L.psk_spmm_csr(4, 4, 4, one, one, one, one, 0, 8, one, 8, 0, 7, one, big, null) == 2       # k = 0
    assert L.psk_spmm_csr(4, 4, 4, one, one, one, one, 8, 4, one, 8, 0, 7, one, big, null) == 2       # ldb < k
    assert L.psk_spmv_bcsr(4, 4, 4, 0, one, one, one, one, one, 0, 7, one, big, null) == 2            # bs = 0
    # NULL
    assert L.psk_spmv_csr(4, 4, 4, null, one, one, one, one, 0, 1, 7, one, big, null) == 1
    assert L.psk_spmv_csr(4, 4, 4, one, null, one, one, one, 0, 1, 7, one, big, null) == 1
    assert L.psk_spmv_csr(4, 4, 4, one, one, one, null, one, 0, 1, 7, one, big, null) == 1
    assert L.psk_spmv_csr(4, 4, 4, one, one, one, one, null, 0, 1, 7, one, big, null) == 1
    assert L.psk_partition_csr(4, 4, null, 4, 0, one, null) == 1
    # TILE
    assert L.psk_spmv_csr(4, 4, 4, one, one, one, one, one, 1000, 1, 7, one, big, null) == 3
    assert L.psk_spmm_csr(4, 4, 4, one, one, one, one, 8, 8, one, 8, 4096, 7, one, big, null) == 3
    assert L.psk_partition_csr(4, 4, one, 0, 0, one, null) == 3
    assert L.psk_partition_csr(4, 4, one, 4, 3, one, null) == 5
    # WORKSPACE
    assert L.psk_spmv_csr(4, 4, 4, one, one, one, one, one, 0, 1, 7, null, big, null) == 4
    assert L.psk_spmv_csr(4, 4, 4, one, one, one, one, one, 0, 1, 7, one, 16, null) == 4
    assert L.psk_spmv_csr(4, 4, 4, one, one, one, one, one, 0, 1, 7, ctypes.c_void_p(264), big, null) == 4
    # UNSUPPORTED
    assert L.psk_spmv_csr(4, 4, 4, one, one, one, one, one, 0, 1, 0, one, big, null) == 5
    assert L.psk_spmv_csr(4, 4, 4, one, one, one, one, one, 0, 1, 8, one, big, null) == 5
    assert L.psk_spmv_bcsr(4, 4, 4, 3, one, one, one, one, one, 0, 7, one, big, null) == 5
    assert L.psk_spmv_bcsr(4, 4, 4, 2, one, one, one, one, one, 64, 7, one, big, null) == 3              # tile of another block size
    assert L.psk_spmv_csr_rowsplit(4, 4, 4, one, one, one, one, one, 2, null) == 5
    assert L.psk_spmv_csr(4, 4, 4, one, one, one, one, one, 0, 9, 7, one, big, null) == 2                # col_passes
    out = ctypes.c_int32(-1)
    assert L.psk_analyze_csr(4, 4, 4, one, one, null, 0, ctypes.byref(out), null) == 4
    assert L.psk_analyze_csr(4, 4, 4, one, one, one, 256, None, null) == 1
    assert L.psk_analyze_csr(4, 4, 4, one, one, one, 256, ctypes.byref(out), null) == 0 and out.value == 1   # small: no launch
    # the widened entry points: MTTKRP, fp64, DCSR, divided, ablations, selector
    assert L.psk_mttkrp_csf3(4, 4, 4, 4, 4, 4, null, null, one, one, one, one, one, 8, one, 8, 8, one, 8, 0, 7, one, big, null) == 1
    assert L.psk_mttkrp_csf3(4, 4, 4, 4, 4, 4, null, one, one, one, one, one, one, 8, one, 8, 0, one, 8, 0, 7, one, big, null) == 2   # j = 0
    assert L.psk_mttkrp_csf3(4, 4, 4, 4, 4, 4, null, one, one, one, one, one, one, 4, one, 8, 8, one, 8, 0, 7, one, big, null) == 2   # ldc < j
    assert L.psk_mttkrp_csf3(4, 4, 4, 4, 4, 4, null, one, one, one, one, one, one, 8, one, 8, 8, one, 8, 100, 7, one, big, null) == 3
    assert L.psk_partition_csf3(4, 4, 4, null, one, 4, one, one, null) == 1
    assert L.psk_partition_csf3(4, 4, 4, one, one, 0, one, one, null) == 3
    assert L.psk_spmv_csr_f64(4, 4, 4, one, one, one, one, null, 0, 1, 7, one, big, null) == 1
    assert L.psk_spmv_csr_f64(4, 4, 4, one, one, ctypes.c_void_p(260), one, one, 0, 1, 7, one, big, null) == 7
    assert L.psk_spmv_csr_f64(4, 4, 4, one, one, one, one, one, 4096, 1, 7, one, big, null) == 3
    assert L.psk_spmv_csr_f64(4, 4, 4, one, one, one, one, one, 0, 7, 7, one, big, null) == 2          # col_passes
    assert L.psk_spmv_dcsr(8, 4, 9, 4, one, one, one, one, one, one, 0, 0, 1, 7, one, big, null) == 2      # nstored > rows
    assert L.psk_spmv_dcsr(8, 4, 2, 4, null, one, one, one, one, one, 0, 0, 1, 7, one, big, null) == 1
    assert L.psk_spmv_dcsr(8, 4, 2, 4, one, one, one, one, one, one, 2, 0, 1, 7, one, big, null) == 5      # cut
    assert L.psk_spmv_dcsr(8, 4, 2, 4, one, one, one, one, one, one, 0, 0, 9, 7, one, big, null) == 2      # col_passes
    assert L.psk_spmv_csr_divide(4, 4, 4, one, one, one, one, one, -1, 7, one, big, null) == 2
    assert L.psk_spmv_csr_divide(4, 4, 4, one, one, one, one, one, 0, 7, null, big, null) == 4
    assert L.psk_spmv_csr_notemp(4, 4, 4, one, one, one, one, one, 100, 7, one, big, null) == 3
    assert L.psk_spmv_csr_atomics(4, 4, 4, one, one, null, one, one, 0, 7, one, big, null) == 1
    assert L.psk_validate_csr(4, 4, 4, one, one, one, 256, None, null) == 1
    assert L.psk_validate_csr(4, 4, 4, one, one, null, 0, ctypes.byref(out), null) == 4
    assert L.psk_suggest_schedule_csr(4, 4, one, one, 256, None, null) == 1
    assert L.psk_suggest_schedule_csr(4, 4, one, null, 0, ctypes.byref(out), null) == 4
    assert L.psk_suggest_schedule_csr(4, 4, one, one, 256, ctypes.byref(out), null) == 0 and out.value == 0  # short rows: no launch
    # ALIGNMENT (BCSR)
    assert L.psk_spmv_bcsr(4, 4, 4, 4, one, one, ctypes.c_void_p(260), one, one, 0, 7, one, big, null) == 7


def test_binding_refuses_host_tensors():
    import torch

    t = torch.zeros(4, dtype=torch.int32)
    with pytest.raises(ValueError):
        psk.psk_partition_csr(t, 0, 4)


def test_binding_refuses_partial_products_on_a_temporary_workspace():
    """Main or fix-up without the partition step read the table from the workspace: a workspace made for the call
    holds garbage row numbers, so the binding refuses before anything reaches the library."""
    for fn, args in ((psk.psk_spmv_csr, (4, 4, 4, None, None, None, None, None)),
                     (psk.psk_spmv_bcsr, (4, 4, 4, 4, None, None, None, None, None)),
                     (psk.psk_spmv_csr_notemp, (4, 4, 4, None, None, None, None, None))):
        with pytest.raises(ValueError):
            fn(*args, phases=psk.PSK_PHASE_MAIN)
        with pytest.raises(ValueError):
            fn(*args, phases=psk.PSK_PHASE_MAIN | psk.PSK_PHASE_FIXUP)
    with pytest.raises(ValueError):
        psk.psk_spmv_csr_divide(4, 4, 4, None, None, None, None, None, phases=psk.PSK_PHASE_MAIN)
