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


def test_slab_product_refuses_a_struct_that_no_build_made():
    """The product over the slab structure checks, on the host and before any launch, that the sizes in the struct are
    the kind a build leaves (they decide grids and index ranges of its kernels)."""
    L = psk.lib()
    one = ctypes.c_void_p(256)

    def struct(**over):
        d = psk.psk_slab()
        d.rows, d.cols, d.nnz = 1000, 100_000, 5000
        d.slab_cols, d.chunk, d.tile, d.value_bytes = 32736, 512, 2048, 4
        d.nslabs = 4
        d.nchunks = 12
        d.nslots = 12 * 512
        d.npairs, d.nq = 5200, 5000
        for name in ("svals", "scol", "chunk_pair", "slab_chunk", "qpos", "qidx", "qtile_row"):
            setattr(d, name, 256)
        for k, v in over.items():
            setattr(d, k, v)
        return d

    def product(d, f64=False):
        fn = L.psk_spmv_slab_f64 if f64 else L.psk_spmv_slab
        return fn(ctypes.byref(d), one, one, 7, None, 0, None)

    assert product(struct()) == 4                       # consistent sizes: only the workspace is missing
    for over in (dict(nslabs=3), dict(nchunks=13), dict(nslots=12 * 512 + 1), dict(nslots=8 * 512, nchunks=8),
                 dict(npairs=12 * 512 + 1), dict(nq=5201), dict(nq=5300, npairs=5300), dict(npairs=0, nq=0),
                 dict(slab_cols=16352), dict(chunk=256), dict(tile=1024), dict(value_bytes=8), dict(rows=-1),
                 dict(nslots=40 * 512, nchunks=40)):
        assert product(struct(**over)) == 2, over
    assert product(struct(), f64=True) == 2             # a structure of the other value type
    assert product(struct(value_bytes=8, slab_cols=16352, tile=1024, nslabs=7), f64=True) == 4
