"""The entry point that allocates nothing: psk_spmv_csr_static keeps the tile->row table, the carry records
and the column ranges in the library's built-in scratch array instead of a caller's workspace.  Called
through the C ABI (raw ctypes, device pointers), twice in a row, the second time on a smaller matrix, and
compared with psk_spmv_csr (bit for bit: same kernels, same tile) and with the oracle."""
import ctypes
import sys

import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_2001_00532_amd as psk  # noqa: E402


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def vp(t):
    return ctypes.c_void_p(t.data_ptr())


def product_pair(A, xh, tile, passes):
    """(y from the static entry point, y from psk_spmv_csr with a workspace), both through the raw C ABI."""
    L = psk.lib()
    pos, crd, vals, x = dev(A.pos), dev(A.crd), dev(A.vals), dev(xh)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    y_static = torch.full((A.rows,), float("nan"), device="cuda")
    y_ws = torch.full((A.rows,), float("nan"), device="cuda")
    ws = psk.workspace(psk.PSK_OP_SPMV_CSR, A.rows, A.nnz, tile=tile)
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["num_alloc_retries"], torch.cuda.memory_allocated()
    st = L.psk_spmv_csr_static(A.rows, A.cols, A.nnz, vp(pos), vp(crd), vp(vals), vp(x), vp(y_static), tile, passes,
                               stream)
    assert st == 0, psk.status_string(st)
    assert (torch.cuda.memory_stats()["num_alloc_retries"], torch.cuda.memory_allocated()) == before
    st = L.psk_spmv_csr(A.rows, A.cols, A.nnz, vp(pos), vp(crd), vp(vals), vp(x), vp(y_ws), tile, passes, 7, vp(ws),
                        ws.numel(), stream)
    assert st == 0, psk.status_string(st)
    torch.cuda.synchronize()
    return y_static.cpu().numpy(), y_ws.cpu().numpy()


@pytest.mark.parametrize("tile,passes", [(0, 1), (1024, 2), (256, 1)])
def test_static_scratch_matches_workspace_path_twice_in_a_row(tile, passes):
    big = wl.config(2, 0.02)            # power-law rows: long rows span tiles, so carries are exercised
    small = wl.config(2, 0.004)
    for name, c in (("first call", big), ("second call, smaller matrix", small)):
        A = c["A"]
        say("static scratch:", name, "rows", A.rows, "nnz", A.nnz, "tile", tile, "passes", passes)
        got, want = product_pair(A, c["x"], tile, passes)
        assert np.array_equal(got, want), "%s: differs from psk_spmv_csr" % name
        ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, c["x"], threads=8)
        ok, worst = oracle.within_tolerance(got, ref, mag)
        assert ok, "%s: worst |err|/bound = %.3g" % (name, worst)


def test_static_scratch_rejects_what_does_not_fit():
    L = psk.lib()
    one = ctypes.c_void_p(256)
    assert psk.psk_static_scratch_bytes() == 4 << 20
    # 2^31 - 1 nonzeros in tiles of 256 need far more than 4 MiB of table and carries
    assert L.psk_spmv_csr_static(4, 4, 2 ** 31 - 1, one, one, one, one, one, 256, 1, None) == 4
    assert L.psk_spmv_csr_static(4, 4, 4, one, one, one, one, one, 1000, 1, None) == 3
    assert L.psk_spmv_csr_static(4, 4, 4, None, one, one, one, one, 0, 1, None) == 1
    assert L.psk_spmv_csr_static(-1, 4, 4, one, one, one, one, one, 0, 1, None) == 2
    # an empty product is valid and only zero-fills y
    y = torch.full((5,), float("nan"), device="cuda")
    pos = torch.zeros(6, dtype=torch.int32, device="cuda")
    assert L.psk_spmv_csr_static(5, 3, 0, vp(pos), None, None, None, vp(y), 0, 1, None) == 0
    torch.cuda.synchronize()
    assert bool((y == 0).all())
