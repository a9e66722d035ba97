"""The entry points only enqueue kernels on the caller's stream (no allocation, no synchronisation, no
memset nodes), so a product can be captured into a HIP graph and replayed.  Every replay is checked
against the eager result, with eager work and synchronisations between the replays."""
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


def test_captured_products_replay_correctly():
    c = wl.config(2, 0.02)
    A = c["A"]
    pos, crd, vals = dev(A.pos), dev(A.crd), dev(A.vals)
    x = dev(c["x"])
    y = torch.zeros(A.rows, device="cuda")
    ws = psk.workspace(psk.PSK_OP_SPMV_CSR, A.rows, A.nnz)
    c4 = wl.config(4, 0.002)
    M = c4["A"]
    mpos, mcrd, mvals, B = dev(M.pos), dev(M.crd), dev(M.vals), dev(c4["B"])
    C = torch.zeros((M.rows, 128), device="cuda")
    ws2 = psk.workspace(psk.PSK_OP_SPMM_CSR, M.rows, M.nnz, k=128)

    # warm-up on a side stream, then capture
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        psk.psk_spmv_csr(A.rows, A.cols, A.nnz, pos, crd, vals, x, y, col_passes=2, ws=ws)
        psk.psk_spmm_csr(M.rows, M.cols, M.nnz, mpos, mcrd, mvals, B, C, ws=ws2)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    say("capturing")
    with torch.cuda.graph(g):
        psk.psk_spmv_csr(A.rows, A.cols, A.nnz, pos, crd, vals, x, y, col_passes=2, ws=ws)
        psk.psk_spmm_csr(M.rows, M.cols, M.nnz, mpos, mcrd, mvals, B, C, ws=ws2)
    for rep in range(4):
        xh = wl.dense_uniform(A.cols, 100 + rep, wl.S_X)
        Bh = wl.dense_uniform(M.cols * 128, 200 + rep, wl.S_B).reshape(M.cols, 128)
        x.copy_(dev(xh))
        B.copy_(dev(Bh))
        y.fill_(float("nan"))
        C.fill_(float("nan"))
        ws.fill_(0xFF)                      # the replay must rebuild the table and the carries itself
        ws2.fill_(0xFF)
        say("replay", rep)
        g.replay()
        torch.cuda.synchronize()
        y_eager = torch.empty_like(y)
        C_eager = torch.empty_like(C)
        psk.psk_spmv_csr(A.rows, A.cols, A.nnz, pos, crd, vals, x, y_eager, col_passes=2)
        psk.psk_spmm_csr(M.rows, M.cols, M.nnz, mpos, mcrd, mvals, B, C_eager)
        torch.cuda.synchronize()
        assert torch.equal(y, y_eager) and torch.equal(C, C_eager), "replay %d differs from the eager result" % rep
        ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, xh, threads=8)
        ok, worst = oracle.within_tolerance(y.cpu().numpy(), ref, mag)
        assert ok, "replay %d: %.3g" % (rep, worst)
        ref, mag = oracle.spmm_csr(M.pos, M.crd, M.vals, Bh, threads=8)
        ok, worst = oracle.within_tolerance(C.cpu().numpy(), ref, mag)
        assert ok, "replay %d, C: %.3g" % (rep, worst)


def test_captured_slab_products_replay_correctly():
    """The products over the column-slab structure (fp32 and fp64) captured into one graph: the structure is built
    before the capture (its build synchronises), the products only enqueue kernels."""
    A = wl.config(2, 0.02)["A"]
    pos, crd = dev(A.pos), dev(A.crd)
    v64 = wl.dense_uniform_f64(A.nnz, 31, wl.S_VALS)
    S32 = psk.psk_slab_build_csr(A.rows, A.cols, A.nnz, pos, crd, dev(A.vals))
    S64 = psk.psk_slab_build_csr_f64(A.rows, A.cols, A.nnz, pos, crd, dev(v64))
    ws32, ws64 = psk.psk_slab_spmv_workspace(S32), psk.psk_slab_spmv_workspace(S64)
    x32 = torch.zeros(A.cols, device="cuda")
    x64 = torch.zeros(A.cols, dtype=torch.float64, device="cuda")
    y32 = torch.zeros(A.rows, device="cuda")
    y64 = torch.zeros(A.rows, dtype=torch.float64, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        psk.psk_spmv_slab(S32, x32, y32, ws=ws32)
        psk.psk_spmv_slab_f64(S64, x64, y64, ws=ws64)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    say("capturing the slab products")
    with torch.cuda.graph(g):
        psk.psk_spmv_slab(S32, x32, y32, ws=ws32)
        psk.psk_spmv_slab_f64(S64, x64, y64, ws=ws64)
    for rep in range(4):
        xh = wl.dense_uniform(A.cols, 300 + rep, wl.S_X)
        xh64 = wl.dense_uniform_f64(A.cols, 400 + rep, wl.S_X)
        x32.copy_(dev(xh))
        x64.copy_(dev(xh64))
        y32.fill_(float("nan"))
        y64.fill_(float("nan"))
        ws32.fill_(0xFF)
        ws64.fill_(0xFF)
        say("slab replay", rep)
        g.replay()
        torch.cuda.synchronize()
        e32, e64 = torch.empty_like(y32), torch.empty_like(y64)
        psk.psk_spmv_slab(S32, x32, e32)
        psk.psk_spmv_slab_f64(S64, x64, e64)
        torch.cuda.synchronize()
        assert torch.equal(y32, e32) and torch.equal(y64, e64), "slab replay %d differs from the eager result" % rep
        ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, xh, threads=8)
        ok, worst = oracle.within_tolerance(y32.cpu().numpy(), ref, mag)
        assert ok, "slab replay %d: %.3g" % (rep, worst)
        ref, mag = oracle.spmv_csr_f64(A.pos, A.crd, v64, xh64, threads=8)
        ok, worst = oracle.within_tolerance(y64.cpu().numpy(), ref, mag, 1e-14, 1e-300)
        assert ok, "fp64 slab replay %d: %.3g" % (rep, worst)
