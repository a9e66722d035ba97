"""IEEE special values.  (1) Positions that do not exist (the padding of the last tile, lanes past the end of a
batch, columns outside a column pass) are guarded, not multiplied by zero: a NaN in an entry of the dense
operand that no stored position refers to must not reach any output.  (2) A NaN or Inf that IS referred to
propagates to exactly the rows that refer to it."""
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
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def shifted(A):
    """The same matrix with every column moved up by one: column 0 is referred to by nobody."""
    return wl.CSR(A.rows, A.cols + 1, A.pos, (A.crd + 1).astype(np.int32), A.vals, A.bs)


def close(got, ref, mag, what, rel=1e-5, floor=1e-30):
    assert np.isfinite(got).all(), what + ": non-finite output"
    ok, worst = oracle.within_tolerance(got, ref, mag, rel, floor)
    assert ok, "%s: %.3g" % (what, worst)


def test_unreferenced_nan_never_reaches_an_output():
    rng = np.random.default_rng(91)
    L = np.minimum(rng.zipf(1.5, size=3000), 2500)
    A = shifted(wl.csr_from_lengths(L, 2600, seed=91))           # nnz is not a multiple of any tile
    x = wl.dense_uniform(A.cols, 91, wl.S_X); x[0] = np.nan
    pos, crd, vals = dev(A.pos), dev(A.crd), dev(A.vals)
    ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, x)
    assert np.isfinite(ref).all()
    for tile in (256, 1024, 4096):
        for passes in (1, 2, 3):
            say("spmv nan-guard tile", tile, "passes", passes)
            y = torch.empty(A.rows, device="cuda")
            psk.psk_spmv_csr(A.rows, A.cols, A.nnz, pos, crd, vals, dev(x), y, tile=tile, col_passes=passes)
            close(y.cpu().numpy(), ref, mag, "spmv tile %d passes %d" % (tile, passes))
    for fn in (psk.psk_spmv_csr_notemp, psk.psk_spmv_csr_atomics):
        y = torch.empty(A.rows, device="cuda")
        fn(A.rows, A.cols, A.nnz, pos, crd, vals, dev(x), y)
        close(y.cpu().numpy(), ref, mag, fn.__name__)
    y = torch.empty(A.rows, device="cuda")
    psk.psk_spmv_csr_divide(A.rows, A.cols, A.nnz, pos, crd, vals, dev(x), y, parts=7)
    close(y.cpu().numpy(), ref, mag, "divide")
    # fp64
    v64 = wl.dense_uniform_f64(A.nnz, 91, wl.S_VALS); x64 = wl.dense_uniform_f64(A.cols, 91, wl.S_X); x64[0] = np.nan
    r64, m64 = oracle.spmv_csr_f64(A.pos, A.crd, v64, x64)
    for passes in (1, 3):
        y64 = torch.empty(A.rows, dtype=torch.float64, device="cuda")
        psk.psk_spmv_csr_f64(A.rows, A.cols, A.nnz, pos, crd, dev(v64), dev(x64), y64, col_passes=passes)
        close(y64.cpu().numpy(), r64, m64, "f64 passes %d" % passes, 1e-14, 1e-300)
    # SpMM, wide and narrow
    for k in (5, 32, 64, 130):
        B = wl.dense_uniform(A.cols * k, 92, wl.S_B).reshape(A.cols, k); B[0, :] = np.nan
        refC, magC = oracle.spmm_csr(A.pos, A.crd, A.vals, B)
        C = torch.empty((A.rows, k), device="cuda")
        say("spmm nan-guard k", k)
        psk.psk_spmm_csr(A.rows, A.cols, A.nnz, pos, crd, vals, dev(B), C, tile=256)
        close(C.cpu().numpy(), refC, magC, "spmm k %d" % k)
    # BCSR 2, 4, 8
    for bs in (2, 4, 8):
        Ab = shifted(wl.csr_from_lengths(np.minimum(L, 300), 400, seed=93, bs=bs))
        xb = wl.dense_uniform(Ab.cols * bs, 93, wl.S_X); xb[:bs] = np.nan
        rb, mb = oracle.spmv_bcsr(Ab.pos, Ab.crd, Ab.vals, xb, bs)
        yb = torch.empty(Ab.rows * bs, device="cuda")
        say("bcsr nan-guard bs", bs)
        psk.psk_spmv_bcsr(Ab.rows, Ab.cols, Ab.nnz, bs, dev(Ab.pos), dev(Ab.crd), dev(Ab.vals), dev(xb), yb)
        close(yb.cpu().numpy(), rb, mb, "bcsr spmv %d" % bs)
        Bb = wl.dense_uniform(Ab.cols * bs * 40, 94, wl.S_B).reshape(Ab.cols * bs, 40); Bb[:bs, :] = np.nan
        rC, mC = oracle.spmm_bcsr(Ab.pos, Ab.crd, Ab.vals, Bb, bs)
        Cb = torch.empty((Ab.rows * bs, 40), device="cuda")
        psk.psk_spmm_bcsr(Ab.rows, Ab.cols, Ab.nnz, bs, dev(Ab.pos), dev(Ab.crd), dev(Ab.vals), dev(Bb), Cb)
        close(Cb.cpu().numpy(), rC, mC, "bcsr spmm %d" % bs)
    # MTTKRP: row 0 of C and of D unreferenced
    T = wl.csf3_powerlaw(1500, 300, 700, 4, 1.6, 200, seed=95)
    for j in (7, 32, 64):
        Cm = wl.dense_uniform((T.dims[1] + 1) * j, 96, wl.S_B).reshape(-1, j); Cm[0, :] = np.nan
        Dm = wl.dense_uniform((T.dims[2] + 1) * j, 97, wl.S_B).reshape(-1, j); Dm[0, :] = np.nan
        ck, cl = (T.crd_k + 1).astype(np.int32), (T.crd_l + 1).astype(np.int32)
        rA, mA = oracle.mttkrp_csf3(T.pos_k, ck, T.pos_l, cl, T.vals, Cm, Dm)
        Aout = torch.empty((T.dims[0], j), device="cuda")
        say("mttkrp nan-guard j", j)
        psk.psk_mttkrp_csf3((T.dims[0], T.dims[1] + 1, T.dims[2] + 1), None, dev(T.pos_k), dev(ck), dev(T.pos_l), dev(cl),
                            dev(T.vals), dev(Cm), dev(Dm), Aout, tile=256)
        close(Aout.cpu().numpy(), rA, mA, "mttkrp j %d" % j)


def test_referenced_nan_and_inf_propagate_to_their_rows_only():
    A = wl.csr_from_lengths(np.random.default_rng(98).integers(0, 30, size=2000), 500, seed=98)
    x = wl.dense_uniform(500, 98, wl.S_X)
    x[17] = np.nan
    x[333] = np.inf
    D = np.zeros((A.rows, 2), dtype=bool)
    for r in range(A.rows):
        cols = A.crd[A.pos[r]:A.pos[r + 1]]
        D[r, 0] = 17 in cols
        D[r, 1] = 333 in cols
    for passes in (1, 2):
        y = torch.empty(A.rows, device="cuda")
        psk.psk_spmv_csr(A.rows, A.cols, A.nnz, dev(A.pos), dev(A.crd), dev(A.vals), dev(x), y, tile=256, col_passes=passes)
        got = y.cpu().numpy()
        assert (np.isnan(got) == D[:, 0]).all()
        assert (np.isinf(got) == (D[:, 1] & ~D[:, 0])).all()
        assert np.isfinite(got[~D[:, 0] & ~D[:, 1]]).all()
