"""Seeded random problems for the widened entry points: DCSR (both cuts, column passes), fp64 SpMV, the
divided variant, the ablation kernels, other block sizes and MTTKRP, each against the oracle."""
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


def ok32(got, ref, mag, what):
    ok, worst = oracle.within_tolerance(got, ref, mag, 1e-5, 1e-30)
    assert ok, "%s: worst |err|/bound = %.3g" % (what, worst)


def lengths(rng, rows, cols):
    style = int(rng.integers(0, 4))
    if style == 0:
        return rng.integers(0, min(cols, 12) + 1, size=rows)
    if style == 1:
        return np.where(rng.random(rows) < 0.9, 0, rng.integers(0, min(cols, 400) + 1, size=rows))
    if style == 2:
        return np.minimum(rng.zipf(1.6, size=rows), cols)
    L = np.zeros(rows, dtype=np.int64)
    L[rng.integers(0, rows, size=3)] = min(cols, int(rng.integers(1, 9000)))
    return L


def test_random_matrices_widened_entry_points():
    rng = np.random.default_rng(532)
    for case in range(40):
        rows = int(rng.integers(1, 5000))
        cols = int(rng.integers(1, 9000))
        L = lengths(rng, rows, cols)
        seed = 3000 + case
        A = wl.csr_from_lengths(L, cols, seed=seed)
        x = wl.dense_uniform(cols, seed, wl.S_X)
        say("case", case, "rows", rows, "cols", cols, "nnz", A.nnz)
        pos, crd, vals, xd = dev(A.pos), dev(A.crd), dev(A.vals), dev(x)
        ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, x)
        # divided, ablations
        for parts in (0, int(rng.integers(1, 50))):
            y = torch.full((rows,), float("nan"), device="cuda")
            psk.psk_spmv_csr_divide(rows, cols, A.nnz, pos, crd, vals, xd, y, parts=parts)
            torch.cuda.synchronize()
            ok32(y.cpu().numpy(), ref, mag, "case %d divide parts %d" % (case, parts))
        tile = int(rng.choice([0, 256, 512, 1024, 2048, 4096]))
        for fn in (psk.psk_spmv_csr_notemp, psk.psk_spmv_csr_atomics):
            y = torch.full((rows,), float("nan"), device="cuda")
            fn(rows, cols, A.nnz, pos, crd, vals, xd, y, tile=tile)
            torch.cuda.synchronize()
            ok32(y.cpu().numpy(), ref, mag, "case %d %s tile %d" % (case, fn.__name__, tile))
        # fp64
        v64 = wl.dense_uniform_f64(A.nnz, seed, wl.S_VALS)
        x64 = wl.dense_uniform_f64(cols, seed, wl.S_X)
        r64, m64 = oracle.spmv_csr_f64(A.pos, A.crd, v64, x64)
        y64 = torch.full((rows,), float("nan"), dtype=torch.float64, device="cuda")
        t64 = int(rng.choice([0, 256, 512, 1024, 2048]))
        psk.psk_spmv_csr_f64(rows, cols, A.nnz, pos, crd, dev(v64), dev(x64), y64, tile=t64)
        torch.cuda.synchronize()
        ok, worst = oracle.within_tolerance(y64.cpu().numpy(), r64, m64, 1e-14, 1e-300)
        assert ok, "case %d f64 tile %d: %.3g" % (case, t64, worst)
        # DCSR: the same stored rows scattered over a larger row space
        big = rows + int(rng.integers(0, 100000))
        Dm = wl.dcsr_from_lengths(big, L, cols, seed=seed)
        rd, md = oracle.spmv_dcsr(big, Dm.crd_i, Dm.pos, Dm.crd, Dm.vals, x)
        for cut, passes in ((psk.PSK_CUT_POSITIONS, 1), (psk.PSK_CUT_POSITIONS, int(rng.integers(2, 5))), (psk.PSK_CUT_ROWS, 1)):
            yd = torch.full((big,), float("nan"), device="cuda")
            psk.psk_spmv_dcsr(big, cols, Dm.nnz, dev(Dm.crd_i), dev(Dm.pos), dev(Dm.crd), dev(Dm.vals), xd, yd, cut=cut,
                              tile=tile if passes == 1 else 0, col_passes=passes)
            torch.cuda.synchronize()
            ok32(yd.cpu().numpy(), rd, md, "case %d dcsr cut %d passes %d" % (case, cut, passes))
        # other block sizes on the same pattern (every fourth case: the operands grow with bs^2)
        if case % 4 == 1:
            for bs in (2, 8):
                Ab = wl.csr_from_lengths(L, cols, seed=seed, bs=bs)
                xb = wl.dense_uniform(cols * bs, seed, wl.S_X)
                rb, mb = oracle.spmv_bcsr(Ab.pos, Ab.crd, Ab.vals, xb, bs)
                yb = torch.full((rows * bs,), float("nan"), device="cuda")
                psk.psk_spmv_bcsr(rows, cols, Ab.nnz, bs, dev(Ab.pos), dev(Ab.crd), dev(Ab.vals), dev(xb), yb)
                torch.cuda.synchronize()
                ok32(yb.cpu().numpy(), rb, mb, "case %d bcsr %d spmv" % (case, bs))
                kb = int(rng.choice([3, 64, 130]))
                Bb = wl.dense_uniform(cols * bs * kb, seed, wl.S_B).reshape(cols * bs, kb)
                rC, mC = oracle.spmm_bcsr(Ab.pos, Ab.crd, Ab.vals, Bb, bs)
                Cb = torch.full((rows * bs, kb), float("nan"), device="cuda")
                psk.psk_spmm_bcsr(rows, cols, Ab.nnz, bs, dev(Ab.pos), dev(Ab.crd), dev(Ab.vals), dev(Bb), Cb)
                torch.cuda.synchronize()
                ok32(Cb.cpu().numpy(), rC, mC, "case %d bcsr %d spmm k %d" % (case, bs, kb))


def test_random_tensors_mttkrp():
    rng = np.random.default_rng(533)
    for case in range(30):
        ns = int(rng.integers(1, 600))
        K, Ld = int(rng.integers(1, 300)), int(rng.integers(1, 3000))
        fps = np.minimum(lengths(rng, ns, K), K)
        nf = int(fps.sum())
        lpf = np.minimum(lengths(rng, nf, Ld), Ld) if nf else np.zeros(0, dtype=np.int64)
        ci = bool(rng.integers(0, 2))
        I = ns + (int(rng.integers(0, 500)) if ci else 0)
        T = wl.csf3_from_lengths(fps, lpf, (I, K, Ld), seed=4000 + case, compressed_i=ci)
        j = int(rng.choice([1, 7, 32, 64, 96, 128, 256]))
        tile = int(rng.choice([0, 256, 512, 1024, 2048]))
        say("tensor", case, "slices", ns, "fibers", T.nfibers, "nnz", T.nnz, "j", j, "tile", tile, "compressed i", ci)
        C = wl.dense_uniform(K * j, case, wl.S_B).reshape(K, j)
        D = wl.dense_uniform(Ld * j, case + 1, wl.S_B).reshape(Ld, j)
        ref, mag = oracle.mttkrp_csf3(T.pos_k, T.crd_k, T.pos_l, T.crd_l, T.vals, C, D)
        full_ref, full_mag = np.zeros((I, j)), np.zeros((I, j))
        rowsel = T.crd_i if T.crd_i is not None else np.arange(ns)
        full_ref[rowsel], full_mag[rowsel] = ref, mag
        A = torch.full((I, j), float("nan"), device="cuda")
        psk.psk_mttkrp_csf3(T.dims, dev(T.crd_i), dev(T.pos_k), dev(T.crd_k), dev(T.pos_l), dev(T.crd_l), dev(T.vals),
                            dev(C), dev(D), A, tile=tile)
        torch.cuda.synchronize()
        ok32(A.cpu().numpy(), full_ref, full_mag, "tensor %d" % case)
        ts, tf = psk.psk_partition_csf3(dev(T.pos_k), dev(T.pos_l), T.nnz, tile or 2048)
        ws, wf = oracle.partition_csf3(T.pos_k, T.pos_l, tile or 2048)
        assert (ts.cpu().numpy() == ws).all() and (tf.cpu().numpy() == wf).all()
