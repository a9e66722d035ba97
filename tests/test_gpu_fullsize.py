"""Parity at the full sizes of the evaluated configurations, in the launch configuration bench.py
times (default tiles, all three phases).  SpMV outputs are compared in full (the oracle does 10^8
nonzeros in about a second); SpMM outputs on sampled rows the oracle computes one by one."""
import sys

import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_2001_00532_amd as psk  # noqa: E402

REL, FLOOR = 1e-5, 1e-30


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def sample_rows(rows, n, seed):
    rng = np.random.default_rng(seed)
    edge = np.concatenate([np.arange(min(64, rows)), np.arange(max(0, rows - 64), rows)])
    return np.unique(np.concatenate([edge, rng.integers(0, rows, size=n)])).astype(np.int64)


def check(got, ref, mag, what):
    ok, worst = oracle.within_tolerance(got, ref, mag, REL, FLOOR)
    assert ok, "%s: worst |err|/bound = %.3g" % (what, worst)
    say(what, "worst |err|/bound = %.3g" % worst)


@pytest.mark.parametrize("n", [2, 3])
def test_spmv_full_size(n):
    c = wl.config(n)
    A = c["A"]
    say("config", n, "rows", A.rows, "nnz", A.nnz)
    pos, crd, vals, x = dev(A.pos), dev(A.crd), dev(A.vals), dev(c["x"])
    tile = psk.psk_default_tile(psk.PSK_OP_SPMV_CSR)
    want = oracle.partition(A.pos, tile)
    for method in (1, 2):
        got = psk.psk_partition_csr(pos, A.nnz, tile, method=method).cpu().numpy()
        assert (got == want).all(), "partition method %d" % method
    y = torch.full((A.rows,), float("nan"), device="cuda")
    ws = psk.workspace(psk.PSK_OP_SPMV_CSR, A.rows, A.nnz)
    psk.psk_spmv_csr(A.rows, A.cols, A.nnz, pos, crd, vals, x, y, ws=ws)
    torch.cuda.synchronize()
    first = y.clone()
    ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, c["x"], threads=16)
    check(y.cpu().numpy(), ref, mag, "config %d full" % n)
    # deterministic: a second run gives the same bits
    y.fill_(float("nan"))
    psk.psk_spmv_csr(A.rows, A.cols, A.nnz, pos, crd, vals, x, y, ws=ws)
    torch.cuda.synchronize()
    assert torch.equal(first, y)
    passes = psk.psk_analyze_csr(A.rows, A.cols, A.nnz, pos, crd)
    if passes > 1:
        y.fill_(float("nan"))
        psk.psk_spmv_csr(A.rows, A.cols, A.nnz, pos, crd, vals, x, y, col_passes=passes, ws=ws)
        torch.cuda.synchronize()
        check(y.cpu().numpy(), ref, mag, "config %d full, %d column passes" % (n, passes))
    if n == 2:   # the wave-per-row baseline agrees within twice the bound (three-way check)
        psk.psk_spmv_csr_rowsplit(A.rows, A.cols, A.nnz, pos, crd, vals, x, y, variant=1)
        torch.cuda.synchronize()
        d = np.abs(y.cpu().numpy().astype(np.float64) - first.cpu().numpy().astype(np.float64))
        assert (d <= 2 * (REL * mag + FLOOR)).all()


def test_spmm_full_size():
    c = wl.config(4)
    A, B = c["A"], c["B"]
    say("config 4 rows", A.rows, "nnz", A.nnz)
    C = torch.full((A.rows, 128), float("nan"), device="cuda")
    psk.psk_spmm_csr(A.rows, A.cols, A.nnz, dev(A.pos), dev(A.crd), dev(A.vals), dev(B), C)
    torch.cuda.synchronize()
    assert not torch.isnan(C).any()
    sel = sample_rows(A.rows, 20000, 4)
    ref, mag = oracle.spmm_csr(A.pos, A.crd, A.vals, B, sel=sel, threads=16)
    check(C[torch.from_numpy(sel).cuda()].cpu().numpy(), ref, mag, "config 4 sampled rows")


def test_bcsr_full_size():
    c = wl.config(5)
    A = c["A"]
    say("config 5 block rows", A.rows, "blocks", A.nnz)
    pos, crd, vals = dev(A.pos), dev(A.crd), dev(A.vals)
    y = torch.full((A.rows * 4,), float("nan"), device="cuda")
    psk.psk_spmv_bcsr(A.rows, A.cols, A.nnz, 4, pos, crd, vals, dev(c["x"]), y)
    torch.cuda.synchronize()
    ref, mag = oracle.spmv_bcsr(A.pos, A.crd, A.vals, c["x"], 4, threads=16)
    check(y.cpu().numpy(), ref, mag, "config 5 spmv full")
    C = torch.full((A.rows * 4, 64), float("nan"), device="cuda")
    psk.psk_spmm_bcsr(A.rows, A.cols, A.nnz, 4, pos, crd, vals, dev(c["B"]), C)
    torch.cuda.synchronize()
    assert not torch.isnan(C).any()
    sel = sample_rows(A.rows, 10000, 5)
    ref, mag = oracle.spmm_bcsr(A.pos, A.crd, A.vals, c["B"], 4, sel=sel, threads=16)
    got = C.view(A.rows, 4, 64)[torch.from_numpy(sel).cuda()].reshape(-1, 64).cpu().numpy()
    check(got, ref, mag, "config 5 spmm sampled block rows")


def test_analyze_full_size():
    """Scattered columns over an x of 8 MB: two passes; the banded stencil (x of 16 MB): one."""
    A = wl.config(2)["A"]
    assert psk.psk_analyze_csr(A.rows, A.cols, A.nnz, dev(A.pos), dev(A.crd)) == 2
    A = wl.config(3)["A"]
    assert psk.psk_analyze_csr(A.rows, A.cols, A.nnz, dev(A.pos), dev(A.crd)) == 1
    # the rule only looks at cols and at sampled column distances: x of 16 MB -> 3, of 32 MB and more -> 4
    A = wl.csr_uniform(1_000_000, 4_000_000, 4, 5)
    assert psk.psk_analyze_csr(A.rows, A.cols, A.nnz, dev(A.pos), dev(A.crd)) == 3
    A = wl.csr_uniform(1_000_000, 20_000_000, 4, 5)
    assert psk.psk_analyze_csr(A.rows, A.cols, A.nnz, dev(A.pos), dev(A.crd)) == 4


def test_mttkrp_full_size():
    T = wl.csf3_powerlaw(500_000, 100_000, 100_000, 8, 1.8, 4096, wl.BASE_SEED + 9)
    I, K, L = T.dims
    say("mttkrp slices", T.nslices, "fibers", T.nfibers, "nnz", T.nnz)
    C = wl.dense_uniform(K * 64, 1, wl.S_B).reshape(K, 64)
    D = wl.dense_uniform(L * 64, 2, wl.S_B).reshape(L, 64)
    pos_k, pos_l = dev(T.pos_k), dev(T.pos_l)
    tile = psk.psk_default_tile(psk.PSK_OP_MTTKRP_CSF3)
    ts, tf = psk.psk_partition_csf3(pos_k, pos_l, T.nnz, tile)
    ws, wf = oracle.partition_csf3(T.pos_k, T.pos_l, tile)
    assert (ts.cpu().numpy() == ws).all() and (tf.cpu().numpy() == wf).all()
    A = torch.full((I, 64), float("nan"), device="cuda")
    psk.psk_mttkrp_csf3(T.dims, None, pos_k, dev(T.crd_k), pos_l, dev(T.crd_l), dev(T.vals), dev(C), dev(D), A)
    torch.cuda.synchronize()
    assert not torch.isnan(A).any()
    sel = sample_rows(T.nslices, 20000, 9)
    ref, mag = oracle.mttkrp_csf3(T.pos_k, T.crd_k, T.pos_l, T.crd_l, T.vals, C, D, sel=sel, threads=16)
    check(A[torch.from_numpy(sel).cuda()].cpu().numpy(), ref, mag, "mttkrp sampled slices")


def test_slab_path_full_size_power_law():
    """The launch configuration bench.py times by default: the power-law matrix at full size through the slab path.
    The structure is compared in full with the oracle's (bit for bit), the product in full with the CSR definition."""
    c = wl.config(2)
    A = c["A"]
    pos, crd, vals, x = dev(A.pos), dev(A.crd), dev(A.vals), dev(c["x"])
    say("slab path, full size: rows", A.rows, "nnz", A.nnz)
    S = psk.psk_slab_build_csr(A.rows, A.cols, A.nnz, pos, crd, vals)
    O = oracle.slab_build(A.rows, A.cols, A.pos, A.crd, A.vals)
    d = S.desc
    assert (d.nslots, d.npairs, d.nq, d.nslabs) == (O.nslots, O.npairs, O.nq, O.nslabs)
    for arr in ("slab_chunk", "chunk_pair", "qpos", "qidx"):
        assert np.array_equal(S.array(arr).cpu().numpy(), getattr(O, arr)), arr
    assert np.array_equal(S.array("scol").cpu().numpy().view(np.uint16), O.scol)
    assert np.array_equal(S.array("svals").cpu().numpy().view(np.uint32), O.svals.view(np.uint32))
    assert np.array_equal(S.array("qtile_row").cpu().numpy(), oracle.partition(O.qpos, d.tile))
    ws = psk.psk_slab_spmv_workspace(S)
    y = torch.full((A.rows,), float("nan"), device="cuda")
    psk.psk_spmv_slab(S, x, y, ws=ws)
    torch.cuda.synchronize()
    first = y.clone()
    ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, c["x"], threads=16)
    check(y.cpu().numpy(), ref, mag, "slab path, configuration 2 in full")
    y.fill_(float("nan"))
    psk.psk_spmv_slab(S, x, y, ws=ws)
    torch.cuda.synchronize()
    assert torch.equal(first, y), "the slab product is not deterministic"


def test_slab_path_full_size_power_law_f64():
    """The configuration `bench.py --workload powerlaw --f64` times: the power-law matrix at full size with fp64
    values through the slab path; structure bit for bit against the oracle's, product in full against the
    extended-precision CSR definition within 1e-14 * sum |a x| + 1e-300."""
    A = wl.config(2)["A"]
    vals = wl.dense_uniform_f64(A.nnz, wl.BASE_SEED + 2, wl.S_VALS)
    xh = wl.dense_uniform_f64(A.cols, wl.BASE_SEED + 2, wl.S_X)
    pos, crd = dev(A.pos), dev(A.crd)
    say("fp64 slab path, full size: rows", A.rows, "nnz", A.nnz)
    S = psk.psk_slab_build_csr_f64(A.rows, A.cols, A.nnz, pos, crd, dev(vals))
    d = S.desc
    O = oracle.slab_build(A.rows, A.cols, A.pos, A.crd, vals, W=int(d.slab_cols), CH=512, f64=True)
    assert int(d.slab_cols) == 16352 and int(d.value_bytes) == 8
    assert (d.nslots, d.npairs, d.nq, d.nslabs) == (O.nslots, O.npairs, O.nq, O.nslabs)
    for arr in ("slab_chunk", "chunk_pair", "qpos", "qidx"):
        assert np.array_equal(S.array(arr).cpu().numpy(), getattr(O, arr)), arr
    assert np.array_equal(S.array("scol").cpu().numpy().view(np.uint16), O.scol)
    assert S.array("svals").cpu().numpy().tobytes() == O.svals.tobytes()
    ws = psk.psk_slab_spmv_workspace(S)
    y = torch.full((A.rows,), float("nan"), dtype=torch.float64, device="cuda")
    psk.psk_spmv_slab_f64(S, dev(xh), y, ws=ws)
    torch.cuda.synchronize()
    ref, mag = oracle.spmv_csr_f64(A.pos, A.crd, vals, xh, threads=16)
    ok, worst = oracle.within_tolerance(y.cpu().numpy(), ref, mag, 1e-14, 1e-300)
    assert ok, "fp64 slab path, configuration 2 in full: worst |err|/bound = %.3g" % worst
