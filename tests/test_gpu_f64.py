"""GPU parity for the fp64 CSR SpMV: |got - ref| <= 1e-14 * sum |a x| + 1e-300 per row against the
extended-precision oracle (fp64 unit round-off 1.1e-16; a row segment is summed from < 45 rounded
operations, carries add one more)."""
import sys

import numpy as np
import pytest

import oracle
import workloads as wl
from conftest import ADVERSARIAL_KINDS, adversarial_lengths

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_2001_00532_amd as psk  # noqa: E402

REL, FLOOR = 1e-14, 1e-300


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run(name, A, tile, offset=0, passes=1):
    vals = wl.dense_uniform_f64(A.nnz, 5, wl.S_VALS)
    x = wl.dense_uniform_f64(A.cols, 6, wl.S_X)
    ref, mag = oracle.spmv_csr_f64(A.pos, A.crd, vals, x, threads=8)
    if offset:   # operands that are 8- but not 16-byte aligned: the 4/8-byte load path
        crd_d = torch.empty(A.nnz + 4, dtype=torch.int32, device="cuda")[offset:offset + A.nnz]
        crd_d.copy_(dev(A.crd))
        vals_d = torch.empty(A.nnz + 1, dtype=torch.float64, device="cuda")[1:]
        vals_d.copy_(dev(vals))
    else:
        crd_d, vals_d = dev(A.crd), dev(vals)
    y = torch.full((A.rows,), float("nan"), dtype=torch.float64, device="cuda")
    say("f64", name, "tile", tile, "offset", offset, "passes", passes, "rows", A.rows, "nnz", A.nnz)
    psk.psk_spmv_csr_f64(A.rows, A.cols, A.nnz, dev(A.pos), crd_d, vals_d, dev(x), y, tile=tile, col_passes=passes)
    torch.cuda.synchronize()
    ok, worst = oracle.within_tolerance(y.cpu().numpy(), ref, mag, REL, FLOOR)
    assert ok, "%s tile %d: worst |err|/bound = %.3g" % (name, tile, worst)
    return y


@pytest.mark.parametrize("tile", [0, 256, 512, 1024, 2048])
def test_f64_structures(tile):
    rng = np.random.default_rng(21)
    for kind in ADVERSARIAL_KINDS:
        A = wl.csr_from_lengths(adversarial_lengths(rng, 3001, 5003, kind), 5003, seed=21)
        run(kind, A, tile)
    run("powerlaw", wl.config(2, 0.01)["A"], tile)
    run("stencil", wl.config(3, 0.01)["A"], tile)


@pytest.mark.parametrize("passes", [2, 3, 4])
def test_f64_column_passes(passes):
    rng = np.random.default_rng(23)
    for kind in ADVERSARIAL_KINDS:
        A = wl.csr_from_lengths(adversarial_lengths(rng, 3001, 5003, kind), 5003, seed=23)
        for tile in (0, 256, 2048):
            run(kind, A, tile, passes=passes)
    run("powerlaw", wl.config(2, 0.01)["A"], 1024, passes=passes)
    run("unaligned", wl.config(2, 0.005)["A"], 512, offset=1, passes=passes)


def test_f64_unaligned_and_edges():
    rng = np.random.default_rng(22)
    A = wl.csr_from_lengths(adversarial_lengths(rng, 2000, 3000, "mixed"), 3000, seed=22)
    run("unaligned", A, 1024, offset=1)
    run("unaligned", A, 256, offset=3)
    run("one entry", wl.csr_from_lengths(np.array([0, 1, 0]), 4, seed=1), 0)
    run("empty", wl.csr_from_lengths(np.zeros(17, dtype=np.int64), 5, seed=1), 0)
    run("exact multiple of the tile", wl.csr_from_lengths(np.full(512, 8), 100, seed=2), 1024)


def test_f64_is_deterministic_and_uses_fp64():
    A = wl.config(2, 0.02)["A"]
    y1 = run("det", A, 0)
    y2 = run("det", A, 0)
    assert torch.equal(y1, y2)
    # an fp32 computation of the same product misses the fp64 bar by orders of magnitude
    vals = wl.dense_uniform_f64(A.nnz, 5, wl.S_VALS)
    x = wl.dense_uniform_f64(A.cols, 6, wl.S_X)
    ref, mag = oracle.spmv_csr_f64(A.pos, A.crd, vals, x, threads=8)
    y32 = torch.empty(A.rows, device="cuda")
    psk.psk_spmv_csr(A.rows, A.cols, A.nnz, dev(A.pos), dev(A.crd), dev(vals.astype(np.float32)),
                     dev(x.astype(np.float32)), y32)
    ok, _ = oracle.within_tolerance(y32.double().cpu().numpy(), ref, mag, REL, FLOOR)
    assert not ok


def test_f64_full_size_powerlaw_sampled():
    A = wl.config(2)["A"]
    vals = wl.dense_uniform_f64(A.nnz, 5, wl.S_VALS)
    x = wl.dense_uniform_f64(A.cols, 6, wl.S_X)
    y = torch.full((A.rows,), float("nan"), dtype=torch.float64, device="cuda")
    say("f64 full size", A.rows, A.nnz)
    psk.psk_spmv_csr_f64(A.rows, A.cols, A.nnz, dev(A.pos), dev(A.crd), dev(vals), dev(x), y, col_passes=3)
    torch.cuda.synchronize()
    assert not torch.isnan(y).any()
    lens = np.diff(A.pos)
    sel = np.unique(np.concatenate([np.random.default_rng(5).integers(0, A.rows, 20000), np.argsort(lens)[-50:]])).astype(np.int64)
    ref, mag = oracle.spmv_csr_f64(A.pos, A.crd, vals, x, sel=sel, threads=16)
    ok, worst = oracle.within_tolerance(y[torch.from_numpy(sel).cuda()].cpu().numpy(), ref, mag, REL, FLOOR)
    assert ok, "worst %.3g" % worst


def test_f64_long_runs_of_empty_rows():
    """Ten million empty rows between two groups of stored rows: the tile that spans the run lists it and the fix-up's
    extra workgroups clear it, as in the fp32 kernel; one and two column passes, a second product on the same table,
    and the row sums of the fp64 slab path."""
    import time

    rng = np.random.default_rng(78)
    rows, cols = 10_000_000 + 45_000, 120_000
    L = np.zeros(rows, dtype=np.int64)
    L[20_000:22_500] = rng.integers(1, 60, size=2_500)
    L[21_000] = 30_000
    L[10_022_500:10_025_000] = rng.integers(0, 60, size=2_500)
    A = wl.csr_from_lengths(L, cols, seed=78)
    vals = wl.dense_uniform_f64(A.nnz, 78, wl.S_VALS)
    x = wl.dense_uniform_f64(cols, 79, wl.S_X)
    ref, mag = oracle.spmv_csr_f64(A.pos, A.crd, vals, x, threads=8)
    pos, crd, vd, xd = dev(A.pos), dev(A.crd), dev(vals), dev(x)
    for tile, passes in ((0, 1), (256, 1), (0, 2)):
        ws = psk.workspace(psk.PSK_OP_SPMV_CSR_F64, rows, A.nnz, tile=tile)
        for rep, phases in enumerate((psk.PSK_PHASE_ALL, psk.PSK_PHASE_MAIN | psk.PSK_PHASE_FIXUP)):
            y = torch.full((rows,), float("nan"), dtype=torch.float64, device="cuda")
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            psk.psk_spmv_csr_f64(rows, cols, A.nnz, pos, crd, vd, xd, y, tile=tile, col_passes=passes, phases=phases, ws=ws)
            torch.cuda.synchronize()
            say("f64 empty-row run: tile", tile, "passes", passes, "product", rep, "%.0f us" % ((time.perf_counter() - t0) * 1e6))
            ok, worst = oracle.within_tolerance(y.cpu().numpy(), ref, mag, REL, FLOOR)
            assert ok, "f64 empty-row run, tile %d passes %d product %d: %.3g" % (tile, passes, rep, worst)
    S = psk.psk_slab_build_csr_f64(rows, cols, A.nnz, pos, crd, vd)
    for rep in range(2):
        y = torch.full((rows,), float("nan"), dtype=torch.float64, device="cuda")
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        psk.psk_spmv_slab_f64(S, xd, y)
        torch.cuda.synchronize()
        say("f64 empty-row run, slab path, product", rep, "%.0f us" % ((time.perf_counter() - t0) * 1e6))
        ok, worst = oracle.within_tolerance(y.cpu().numpy(), ref, mag, REL, FLOOR)
        assert ok, "f64 empty-row run, slab path, product %d: %.3g" % (rep, worst)
