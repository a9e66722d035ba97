"""GPU parity at the small end and at the shapes of the paper's two synthetic studies.

Small end: with the default tile a matrix of at most 16384 entries is one tile of one workgroup (one launch, no
table, no carries).  Sweeps: the few-long-rows matrix of Section 8.5 (100 x 100000, 10000 per row) and the
exponentially skewed rows of Section 8.4 (65536 x 1M, 4M entries, lengths ~ base^rank, shuffled), each through
the position cut, the divided variant, the row split and the schedule the selector suggests."""
import sys

import numpy as np
import pytest

import oracle
import workloads as wl
from conftest import ADVERSARIAL_KINDS, adversarial_lengths

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_2001_00532_amd as psk  # noqa: E402


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check(got, ref, mag, what):
    ok, worst = oracle.within_tolerance(got, ref, mag)
    assert ok, "%s: worst |err|/bound = %.3g" % (what, worst)


@pytest.mark.parametrize("kind", ADVERSARIAL_KINDS)
def test_single_tile_path_structures(kind):
    rng = np.random.default_rng(31)
    for rows, cols in ((3, 2), (7, 5000), (1024, 1024), (5000, 300), (16000, 17)):
        A = wl.csr_from_lengths(adversarial_lengths(rng, rows, cols, kind), cols, seed=rows + cols)
        if A.nnz > 16384:
            continue
        x = wl.dense_uniform(cols, rows, wl.S_X)
        ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, x)
        say("single tile:", kind, rows, "x", cols, "nnz", A.nnz)
        y = torch.full((rows,), float("nan"), device="cuda")
        psk.psk_spmv_csr(rows, cols, A.nnz, dev(A.pos), dev(A.crd), dev(A.vals), dev(x), y)
        torch.cuda.synchronize()
        check(y.cpu().numpy(), ref, mag, "single tile %s %dx%d" % (kind, rows, cols))


@pytest.mark.parametrize("nnz", [1, 2, 63, 64, 65, 4095, 4096, 16383, 16384, 16385, 20000])
def test_single_tile_boundary_sizes(nnz):
    """Around the size limit of the one-launch path (16384 entries) and around wave and load granules; rows of
    mixed lengths, the last row takes what is left.  Unaligned crd/vals take the 4-byte load path."""
    rng = np.random.default_rng(nnz)
    L = []
    left = nnz
    while left > 0:
        take = int(min(left, rng.choice([0, 1, 2, 3, 31, 32, 33, 200, 5000])))
        L.append(take)
        left -= take
    cols = 6000
    A = wl.csr_from_lengths(np.array(L), cols, seed=nnz)
    assert A.nnz == nnz
    x = wl.dense_uniform(cols, nnz, wl.S_X)
    ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, x)
    for shift in (0, 1):            # shift 1: crd and vals start 4 bytes into their buffers
        crd = torch.zeros(nnz + shift, dtype=torch.int32, device="cuda")
        vals = torch.zeros(nnz + shift, device="cuda")
        crd[shift:] = dev(A.crd)
        vals[shift:] = dev(A.vals)
        y = torch.full((A.rows,), float("nan"), device="cuda")
        say("single tile boundary: nnz", nnz, "rows", A.rows, "shift", shift)
        psk.psk_spmv_csr(A.rows, cols, nnz, dev(A.pos), crd[shift:], vals[shift:], dev(x), y)
        torch.cuda.synchronize()
        check(y.cpu().numpy(), ref, mag, "nnz %d shift %d" % (nnz, shift))


def test_configuration_1_is_one_launch_and_needs_no_table():
    c = wl.config(1)
    A = c["A"]
    ws = psk.workspace(psk.PSK_OP_SPMV_CSR, A.rows, A.nnz)
    ws.fill_(0xFF)                          # a table, if it were read, would send the kernel out of bounds
    y = torch.full((A.rows,), float("nan"), device="cuda")
    psk.psk_spmv_csr(A.rows, A.cols, A.nnz, dev(A.pos), dev(A.crd), dev(A.vals), dev(c["x"]), y, ws=ws,
                     phases=psk.PSK_PHASE_MAIN)
    torch.cuda.synchronize()
    assert bool((ws == 0xFF).all()), "the one-launch path wrote to the workspace"
    ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, c["x"])
    check(y.cpu().numpy(), ref, mag, "configuration 1")


def sweep_matrices():
    A = wl.csr_uniform(100, 100_000, 10_000, wl.BASE_SEED + 7)
    yield "few long rows (100 x 100000, 10000 per row)", A, wl.dense_uniform(A.cols, wl.BASE_SEED + 7, wl.S_X)
    for base in (1.0, 1.0005, 1.00256, 1.005):
        Ls = wl.exponential_lengths(65536, 4_000_000, base, 1_000_000, wl.BASE_SEED + 8)
        A = wl.csr_from_lengths(Ls, 1_000_000, wl.BASE_SEED + 8)
        yield "exponential rows, base %g" % base, A, wl.dense_uniform(A.cols, wl.BASE_SEED + 8, wl.S_X)


def test_sweep_shapes_every_schedule():
    for name, A, x in sweep_matrices():
        ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, x, threads=8)
        pos, crd, vals, xd = dev(A.pos), dev(A.crd), dev(A.vals), dev(x)
        runs = [("position cut", lambda y: psk.psk_spmv_csr(A.rows, A.cols, A.nnz, pos, crd, vals, xd, y)),
                ("position cut, tile 256", lambda y: psk.psk_spmv_csr(A.rows, A.cols, A.nnz, pos, crd, vals, xd, y, tile=256)),
                ("divided", lambda y: psk.psk_spmv_csr_divide(A.rows, A.cols, A.nnz, pos, crd, vals, xd, y)),
                ("wave per row", lambda y: psk.psk_spmv_csr_rowsplit(A.rows, A.cols, A.nnz, pos, crd, vals, xd, y, variant=1)),
                ("thread per row", lambda y: psk.psk_spmv_csr_rowsplit(A.rows, A.cols, A.nnz, pos, crd, vals, xd, y, variant=0))]
        choice = psk.psk_suggest_schedule_csr(A.rows, A.nnz, pos)
        runs.append(("the selector's choice (%s)" % ("rows" if choice == psk.PSK_SCHEDULE_ROWS else "positions"),
                     runs[3][1] if choice == psk.PSK_SCHEDULE_ROWS else runs[0][1]))
        for what, fn in runs:
            say(name, "|", what, "| nnz", A.nnz, "longest row", int(np.diff(A.pos).max()))
            y = torch.full((A.rows,), float("nan"), device="cuda")
            fn(y)
            torch.cuda.synchronize()
            check(y.cpu().numpy(), ref, mag, "%s, %s" % (name, what))


def test_long_runs_of_empty_rows():
    """Ten million empty rows between two groups of stored rows (and more before the first and after the last): the
    tile that spans the run must not walk it.  Every path that walks rows is exercised: the CSR position cut with one
    and two column passes and a small tile, a second product on the same table (the run list must start empty again),
    and the row sums of the slab path."""
    import time

    rng = np.random.default_rng(77)
    rows, cols = 10_000_000 + 45_000, 120_000
    L = np.zeros(rows, dtype=np.int64)
    L[20_000:22_500] = rng.integers(1, 60, size=2_500)
    L[21_000] = 30_000                                      # a long row right before the run
    L[10_022_500:10_025_000] = rng.integers(0, 60, size=2_500)
    A = wl.csr_from_lengths(L, cols, seed=77)
    x = wl.dense_uniform(cols, 77, wl.S_X)
    ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, x, threads=8)
    pos, crd, vals, xd = dev(A.pos), dev(A.crd), dev(A.vals), dev(x)
    for tile, passes in ((0, 1), (256, 1), (0, 2), (4096, 1)):
        ws = psk.workspace(psk.PSK_OP_SPMV_CSR, rows, A.nnz, tile=tile)
        for rep, phases in enumerate((psk.PSK_PHASE_ALL, psk.PSK_PHASE_MAIN | psk.PSK_PHASE_FIXUP)):
            y = torch.full((rows,), float("nan"), device="cuda")
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            psk.psk_spmv_csr(rows, cols, A.nnz, pos, crd, vals, xd, y, tile=tile, col_passes=passes, phases=phases, ws=ws)
            torch.cuda.synchronize()
            say("empty-row run: tile", tile, "passes", passes, "product", rep, "nnz", A.nnz,
                "%.0f us" % ((time.perf_counter() - t0) * 1e6))
            check(y.cpu().numpy(), ref, mag, "empty-row run, tile %d passes %d product %d" % (tile, passes, rep))
    S = psk.psk_slab_build_csr(rows, cols, A.nnz, pos, crd, vals)
    for rep in range(2):
        y = torch.full((rows,), float("nan"), device="cuda")
        psk.psk_spmv_slab(S, xd, y)
        torch.cuda.synchronize()
        check(y.cpu().numpy(), ref, mag, "empty-row run, slab path, product %d" % rep)
