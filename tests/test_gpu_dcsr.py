"""GPU parity for SpMV on a DCSR (hypersparse) operand, position cut at the column level and at the
row level: every output row within |got - ref| <= 1e-5 * sum |a x| + 1e-30, rows that are not stored
exactly zero."""
import sys

import numpy as np
import pytest

import oracle
import workloads as wl
from conftest import ADVERSARIAL_KINDS, adversarial_lengths

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_2001_00532_amd as psk  # noqa: E402

REL, FLOOR = 1e-5, 1e-30
CUTS = [psk.PSK_CUT_POSITIONS, psk.PSK_CUT_ROWS]


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run(name, A, cut, tile, x=None, passes=1):
    x = wl.dense_uniform(A.cols, 9, wl.S_X) if x is None else x
    ref, mag = oracle.spmv_dcsr(A.rows, A.crd_i, A.pos, A.crd, A.vals, x)
    y = torch.full((A.rows,), float("nan"), device="cuda")
    say("dcsr", name, "cut", cut, "tile", tile, "passes", passes, "rows", A.rows, "stored", A.nstored, "nnz", A.nnz)
    psk.psk_spmv_dcsr(A.rows, A.cols, A.nnz, dev(A.crd_i), dev(A.pos), dev(A.crd), dev(A.vals), dev(x), y, cut=cut,
                      tile=tile, col_passes=passes)
    torch.cuda.synchronize()
    got = y.cpu().numpy()
    ok, worst = oracle.within_tolerance(got, ref, mag, REL, FLOOR)
    assert ok, "%s cut %d tile %d: worst |err|/bound = %.3g" % (name, cut, tile, worst)
    absent = np.ones(A.rows, dtype=bool)
    absent[A.crd_i] = False
    assert np.all(got[absent] == 0.0)
    return y


@pytest.mark.parametrize("cut", CUTS)
@pytest.mark.parametrize("tile", [0, 256, 1024, 4096])
def test_dcsr_structures(cut, tile):
    rng = np.random.default_rng(31)
    for kind in ADVERSARIAL_KINDS:
        L = adversarial_lengths(rng, 1501, 4001, kind)
        run(kind, wl.dcsr_from_lengths(200_000, L, 4001, seed=31), cut, tile)
    # every row stored: must agree with CSR
    L = rng.integers(0, 40, size=3000)
    run("all stored", wl.dcsr_from_lengths(3000, L, 500, seed=32), cut, tile)


@pytest.mark.parametrize("passes", [2, 3, 4])
def test_dcsr_column_passes(passes):
    rng = np.random.default_rng(34)
    for kind in ADVERSARIAL_KINDS:
        L = adversarial_lengths(rng, 1501, 4001, kind)
        for tile in (0, 256, 2048):
            run(kind, wl.dcsr_from_lengths(200_000, L, 4001, seed=34), psk.PSK_CUT_POSITIONS, tile, passes=passes)


@pytest.mark.parametrize("cut", CUTS)
def test_dcsr_edges(cut):
    run("nothing stored", wl.dcsr_from_lengths(1000, np.zeros(0, dtype=np.int64), 10, seed=1), cut, 0)
    run("stored but empty", wl.dcsr_from_lengths(1000, np.zeros(7, dtype=np.int64), 10, seed=1), cut, 0)
    run("one entry", wl.dcsr_from_lengths(1000, np.array([1]), 10, seed=1), cut, 0)
    run("one long row", wl.dcsr_from_lengths(10, np.array([9000]), 9000, seed=2), cut, 256)


def test_dcsr_position_cut_is_deterministic_and_matches_csr_kernel_when_all_rows_stored():
    L = np.random.default_rng(33).integers(0, 200, size=5000)
    A = wl.dcsr_from_lengths(5000, L, 3000, seed=33)
    x = wl.dense_uniform(3000, 9, wl.S_X)
    y1 = run("det", A, psk.PSK_CUT_POSITIONS, 1024, x)
    y2 = run("det", A, psk.PSK_CUT_POSITIONS, 1024, x)
    assert torch.equal(y1, y2)
    y3 = torch.empty(5000, device="cuda")
    psk.psk_spmv_csr(5000, 3000, A.nnz, dev(A.pos), dev(A.crd), dev(A.vals), dev(x), y3, tile=1024)
    torch.cuda.synchronize()
    assert torch.equal(y1, y3)


@pytest.mark.parametrize("cut", CUTS)
def test_dcsr_hypersparse_full_size(cut):
    """2^26 rows of which one million are stored, Zipf row lengths (alpha 1.8, <= 50 000): ~25 M nonzeros."""
    L = wl.zipf_lengths(1_000_000, 1.8, 1, 50_000, wl.BASE_SEED + 11)
    A = wl.dcsr_from_lengths(1 << 26, L, 1 << 21, seed=wl.BASE_SEED + 11)
    run("hypersparse", A, cut, 0)
    if cut == psk.PSK_CUT_POSITIONS:
        run("hypersparse", A, cut, 0, passes=2)
