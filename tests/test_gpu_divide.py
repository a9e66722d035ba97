"""GPU parity for the divided (fixed number of parts, persistent workgroups, in-kernel search) CSR SpMV."""
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


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run(name, A, parts, x=None, offset=0):
    x = wl.dense_uniform(A.cols, 4, wl.S_X) if x is None else x
    ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, x, threads=8)
    if offset:
        crd_d = torch.empty(A.nnz + 4, dtype=torch.int32, device="cuda")[offset:offset + A.nnz]
        crd_d.copy_(dev(A.crd))
    else:
        crd_d = dev(A.crd)
    y = torch.full((A.rows,), float("nan"), device="cuda")
    say("divide", name, "parts", parts, "rows", A.rows, "nnz", A.nnz, "offset", offset)
    psk.psk_spmv_csr_divide(A.rows, A.cols, A.nnz, dev(A.pos), crd_d, dev(A.vals), dev(x), y, parts=parts)
    torch.cuda.synchronize()
    ok, worst = oracle.within_tolerance(y.cpu().numpy(), ref, mag, REL, FLOOR)
    assert ok, "%s parts %d: worst |err|/bound = %.3g" % (name, parts, worst)
    return y


@pytest.mark.parametrize("parts", [0, 1, 2, 3, 7, 64, 100000])
def test_divide_structures(parts):
    rng = np.random.default_rng(41)
    for kind in ADVERSARIAL_KINDS:
        run(kind, wl.csr_from_lengths(adversarial_lengths(rng, 20011, 30011, kind), 30011, seed=41), parts)
    run("powerlaw", wl.config(2, 0.02)["A"], parts)
    run("stencil", wl.config(3, 0.01)["A"], parts)


def test_divide_edges_and_alignment():
    run("empty", wl.csr_from_lengths(np.zeros(33, dtype=np.int64), 5, seed=1), 0)
    run("one entry", wl.csr_from_lengths(np.array([0, 0, 1, 0]), 3, seed=1), 0)
    run("exactly one chunk", wl.csr_from_lengths(np.full(256, 8), 64, seed=2), 0)
    run("exactly three chunks, three parts", wl.csr_from_lengths(np.full(768, 8), 64, seed=2), 3)
    run("one row over many parts", wl.csr_from_lengths(np.array([0, 50000, 0, 3]), 60000, seed=3), 5)
    A = wl.csr_from_lengths(adversarial_lengths(np.random.default_rng(42), 5000, 7000, "mixed"), 7000, seed=42)
    run("unaligned crd", A, 4, offset=1)


def test_divide_is_deterministic():
    A = wl.config(2, 0.03)["A"]
    y1 = run("det", A, 16)
    y2 = run("det", A, 16)
    assert torch.equal(y1, y2)


def test_divide_full_size_powerlaw_sampled():
    c = wl.config(2)
    A, x = c["A"], c["x"]
    y = torch.full((A.rows,), float("nan"), device="cuda")
    say("divide full size", A.rows, A.nnz)
    psk.psk_spmv_csr_divide(A.rows, A.cols, A.nnz, dev(A.pos), dev(A.crd), dev(A.vals), dev(x), y)
    torch.cuda.synchronize()
    assert not torch.isnan(y).any()
    lens = np.diff(A.pos)
    sel = np.unique(np.concatenate([np.random.default_rng(6).integers(0, A.rows, 20000), np.argsort(lens)[-50:]])).astype(np.int64)
    ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, x, sel=sel, threads=16)
    ok, worst = oracle.within_tolerance(y[torch.from_numpy(sel).cuda()].cpu().numpy(), ref, mag, REL, FLOOR)
    assert ok, "worst %.3g" % worst
