"""GPU parity of the column-slab path with fp64 values (the value type of the paper's own schedules, appendix
"SPMV on a GPU"): the structure built on the device is compared bit for bit with the oracle's (slabs of 16 352
columns, 8-byte storage order of the values), the product with the extended-precision oracle of the CSR definition
within |got - ref| <= 1e-14 * sum_j |a_ij x_j| + 1e-300 (fp64 unit round-off 1.1e-16; a pair is summed through at
most 8 + 6 rounded additions, a row's pairs through fewer than 45 more, carries add one)."""
import ctypes
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
W64 = 16352


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def build_and_compare(A, vals, name):
    say("f64 slab build:", name, "rows", A.rows, "cols", A.cols, "nnz", A.nnz)
    S = psk.psk_slab_build_csr_f64(A.rows, A.cols, A.nnz, dev(A.pos), dev(A.crd), dev(vals) if A.nnz else None)
    O = oracle.slab_build(A.rows, A.cols, A.pos, A.crd, vals, W=W64, CH=512, f64=True)
    d = S.desc
    assert (d.nslots, d.npairs, d.nq, d.nslabs, d.nchunks) == (O.nslots, O.npairs, O.nq, O.nslabs, O.nslots // 512), name
    assert (d.slab_cols, d.chunk, d.value_bytes) == (W64, 512, 8)
    for arr in ("slab_chunk", "chunk_pair", "qpos", "qidx"):
        assert np.array_equal(S.array(arr).cpu().numpy(), getattr(O, arr)), "%s: %s differs" % (name, arr)
    assert np.array_equal(S.array("scol").cpu().numpy().view(np.uint16), O.scol), "%s: scol differs" % name
    assert S.array("svals").cpu().numpy().tobytes() == O.svals.tobytes(), "%s: svals differs" % name
    assert np.array_equal(S.array("qtile_row").cpu().numpy(), oracle.partition(O.qpos, d.tile)), "%s: row-list cut" % name
    return S


def product_ok(S, A, vals, x, name):
    y = torch.full((A.rows,), float("nan"), dtype=torch.float64, device="cuda")
    psk.psk_spmv_slab_f64(S, dev(x), y)
    torch.cuda.synchronize()
    ref, mag = oracle.spmv_csr_f64(A.pos, A.crd, vals, x, threads=8)
    ok, worst = oracle.within_tolerance(y.cpu().numpy(), ref, mag, REL, FLOOR)
    assert ok, "%s: worst |err|/bound = %.3g" % (name, worst)
    return y


def operands(A, seed):
    return wl.dense_uniform_f64(A.nnz, seed, wl.S_VALS), wl.dense_uniform_f64(A.cols, seed + 1, wl.S_X)


def test_slab_f64_configurations_scaled():
    for n, scale in [(1, 1.0), (2, 0.02), (3, 0.003), (4, 0.005)]:
        A = wl.config(n, scale)["A"]
        vals, x = operands(A, 40 + n)
        S = build_and_compare(A, vals, "config %d" % n)
        product_ok(S, A, vals, x, "config %d" % n)


@pytest.mark.parametrize("kind", ADVERSARIAL_KINDS)
def test_slab_f64_adversarial_structures(kind):
    rng = np.random.default_rng(9)
    for rows, cols in ((3001, 100_003), (700, W64), (513, W64 + 1), (40_000, 1_000_000)):
        A = wl.csr_from_lengths(adversarial_lengths(rng, rows, cols, kind), cols, seed=rows)
        vals, x = operands(A, rows)
        S = build_and_compare(A, vals, "%s %dx%d" % (kind, rows, cols))
        product_ok(S, A, vals, x, kind)


def test_slab_f64_few_long_rows_and_skewed_rows():
    """The shapes of the paper's load-balance (Section 8.4) and few-long-rows (Section 8.5) experiments."""
    A = wl.csr_uniform(100, 100_000, 10_000, wl.BASE_SEED + 7)
    vals, x = operands(A, 7)
    S = build_and_compare(A, vals, "100 x 100000, 10000 per row")
    product_ok(S, A, vals, x, "few long rows")
    Ls = wl.exponential_lengths(65536, 4_000_000, 1.00256, 1_000_000, wl.BASE_SEED + 8)
    A = wl.csr_from_lengths(Ls, 1_000_000, wl.BASE_SEED + 8)
    vals, x = operands(A, 8)
    S = build_and_compare(A, vals, "exponential row lengths")
    product_ok(S, A, vals, x, "exponential row lengths")


def test_slab_f64_empty_and_degenerate():
    pos = np.zeros(8, dtype=np.int32)
    S = psk.psk_slab_build_csr_f64(7, 50_000, 0, dev(pos), None, None)
    assert (S.desc.nslots, S.desc.npairs, S.desc.nq, S.desc.value_bytes) == (0, 0, 0, 8)
    y = torch.full((7,), float("nan"), dtype=torch.float64, device="cuda")
    psk.psk_spmv_slab_f64(S, None, y)
    torch.cuda.synchronize()
    assert bool((y == 0).all())
    for rows, cols, L in ((1, 1, [1]), (3, 40_000, [0, 40_000, 0]), (5, 1, [1, 0, 1, 1, 0])):
        A = wl.csr_from_lengths(np.array(L), cols, seed=3)
        vals, x = operands(A, 3)
        S = build_and_compare(A, vals, "degenerate %dx%d" % (rows, cols))
        product_ok(S, A, vals, x, "degenerate")


def test_slab_f64_is_deterministic_and_keeps_what_fp32_would_lose():
    A = wl.config(2, 0.02)["A"]
    vals, x = operands(A, 77)
    S = build_and_compare(A, vals, "power-law 2 %")
    ws = psk.psk_slab_spmv_workspace(S)
    y1 = torch.empty(A.rows, dtype=torch.float64, device="cuda")
    y2 = torch.empty(A.rows, dtype=torch.float64, device="cuda")
    psk.psk_spmv_slab_f64(S, dev(x), y1, ws=ws)
    ws.fill_(0xFF)
    psk.psk_spmv_slab_f64(S, dev(x), y2, ws=ws)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)
    # the values are not representable in fp32: a path that rounded them on the way would miss the bar by 1e7
    assert not np.array_equal(vals, vals.astype(np.float32).astype(np.float64))


def test_slab_f64_rejects_bad_arguments_and_mixed_types():
    L = psk.lib()
    one = ctypes.c_void_p(256)
    d = psk.psk_slab()
    assert L.psk_slab_mem_bytes_f64(4, 8192 * W64 + 1, 4) == 0                 # too many slabs
    assert L.psk_slab_build_csr_f64(4, 4, 4, None, one, one, one, 1 << 30, one, 1 << 30, ctypes.byref(d), None) == 1
    assert L.psk_slab_build_csr_f64(4, 4, 4, one, one, ctypes.c_void_p(260), one, 1 << 30, one, 1 << 30, ctypes.byref(d), None) == 7
    assert L.psk_slab_build_csr_f64(4, 4, 4, one, one, one, one, 16, one, 1 << 30, ctypes.byref(d), None) == 4
    # a structure of one value type is refused by the product of the other
    A = wl.csr_from_lengths(np.array([3, 0, 5]), 100, seed=1)
    S32 = psk.psk_slab_build_csr(A.rows, A.cols, A.nnz, dev(A.pos), dev(A.crd), dev(A.vals))
    S64 = psk.psk_slab_build_csr_f64(A.rows, A.cols, A.nnz, dev(A.pos), dev(A.crd), dev(A.vals.astype(np.float64)))
    ws = psk.psk_slab_spmv_workspace(S64)
    x64 = torch.zeros(100, dtype=torch.float64, device="cuda")
    y64 = torch.zeros(3, dtype=torch.float64, device="cuda")
    assert L.psk_spmv_slab_f64(ctypes.byref(S32.desc), x64.data_ptr(), y64.data_ptr(), 7, ws.data_ptr(), ws.numel(), None) == 2
    assert L.psk_spmv_slab(ctypes.byref(S64.desc), x64.data_ptr(), y64.data_ptr(), 7, ws.data_ptr(), ws.numel(), None) == 2


def test_slab_f64_many_slabs():
    """Ten million columns: 612 slabs, more than the staged scatter of the analysis step takes (the bucketing then
    goes through the one-wave-per-block kernel)."""
    rows, cols = 4000, 10_000_000
    L = np.random.default_rng(35).integers(0, 70, size=rows)
    L[9] = 5000
    A = wl.csr_from_lengths(L, cols, seed=35)
    vals, x = operands(A, 35)
    S = build_and_compare(A, vals, "%d x %d" % (rows, cols))
    assert S.desc.nslabs == -(-cols // W64)
    product_ok(S, A, vals, x, "many slabs")
