"""GPU parity of the column-slab path: the structure built on the device is compared bit for bit with
the oracle's (integer and byte work), the product over it with the oracle's CSR definition within the
fp32 bar |got - ref| <= 1e-5 * sum_j |a_ij x_j| + 1e-30."""
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


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def build_and_compare(A, name):
    say("slab build:", name, "rows", A.rows, "cols", A.cols, "nnz", A.nnz)
    S = psk.psk_slab_build_csr(A.rows, A.cols, A.nnz, dev(A.pos), dev(A.crd), dev(A.vals))
    O = oracle.slab_build(A.rows, A.cols, A.pos, A.crd, A.vals)
    d = S.desc
    assert (d.nslots, d.npairs, d.nq, d.nslabs, d.nchunks) == (O.nslots, O.npairs, O.nq, O.nslabs, O.nslots // 512), name
    assert (d.slab_cols, d.chunk) == (O.W, O.CH)
    for arr in ("slab_chunk", "chunk_pair", "qpos", "qidx"):
        assert np.array_equal(S.array(arr).cpu().numpy(), getattr(O, arr)), "%s: %s differs" % (name, arr)
    assert np.array_equal(S.array("scol").cpu().numpy().view(np.uint16), O.scol), "%s: scol differs" % name
    assert np.array_equal(S.array("svals").cpu().numpy().view(np.uint32), O.svals.view(np.uint32)), "%s: svals differs" % name
    assert np.array_equal(S.array("qtile_row").cpu().numpy(), oracle.partition(O.qpos, d.tile)), "%s: row-list cut" % name
    return S


def product_ok(S, A, x, name):
    y = torch.full((A.rows,), float("nan"), device="cuda")
    psk.psk_spmv_slab(S, dev(x), y)
    torch.cuda.synchronize()
    ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, x, threads=8)
    ok, worst = oracle.within_tolerance(y.cpu().numpy(), ref, mag)
    assert ok, "%s: worst |err|/bound = %.3g" % (name, worst)
    return y


def test_slab_configurations_scaled():
    for n, scale in [(1, 1.0), (2, 0.02), (3, 0.003), (4, 0.005)]:
        c = wl.config(n, scale)
        A = c["A"]
        x = c["x"] if "x" in c else wl.dense_uniform(A.cols, 5, wl.S_X)
        S = build_and_compare(A, "config %d" % n)
        product_ok(S, A, x, "config %d" % n)


@pytest.mark.parametrize("kind", ADVERSARIAL_KINDS)
def test_slab_adversarial_structures(kind):
    rng = np.random.default_rng(8)
    for rows, cols in ((3001, 100_003), (700, 32736), (513, 32737), (40_000, 1_000_000)):
        A = wl.csr_from_lengths(adversarial_lengths(rng, rows, cols, kind), cols, seed=rows)
        S = build_and_compare(A, "%s %dx%d" % (kind, rows, cols))
        product_ok(S, A, wl.dense_uniform(cols, rows, wl.S_X), kind)


def test_slab_few_long_rows_and_skewed_rows():
    """The shapes of the paper's load-balance (Section 8.4) and few-long-rows (Section 8.5) experiments."""
    A = wl.csr_uniform(100, 100_000, 10_000, wl.BASE_SEED + 7)
    S = build_and_compare(A, "100 x 100000, 10000 per row")
    product_ok(S, A, wl.dense_uniform(A.cols, 7, wl.S_X), "few long rows")
    Ls = wl.exponential_lengths(65536, 4_000_000, 1.00256, 1_000_000, wl.BASE_SEED + 8)
    A = wl.csr_from_lengths(Ls, 1_000_000, wl.BASE_SEED + 8)
    S = build_and_compare(A, "exponential row lengths")
    product_ok(S, A, wl.dense_uniform(A.cols, 8, wl.S_X), "exponential row lengths")


def test_slab_unsorted_and_repeated_columns():
    rng = np.random.default_rng(21)
    rows, cols = 2000, 70_000
    L = rng.integers(0, 60, size=rows)
    pos = np.zeros(rows + 1, dtype=np.int32)
    pos[1:] = np.cumsum(L)
    crd = rng.integers(0, cols, size=int(pos[-1])).astype(np.int32)        # unsorted, duplicates allowed
    vals = wl.dense_uniform(int(pos[-1]), 21, wl.S_VALS)

    class M:
        pass
    A = M()
    A.rows, A.cols, A.nnz, A.pos, A.crd, A.vals = rows, cols, int(pos[-1]), pos, crd, vals
    S = build_and_compare(A, "unsorted columns")
    product_ok(S, A, wl.dense_uniform(cols, 22, wl.S_X), "unsorted columns")


def test_slab_empty_and_degenerate():
    # no entries at all
    pos = np.zeros(8, dtype=np.int32)
    S = psk.psk_slab_build_csr(7, 50_000, 0, dev(pos), None, None)
    assert (S.desc.nslots, S.desc.npairs, S.desc.nq) == (0, 0, 0)
    y = torch.full((7,), float("nan"), device="cuda")
    psk.psk_spmv_slab(S, None, y)
    torch.cuda.synchronize()
    assert bool((y == 0).all())
    # one entry; one full row; a single column
    for rows, cols, L in ((1, 1, [1]), (3, 40_000, [0, 40_000, 0]), (5, 1, [1, 0, 1, 1, 0])):
        A = wl.csr_from_lengths(np.array(L), cols, seed=3)
        S = build_and_compare(A, "degenerate %dx%d" % (rows, cols))
        product_ok(S, A, wl.dense_uniform(cols, 3, wl.S_X), "degenerate")


def test_slab_is_deterministic_and_reusable():
    c = wl.config(2, 0.02)
    A = c["A"]
    S = build_and_compare(A, "power-law 2 %")
    ws = psk.psk_slab_spmv_workspace(S)
    y1 = torch.empty(A.rows, device="cuda")
    y2 = torch.empty(A.rows, device="cuda")
    psk.psk_spmv_slab(S, dev(c["x"]), y1, ws=ws)
    x2 = wl.dense_uniform(A.cols, 99, wl.S_X)
    product_ok(S, A, x2, "second vector")
    ws.fill_(0xFF)
    psk.psk_spmv_slab(S, dev(c["x"]), y2, ws=ws)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)


def test_slab_special_values_propagate():
    """IEEE propagation: an infinite or NaN entry of x reaches exactly the rows that use its column; pad slots
    (value 0 in column 0 of a slab) never leak into a row."""
    A = wl.csr_from_lengths(np.random.default_rng(5).integers(0, 30, size=4000), 90_000, seed=5)
    x = wl.dense_uniform(A.cols, 6, wl.S_X)
    x[0] = np.inf                      # column 0 of slab 0: where slab 0's pad slots point
    x[32736] = np.nan                  # column 0 of slab 1
    S = psk.psk_slab_build_csr(A.rows, A.cols, A.nnz, dev(A.pos), dev(A.crd), dev(A.vals))
    y = torch.empty(A.rows, device="cuda")
    psk.psk_spmv_slab(S, dev(x), y)
    torch.cuda.synchronize()
    y = y.cpu().numpy()
    rows_of = np.repeat(np.arange(A.rows), np.diff(A.pos))
    hit = np.zeros(A.rows, dtype=bool)
    hit[rows_of[(A.crd == 0) | (A.crd == 32736)]] = True
    assert np.isfinite(y[~hit]).all() and not np.isfinite(y[hit]).any()


def test_slab_rejects_bad_arguments():
    L = psk.lib()
    one = ctypes.c_void_p(256)
    d = psk.psk_slab()
    assert L.psk_slab_mem_bytes(4, 8192 * 32736 + 1, 4) == 0                 # too many slabs
    assert L.psk_slab_build_csr(4, 4, 4, None, one, one, one, 1 << 30, one, 1 << 30, ctypes.byref(d), None) == 1
    assert L.psk_slab_build_csr(4, 4, 4, one, one, one, one, 16, one, 1 << 30, ctypes.byref(d), None) == 4
    assert L.psk_slab_build_csr(-1, 4, 4, one, one, one, one, 1 << 30, one, 1 << 30, ctypes.byref(d), None) == 2
    assert L.psk_spmv_slab(None, one, one, 7, one, 1 << 30, None) == 1


def test_slab_unaligned_vector_split_phases_own_buffers_and_stream():
    """x that is 4-byte but not 16-byte aligned (the window is then loaded element by element), the two phases of a
    product issued by separate calls, caller-provided structure memory and build workspace, and a stream of the
    caller's; the same for fp64 with an x that is 8- but not 16-byte aligned."""
    A = wl.config(2, 0.01)["A"]
    xh = wl.dense_uniform(A.cols, 61, wl.S_X)
    pos, crd, vals = dev(A.pos), dev(A.crd), dev(A.vals)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    mem = torch.empty(psk.psk_slab_mem_bytes(A.rows, A.cols, A.nnz), dtype=torch.uint8, device="cuda")
    bws = torch.empty(psk.psk_slab_build_workspace_bytes(A.rows, A.cols, A.nnz), dtype=torch.uint8, device="cuda")
    mem.fill_(0xA5)
    bws.fill_(0x5A)
    xbuf = torch.zeros(A.cols + 4, device="cuda")
    x = xbuf[1:1 + A.cols]
    x.copy_(dev(xh))
    assert x.data_ptr() % 16 == 4
    y = torch.full((A.rows,), float("nan"), device="cuda")
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        S = psk.psk_slab_build_csr(A.rows, A.cols, A.nnz, pos, crd, vals, mem=mem, ws=bws, stream=side)
        ws = psk.psk_slab_spmv_workspace(S, stream=side)
        psk.psk_spmv_slab(S, x, y, phases=psk.PSK_PHASE_MAIN, ws=ws, stream=side)
        psk.psk_spmv_slab(S, x, y, phases=psk.PSK_PHASE_FIXUP, ws=ws, stream=side)
    side.synchronize()
    O = oracle.slab_build(A.rows, A.cols, A.pos, A.crd, A.vals)
    assert np.array_equal(S.array("qidx").cpu().numpy(), O.qidx) and np.array_equal(S.array("scol").cpu().numpy().view(np.uint16), O.scol)
    ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, xh, threads=8)
    ok, worst = oracle.within_tolerance(y.cpu().numpy(), ref, mag)
    assert ok, "unaligned x, split phases: worst |err|/bound = %.3g" % worst
    # fp64
    v64 = wl.dense_uniform_f64(A.nnz, 62, wl.S_VALS)
    x64h = wl.dense_uniform_f64(A.cols, 63, wl.S_X)
    xbuf64 = torch.zeros(A.cols + 2, dtype=torch.float64, device="cuda")
    x64 = xbuf64[1:1 + A.cols]
    x64.copy_(dev(x64h))
    assert x64.data_ptr() % 16 == 8
    y64 = torch.full((A.rows,), float("nan"), dtype=torch.float64, device="cuda")
    S64 = psk.psk_slab_build_csr_f64(A.rows, A.cols, A.nnz, pos, crd, dev(v64))
    ws64 = psk.psk_slab_spmv_workspace(S64)
    psk.psk_spmv_slab_f64(S64, x64, y64, phases=psk.PSK_PHASE_MAIN, ws=ws64)
    psk.psk_spmv_slab_f64(S64, x64, y64, phases=psk.PSK_PHASE_FIXUP, ws=ws64)
    torch.cuda.synchronize()
    ref, mag = oracle.spmv_csr_f64(A.pos, A.crd, v64, x64h, threads=8)
    ok, worst = oracle.within_tolerance(y64.cpu().numpy(), ref, mag, 1e-14, 1e-300)
    assert ok, "fp64, unaligned x, split phases: worst |err|/bound = %.3g" % worst


def test_slab_many_slabs():
    """A hundred million columns: 3 055 slabs (the bucketing kernels keep one counter per slab in LDS and rank lanes with one
    ballot per bit of the slab number: 12 bits here), most of them empty, a few entries each in the others."""
    rows, cols = 5000, 100_000_000
    rng = np.random.default_rng(33)
    L = rng.integers(0, 80, size=rows)
    L[17] = 3000
    A = wl.csr_from_lengths(L, cols, seed=33)
    S = build_and_compare(A, "%d x %d" % (rows, cols))
    assert S.desc.nslabs == -(-cols // 32736)
    x = wl.dense_uniform(cols, 34, wl.S_X)
    product_ok(S, A, x, "many slabs")
