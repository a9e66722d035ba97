"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bars: the tile->row table is bit-exact; fp32 results satisfy
|got - ref| <= 1e-5 * sum_j |a_ij x_j| + 1e-30 per output element.
"""
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


class DevCSR:
    def __init__(self, A):
        self.A = A
        self.pos, self.crd, self.vals = dev(A.pos), dev(A.crd), dev(A.vals)


def check(got, ref, mag, what):
    ok, worst = oracle.within_tolerance(got, ref, mag, REL, FLOOR)
    assert ok, "%s: worst |err|/bound = %.3g" % (what, worst)
    return worst


def run_spmv(D, x, tile=0, **kw):
    A = D.A
    y = torch.full((A.rows,), float("nan"), device="cuda")
    psk.psk_spmv_csr(A.rows, A.cols, A.nnz, D.pos, D.crd, D.vals, x, y, tile=tile, **kw)
    torch.cuda.synchronize()
    return y.cpu().numpy()


# ------------------------------------------------------------------ partition (bit exact)
@pytest.mark.parametrize("tile", [1, 3, 64, 256, 1024, 2048, 4096])
def test_partition_bit_exact_configs(tile):
    for n, scale in [(1, 1.0), (2, 0.01), (3, 0.003), (4, 0.005), (5, 0.01)]:
        A = wl.config(n, scale)["A"]
        say("partition config", n, "tile", tile, "nnz", A.nnz)
        want = oracle.partition(A.pos, tile)
        for method in (0, 1, 2):
            got = psk.psk_partition_csr(dev(A.pos), A.nnz, tile, method=method).cpu().numpy()
            assert (got == want).all(), "method %d" % method


@pytest.mark.parametrize("kind", ADVERSARIAL_KINDS)
def test_partition_bit_exact_adversarial(kind):
    rng = np.random.default_rng(1)
    L = adversarial_lengths(rng, 3001, 6000, kind)
    pos = np.concatenate([[0], np.cumsum(L)]).astype(np.int32)
    for tile in (1, 5, 256, 1000, 2048):
        say("partition", kind, "tile", tile)
        want = oracle.partition(pos, tile)
        for method in (0, 1, 2):
            got = psk.psk_partition_csr(dev(pos), int(pos[-1]), tile, method=method).cpu().numpy()
            assert (got == want).all(), "method %d" % method


# ------------------------------------------------------------------ CSR SpMV
SPMV_TILES = [256, 512, 1024, 2048, 4096]


@pytest.mark.parametrize("tile", [0] + SPMV_TILES)
def test_spmv_configs_scaled(tile):
    for n, scale in [(1, 1.0), (2, 0.02), (3, 0.01)]:
        c = wl.config(n, scale)
        A = c["A"]
        say("spmv config", n, "tile", tile, "rows", A.rows, "nnz", A.nnz)
        ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, c["x"], threads=8)
        got = run_spmv(DevCSR(A), dev(c["x"]), tile)
        check(got, ref, mag, "spmv config %d tile %d" % (n, tile))


@pytest.mark.parametrize("kind", ADVERSARIAL_KINDS)
def test_spmv_adversarial(kind):
    rng = np.random.default_rng(2)
    rows, cols = 5003, 7001
    A = wl.csr_from_lengths(adversarial_lengths(rng, rows, cols, kind), cols, seed=77)
    x = wl.dense_uniform(cols, 77, wl.S_X)
    ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, x)
    D, xd = DevCSR(A), dev(x)
    for tile in SPMV_TILES:
        say("spmv", kind, "tile", tile, "nnz", A.nnz)
        got = run_spmv(D, xd, tile)
        check(got, ref, mag, "spmv %s tile %d" % (kind, tile))
        if kind == "all_empty":
            assert (got == 0).all() and not np.signbit(got).any()


def test_spmv_tile_boundaries_and_tails():
    """nnz an exact multiple of the tile, nnz < tile, one row, one column, rows ending exactly on a
    tile boundary followed by empty rows."""
    cases = {
        "exact_multiple": ([256] * 8, 4096),
        "less_than_tile": ([3, 0, 5], 16),
        "one_row": ([5000], 6000),
        "one_col": ([1, 0, 1, 1, 0], 1),
        "boundary_then_empty": ([256, 0, 0, 0, 256, 0, 512, 0, 0, 1], 1024),
        "single_nnz": ([0, 0, 1, 0], 7),
    }
    for name, (L, cols) in cases.items():
        A = wl.csr_from_lengths(L, cols, seed=5)
        x = wl.dense_uniform(cols, 5, wl.S_X)
        ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, x)
        D, xd = DevCSR(A), dev(x)
        for tile in SPMV_TILES:
            say("spmv edge", name, "tile", tile)
            check(run_spmv(D, xd, tile), ref, mag, "%s tile %d" % (name, tile))


def test_spmv_unsorted_duplicate_columns_and_unaligned_views():
    rng = np.random.default_rng(9)
    rows, cols = 999, 500
    L = rng.integers(0, 40, size=rows)
    pos = np.concatenate([[0], np.cumsum(L)]).astype(np.int32)
    crd = rng.integers(0, cols, size=int(pos[-1])).astype(np.int32)     # unsorted, duplicates likely
    vals = wl.dense_uniform(int(pos[-1]), 9, wl.S_VALS)
    x = wl.dense_uniform(cols, 9, wl.S_X)
    ref, mag = oracle.spmv_csr(pos, crd, vals, x)
    y = torch.empty(rows, device="cuda")
    # crd/vals at a 4-byte (not 16-byte) aligned address: the kernel must fall back to scalar loads
    crd_d = torch.empty(crd.size + 1, dtype=torch.int32, device="cuda")
    vals_d = torch.empty(vals.size + 1, dtype=torch.float32, device="cuda")
    crd_d[1:] = dev(crd)
    vals_d[1:] = dev(vals)
    for tile in SPMV_TILES:
        say("spmv unaligned tile", tile)
        psk.psk_spmv_csr(rows, cols, int(pos[-1]), dev(pos), crd_d[1:], vals_d[1:], dev(x), y, tile=tile)
        torch.cuda.synchronize()
        check(y.cpu().numpy(), ref, mag, "unaligned tile %d" % tile)


def test_spmv_deterministic_and_partition_reuse():
    c = wl.config(2, 0.02)
    A = c["A"]
    D, xd = DevCSR(A), dev(c["x"])
    ws = psk.workspace(psk.PSK_OP_SPMV_CSR, A.rows, A.nnz)
    y1 = torch.empty(A.rows, device="cuda")
    y2 = torch.empty(A.rows, device="cuda")
    psk.psk_spmv_csr(A.rows, A.cols, A.nnz, D.pos, D.crd, D.vals, xd, y1, ws=ws)
    # second call reuses the tile->row table that the first left in the workspace
    psk.psk_spmv_csr(A.rows, A.cols, A.nnz, D.pos, D.crd, D.vals, xd, y2, ws=ws,
                     phases=psk.PSK_PHASE_MAIN | psk.PSK_PHASE_FIXUP)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)
    ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, c["x"], threads=8)
    check(y2.cpu().numpy(), ref, mag, "reuse")


@pytest.mark.parametrize("variant", [0, 1])
def test_spmv_rowsplit_baselines(variant):
    for n, scale in [(1, 1.0), (3, 0.01), (2, 0.005)]:
        c = wl.config(n, scale)
        A = c["A"]
        say("rowsplit variant", variant, "config", n)
        D = DevCSR(A)
        y = torch.full((A.rows,), float("nan"), device="cuda")
        psk.psk_spmv_csr_rowsplit(A.rows, A.cols, A.nnz, D.pos, D.crd, D.vals, dev(c["x"]), y, variant=variant)
        torch.cuda.synchronize()
        ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, c["x"])
        check(y.cpu().numpy(), ref, mag, "rowsplit %d config %d" % (variant, n))


# ------------------------------------------------------------------ CSR SpMM
def run_spmm(D, B, tile=0, ldc=None):
    A = D.A
    k = B.shape[1]
    Cfull = torch.full((A.rows, ldc or k), float("nan"), device="cuda")
    C = Cfull[:, :k]
    psk.psk_spmm_csr(A.rows, A.cols, A.nnz, D.pos, D.crd, D.vals, B, C, tile=tile)
    torch.cuda.synchronize()
    return C.cpu().numpy()


@pytest.mark.parametrize("tile", [0, 256, 512, 1024, 2048])
def test_spmm_config4_scaled(tile):
    c = wl.config(4, 0.01)
    A, B = c["A"], c["B"]
    say("spmm config 4 tile", tile, "rows", A.rows)
    ref, mag = oracle.spmm_csr(A.pos, A.crd, A.vals, B, threads=8)
    check(run_spmm(DevCSR(A), dev(B), tile), ref, mag, "spmm tile %d" % tile)


@pytest.mark.parametrize("k", [1, 8, 9, 12, 16, 17, 24, 32, 33, 64, 100, 128, 130, 256, 300])
def test_spmm_any_k_and_strides(k):
    rng = np.random.default_rng(k)
    rows, cols = 1501, 1203
    A = wl.csr_from_lengths(adversarial_lengths(rng, rows, cols, "mixed"), cols, seed=31)
    Bh = wl.dense_uniform(cols * (k + 3), 31, wl.S_B).reshape(cols, k + 3)
    ref, mag = oracle.spmm_csr(A.pos, A.crd, A.vals, Bh[:, :k])
    D = DevCSR(A)
    say("spmm k", k, "contiguous")
    check(run_spmm(D, dev(Bh[:, :k]), 512), ref, mag, "spmm k=%d" % k)
    say("spmm k", k, "strided B and C")
    check(run_spmm(D, dev(Bh)[:, :k], 1024, ldc=k + 5), ref, mag, "spmm k=%d strided" % k)


@pytest.mark.parametrize("kind", ADVERSARIAL_KINDS)
def test_spmm_adversarial(kind):
    rng = np.random.default_rng(4)
    rows, cols, k = 2003, 3001, 128
    A = wl.csr_from_lengths(adversarial_lengths(rng, rows, cols, kind), cols, seed=41)
    B = wl.dense_uniform(cols * k, 41, wl.S_B).reshape(cols, k)
    ref, mag = oracle.spmm_csr(A.pos, A.crd, A.vals, B, threads=8)
    D, Bd = DevCSR(A), dev(B)
    for tile in (256, 1024, 2048):
        say("spmm", kind, "tile", tile)
        got = run_spmm(D, Bd, tile)
        check(got, ref, mag, "spmm %s tile %d" % (kind, tile))


def test_spmm_rowsplit_baseline():
    c = wl.config(4, 0.005)
    A, B = c["A"], c["B"]
    D = DevCSR(A)
    C = torch.full((A.rows, 128), float("nan"), device="cuda")
    psk.psk_spmm_csr_rowsplit(A.rows, A.cols, A.nnz, D.pos, D.crd, D.vals, dev(B), C)
    torch.cuda.synchronize()
    ref, mag = oracle.spmm_csr(A.pos, A.crd, A.vals, B, threads=8)
    check(C.cpu().numpy(), ref, mag, "spmm rowsplit")


# ------------------------------------------------------------------ BCSR
BCSR_TILES = [0, 64, 128, 256, 512]


def bcsr_cases():
    rng = np.random.default_rng(6)
    yield "config5", wl.config(5, 0.02)["A"]
    for kind in ADVERSARIAL_KINDS:
        yield kind, wl.csr_from_lengths(adversarial_lengths(rng, 1203, 1501, kind), 1501, seed=51, bs=4)


def test_bcsr_spmv():
    for name, A in bcsr_cases():
        x = wl.dense_uniform(A.cols * 4, 51, wl.S_X)
        ref, mag = oracle.spmv_bcsr(A.pos, A.crd, A.vals, x, 4, threads=8)
        D, xd = DevCSR(A), dev(x)
        for tile in BCSR_TILES:
            say("bcsr spmv", name, "tile", tile, "blocks", A.nnz)
            y = torch.full((A.rows * 4,), float("nan"), device="cuda")
            psk.psk_spmv_bcsr(A.rows, A.cols, A.nnz, 4, D.pos, D.crd, D.vals, xd, y, tile=tile)
            torch.cuda.synchronize()
            check(y.cpu().numpy(), ref, mag, "bcsr spmv %s tile %d" % (name, tile))


@pytest.mark.parametrize("k", [64, 128, 40])
def test_bcsr_spmm(k):
    for name, A in bcsr_cases():
        B = wl.dense_uniform(A.cols * 4 * k, 52, wl.S_B).reshape(A.cols * 4, k)
        ref, mag = oracle.spmm_bcsr(A.pos, A.crd, A.vals, B, 4, threads=8)
        D, Bd = DevCSR(A), dev(B)
        for tile in (0, 64, 512):
            say("bcsr spmm", name, "k", k, "tile", tile)
            C = torch.full((A.rows * 4, k), float("nan"), device="cuda")
            psk.psk_spmm_bcsr(A.rows, A.cols, A.nnz, 4, D.pos, D.crd, D.vals, Bd, C, tile=tile)
            torch.cuda.synchronize()
            check(C.cpu().numpy(), ref, mag, "bcsr spmm %s k=%d tile %d" % (name, k, tile))


@pytest.mark.parametrize("bs", [2, 4, 8])
@pytest.mark.parametrize("k", [64, 40, 7])
def test_bcsr_spmm_strided_operands(bs, k):
    """B and C with row strides larger than k (ldb = k + 3, ldc = k + 5): the padding of C stays untouched."""
    rng = np.random.default_rng(70 + bs)
    A = wl.csr_from_lengths(adversarial_lengths(rng, 1203, 1501, "mixed"), 1501, seed=57, bs=bs)
    Bh = wl.dense_uniform(A.cols * bs * (k + 3), 58, wl.S_B).reshape(A.cols * bs, k + 3)
    ref, mag = oracle.spmm_bcsr(A.pos, A.crd, A.vals, Bh[:, :k], bs, threads=8)
    D = DevCSR(A)
    Bd = dev(Bh)[:, :k]
    for tile in (0, 64):
        say("bcsr spmm strided bs", bs, "k", k, "tile", tile)
        Cfull = torch.full((A.rows * bs, k + 5), -7.0, device="cuda")
        C = Cfull[:, :k]
        C.fill_(float("nan"))
        psk.psk_spmm_bcsr(A.rows, A.cols, A.nnz, bs, D.pos, D.crd, D.vals, Bd, C, tile=tile)
        torch.cuda.synchronize()
        check(C.cpu().numpy(), ref, mag, "bcsr spmm strided bs %d k %d tile %d" % (bs, k, tile))
        assert bool((Cfull[:, k:] == -7.0).all()), "columns beyond k were written"


@pytest.mark.parametrize("bs,tiles", [(2, [0, 512, 1024, 2048]), (8, [0, 32, 64, 128])])
def test_bcsr_other_block_sizes(bs, tiles):
    """2 x 2 and 8 x 8 blocks: SpMV (kernel of its own) and SpMM (the 4 x 4 kernel's template)."""
    rng = np.random.default_rng(60 + bs)
    cases = [(kind, wl.csr_from_lengths(adversarial_lengths(rng, 1203, 1501, kind), 1501, seed=53, bs=bs))
             for kind in ADVERSARIAL_KINDS]
    cases.append(("eight per block row", wl.csr_from_lengths(np.full(6000, 8), 6000, seed=54, bs=bs)))
    for name, A in cases:
        x = wl.dense_uniform(A.cols * bs, 53, wl.S_X)
        ref, mag = oracle.spmv_bcsr(A.pos, A.crd, A.vals, x, bs, threads=8)
        D, xd = DevCSR(A), dev(x)
        for tile in tiles:
            say("bcsr spmv", name, "bs", bs, "tile", tile, "blocks", A.nnz)
            y = torch.full((A.rows * bs,), float("nan"), device="cuda")
            psk.psk_spmv_bcsr(A.rows, A.cols, A.nnz, bs, D.pos, D.crd, D.vals, xd, y, tile=tile)
            torch.cuda.synchronize()
            check(y.cpu().numpy(), ref, mag, "bcsr spmv %s bs %d tile %d" % (name, bs, tile))
        for k in (64, 40, 256):
            B = wl.dense_uniform(A.cols * bs * k, 55, wl.S_B).reshape(A.cols * bs, k)
            refC, magC = oracle.spmm_bcsr(A.pos, A.crd, A.vals, B, bs, threads=8)
            say("bcsr spmm", name, "bs", bs, "k", k)
            C = torch.full((A.rows * bs, k), float("nan"), device="cuda")
            psk.psk_spmm_bcsr(A.rows, A.cols, A.nnz, bs, D.pos, D.crd, D.vals, dev(B), C, tile=128)
            torch.cuda.synchronize()
            check(C.cpu().numpy(), refC, magC, "bcsr spmm %s bs %d k %d" % (name, bs, k))


# ------------------------------------------------------------------ cross checks that need no oracle
def test_three_way_agreement_and_tile_invariance():
    c = wl.config(2, 0.01)
    A = c["A"]
    D, xd = DevCSR(A), dev(c["x"])
    ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, c["x"], threads=8)
    bound = 2 * (REL * mag + FLOOR)
    ys = [run_spmv(D, xd, t) for t in SPMV_TILES]
    yw = torch.empty(A.rows, device="cuda")
    psk.psk_spmv_csr_rowsplit(A.rows, A.cols, A.nnz, D.pos, D.crd, D.vals, xd, yw, variant=1)
    torch.cuda.synchronize()
    ys.append(yw.cpu().numpy())
    for a in ys[1:]:
        assert (np.abs(a.astype(np.float64) - ys[0].astype(np.float64)) <= bound).all()


# ------------------------------------------------------------------ column passes
@pytest.mark.parametrize("passes", [2, 3, 4])
def test_spmv_column_passes(passes):
    rng = np.random.default_rng(passes)
    cases = [("powerlaw", wl.config(2, 0.02)["A"])]
    for kind in ("mixed", "one_row_has_all", "mostly_empty", "all_empty", "single_long_rows"):
        cases.append((kind, wl.csr_from_lengths(adversarial_lengths(rng, 3001, 5003, kind), 5003, seed=61)))
    for name, A in cases:
        x = wl.dense_uniform(A.cols, 61, wl.S_X)
        ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, x, threads=8)
        D, xd = DevCSR(A), dev(x)
        for tile in (0, 256, 4096):
            say("column passes", passes, name, "tile", tile)
            got = run_spmv(D, xd, tile, col_passes=passes)
            check(got, ref, mag, "passes %d %s tile %d" % (passes, name, tile))
            again = run_spmv(D, xd, tile, col_passes=passes)
            assert (got == again).all()          # still deterministic


def test_analyze_small_problems_need_no_passes():
    A = wl.config(2, 0.02)["A"]
    D = DevCSR(A)
    assert psk.psk_analyze_csr(A.rows, A.cols, A.nnz, D.pos, D.crd) == 1


def test_validate_matches_the_oracle_on_broken_structures():
    """Integer work: the verdict is compared exactly with the oracle's on planted structural errors."""
    A = wl.csr_from_lengths(np.random.default_rng(12).integers(0, 40, size=5000), 3000, seed=12)
    cases = [("valid", A.pos, A.crd, A.nnz)]
    p = A.pos.copy(); p[0] = 1
    cases.append(("pos[0] != 0", p, A.crd, A.nnz))
    p = A.pos.copy(); p[2500] = p[2499] - 1 if p[2499] > 0 else p[2501] + 1
    cases.append(("pos decreases", p, A.crd, A.nnz))
    cases.append(("pos[rows] != nnz", A.pos, A.crd, A.nnz - 1))
    c = A.crd.copy(); c[A.nnz // 2] = 3000
    cases.append(("column too large", A.pos, c, A.nnz))
    c = A.crd.copy(); c[7] = -1
    cases.append(("negative column", A.pos, c, A.nnz))
    p = A.pos.copy(); p[0] = 1; c = A.crd.copy(); c[0] = 99999
    cases.append(("two errors: the first in order is reported", p, c, A.nnz))
    for name, pos, crd, nnz in cases:
        # the oracle takes the stated nnz from the length of crd: a shortened crd states nnz - 1
        want = oracle.validate_csr(pos, crd[:nnz], A.cols)
        say("validate", name, "expect", want)
        assert psk.psk_validate_csr(A.rows, A.cols, nnz, dev(pos), dev(crd)) == want, name
    assert psk.psk_validate_csr(0, 5, 0, dev(np.zeros(1, dtype=np.int32)), dev(np.zeros(0, dtype=np.int32))) == 0


def test_suggest_schedule_follows_its_rule():
    """Row split only for small matrices with long, alike rows; the position cut otherwise."""
    def ask(lengths):
        pos = np.zeros(len(lengths) + 1, dtype=np.int32)
        pos[1:] = np.cumsum(lengths)
        return psk.psk_suggest_schedule_csr(len(lengths), int(pos[-1]), dev(pos))

    assert ask(np.full(65536, 61)) == psk.PSK_SCHEDULE_ROWS
    assert ask(np.full(4096, 977)) == psk.PSK_SCHEDULE_ROWS
    assert ask(np.full(262144, 15)) == psk.PSK_SCHEDULE_POSITIONS           # short rows
    assert ask(np.full(262144, 61)) == psk.PSK_SCHEDULE_POSITIONS           # 16 M nonzeros: not small
    skew = np.full(16384, 244)
    skew[7] = 244 * 4
    assert ask(skew) == psk.PSK_SCHEDULE_POSITIONS                          # one row 4 x the mean
    skew[7] = 244 * 3
    assert ask(skew) == psk.PSK_SCHEDULE_ROWS
    assert ask(np.diff(wl.config(2, 0.02)["A"].pos)) == psk.PSK_SCHEDULE_POSITIONS
    assert ask(np.zeros(0, dtype=np.int64)) == psk.PSK_SCHEDULE_POSITIONS


# ------------------------------------------------------------------ the schedule's atomics strategy (baseline)
def test_spmv_atomics_baseline():
    rng = np.random.default_rng(8)
    cases = [("powerlaw", wl.config(2, 0.02)["A"]), ("stencil", wl.config(3, 0.01)["A"])]
    for kind in ("mixed", "one_row_has_all", "all_empty", "single_long_rows", "empty_head_tail"):
        cases.append((kind, wl.csr_from_lengths(adversarial_lengths(rng, 3001, 5003, kind), 5003, seed=71)))
    for name, A in cases:
        x = wl.dense_uniform(A.cols, 71, wl.S_X)
        ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, x, threads=8)
        D, xd = DevCSR(A), dev(x)
        for tile in (0, 256, 1024):
            say("atomics", name, "tile", tile)
            y = torch.full((A.rows,), float("nan"), device="cuda")
            psk.psk_spmv_csr_atomics(A.rows, A.cols, A.nnz, D.pos, D.crd, D.vals, xd, y, tile=tile)
            torch.cuda.synchronize()
            check(y.cpu().numpy(), ref, mag, "atomics %s tile %d" % (name, tile))


def test_spmv_without_temporary_ablation():
    """The ablation kernel (rolled load loop, no register temporary) computes the same product."""
    rng = np.random.default_rng(9)
    cases = [("powerlaw", wl.config(2, 0.02)["A"]), ("stencil", wl.config(3, 0.01)["A"])]
    for kind in ("mixed", "one_row_has_all", "all_empty", "single_long_rows", "empty_head_tail"):
        cases.append((kind, wl.csr_from_lengths(adversarial_lengths(rng, 3001, 5003, kind), 5003, seed=72)))
    for name, A in cases:
        x = wl.dense_uniform(A.cols, 72, wl.S_X)
        ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, x, threads=8)
        D, xd = DevCSR(A), dev(x)
        for tile in (0, 256, 512, 1024, 4096):
            say("no temporary", name, "tile", tile)
            y = torch.full((A.rows,), float("nan"), device="cuda")
            psk.psk_spmv_csr_notemp(A.rows, A.cols, A.nnz, D.pos, D.crd, D.vals, xd, y, tile=tile)
            torch.cuda.synchronize()
            check(y.cpu().numpy(), ref, mag, "no temporary %s tile %d" % (name, tile))


# ------------------------------------------------------------------ randomised shapes
def test_random_shapes_all_operations():
    """Sixty seeded random problems: sizes, row-length mixes, tiles, dense widths and pass counts drawn
    at random; every operation against the oracle."""
    rng = np.random.default_rng(20010532)
    for case in range(60):
        rows = int(rng.integers(1, 4000))
        cols = int(rng.integers(1, 6000))
        style = rng.integers(0, 4)
        if style == 0:
            L = rng.integers(0, min(cols, 12) + 1, size=rows)
        elif style == 1:
            L = np.where(rng.random(rows) < 0.9, 0, rng.integers(0, min(cols, 400) + 1, size=rows))
        elif style == 2:
            L = np.minimum(rng.zipf(1.6, size=rows), cols)
        else:
            L = np.zeros(rows, dtype=np.int64)
            L[rng.integers(0, rows, size=3)] = min(cols, int(rng.integers(1, 6000)))
        seed = 1000 + case
        A = wl.csr_from_lengths(L, cols, seed=seed)
        x = wl.dense_uniform(cols, seed, wl.S_X)
        k = int(rng.choice([1, 3, 32, 64, 65, 128, 200]))
        B = wl.dense_uniform(cols * k, seed, wl.S_B).reshape(cols, k)
        tile_v = int(rng.choice([0, 256, 512, 1024, 2048, 4096]))
        tile_m = int(rng.choice([0, 256, 512, 1024, 2048]))
        passes = int(rng.choice([1, 1, 2, 3, 4]))
        say("random case", case, "rows", rows, "cols", cols, "nnz", A.nnz, "style", int(style), "k", k,
            "tiles", tile_v, tile_m, "passes", passes)
        D, xd, Bd = DevCSR(A), dev(x), dev(B)
        want = oracle.partition(A.pos, tile_v or 2048)
        got = psk.psk_partition_csr(D.pos, A.nnz, tile_v or 2048).cpu().numpy()
        assert (got == want).all()
        ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, x)
        check(run_spmv(D, xd, tile_v, col_passes=passes), ref, mag, "random %d spmv" % case)
        refC, magC = oracle.spmm_csr(A.pos, A.crd, A.vals, B)
        check(run_spmm(D, Bd, tile_m), refC, magC, "random %d spmm" % case)
        # the same pattern as a BCSR matrix of 4x4 blocks
        Ab = wl.csr_from_lengths(L, cols, seed=seed, bs=4)
        xb = wl.dense_uniform(cols * 4, seed, wl.S_X)
        tile_b = int(rng.choice([0, 64, 128, 256, 512]))
        Db = DevCSR(Ab)
        yb = torch.full((rows * 4,), float("nan"), device="cuda")
        psk.psk_spmv_bcsr(rows, cols, Ab.nnz, 4, Db.pos, Db.crd, Db.vals, dev(xb), yb, tile=tile_b)
        torch.cuda.synchronize()
        refb, magb = oracle.spmv_bcsr(Ab.pos, Ab.crd, Ab.vals, xb, 4)
        check(yb.cpu().numpy(), refb, magb, "random %d bcsr spmv" % case)
        if case % 4 == 0:
            kb = int(rng.choice([8, 64, 100]))
            Bb = wl.dense_uniform(cols * 4 * kb, seed, wl.S_B).reshape(cols * 4, kb)
            Cb = torch.full((rows * 4, kb), float("nan"), device="cuda")
            psk.psk_spmm_bcsr(rows, cols, Ab.nnz, 4, Db.pos, Db.crd, Db.vals, dev(Bb), Cb, tile=tile_b)
            torch.cuda.synchronize()
            refCb, magCb = oracle.spmm_bcsr(Ab.pos, Ab.crd, Ab.vals, Bb, 4)
            check(Cb.cpu().numpy(), refCb, magCb, "random %d bcsr spmm" % case)
