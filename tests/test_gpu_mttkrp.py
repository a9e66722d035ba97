"""GPU parity for MTTKRP on a three-level compressed tensor: the two-level position cut bit for bit,
the result within |got - ref| <= 1e-5 * sum |b c d| + 1e-30 per output element."""
import sys

import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_2001_00532_amd as psk  # noqa: E402

REL, FLOOR = 1e-5, 1e-30
TILES = [0, 256, 512, 1024, 2048]


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def tensors():
    rng = np.random.default_rng(12)
    # (name, fibers per slice, leaves per fiber, dims, compressed first level)
    ns = 700
    fps = rng.integers(0, 9, size=ns)
    yield "mixed", fps, rng.integers(0, 12, size=int(fps.sum())), (ns, 900, 1100), False
    fps = rng.integers(0, 5, size=300)
    yield "compressed_i", fps, rng.integers(1, 30, size=int(fps.sum())), (5000, 400, 700), True
    fps = np.zeros(200, dtype=np.int64)
    fps[[3, 77, 150]] = [2, 300, 1]
    lpf = np.full(int(fps.sum()), 3, dtype=np.int64)
    lpf[[0, 5, 200]] = [2500, 0, 1999]                      # long fibers, an empty one
    yield "long_fibers_few_slices", fps, lpf, (200, 350, 3000), False
    yield "all_empty", np.zeros(50, dtype=np.int64), np.zeros(0, dtype=np.int64), (50, 10, 10), False
    yield "empty_fibers_only", np.full(40, 3), np.zeros(120, dtype=np.int64), (40, 10, 10), False
    yield "one_leaf", np.array([0, 0, 1, 0]), np.array([1]), (4, 5, 6), False
    yield "ones", np.ones(3000, dtype=np.int64), np.ones(3000, dtype=np.int64), (3000, 64, 64), False


def run_case(name, T, j, tile, ld_extra=0):
    I, K, L = T.dims
    Cfull = wl.dense_uniform(K * (j + ld_extra), 7, wl.S_B).reshape(K, j + ld_extra)
    Dfull = wl.dense_uniform(L * (j + ld_extra), 8, wl.S_B).reshape(L, j + ld_extra)
    C, D = Cfull[:, :j], Dfull[:, :j]
    ref, mag = oracle.mttkrp_csf3(T.pos_k, T.crd_k, T.pos_l, T.crd_l, T.vals, C, D, threads=8)
    full_ref = np.zeros((I, j))
    full_mag = np.zeros((I, j))
    rows = T.crd_i if T.crd_i is not None else np.arange(T.nslices)
    full_ref[rows] = ref
    full_mag[rows] = mag
    Cd, Dd = dev(Cfull)[:, :j], dev(Dfull)[:, :j]
    Afull = torch.full((I, j + ld_extra), float("nan"), device="cuda")
    A = Afull[:, :j]
    psk.psk_mttkrp_csf3(T.dims, dev(T.crd_i), dev(T.pos_k), dev(T.crd_k), dev(T.pos_l), dev(T.crd_l), dev(T.vals),
                        Cd, Dd, A, tile=tile)
    torch.cuda.synchronize()
    ok, worst = oracle.within_tolerance(A.cpu().numpy(), full_ref, full_mag, REL, FLOOR)
    assert ok, "%s j=%d tile=%d: worst |err|/bound = %.3g" % (name, j, tile, worst)


def test_partition_csf3_bit_exact():
    for name, fps, lpf, dims, ci in tensors():
        T = wl.csf3_from_lengths(fps, lpf, dims, seed=33, compressed_i=ci)
        for tile in (1, 7, 256, 1024):
            say("csf3 partition", name, "tile", tile, "nnz", T.nnz)
            ts, tf = psk.psk_partition_csf3(dev(T.pos_k), dev(T.pos_l), T.nnz, tile)
            ws, wf = oracle.partition_csf3(T.pos_k, T.pos_l, tile)
            assert (ts.cpu().numpy() == ws).all() and (tf.cpu().numpy() == wf).all()


@pytest.mark.parametrize("tile", TILES)
def test_mttkrp_structures(tile):
    for name, fps, lpf, dims, ci in tensors():
        T = wl.csf3_from_lengths(fps, lpf, dims, seed=33, compressed_i=ci)
        say("mttkrp", name, "tile", tile, "slices", T.nslices, "fibers", T.nfibers, "nnz", T.nnz)
        run_case(name, T, 64, tile)


@pytest.mark.parametrize("j", [1, 16, 32, 64, 100, 128, 256])
def test_mttkrp_any_rank_and_strides(j):
    T = wl.csf3_powerlaw(2000, 500, 800, 4, 1.6, 300, seed=44)
    say("mttkrp powerlaw j", j, "nnz", T.nnz)
    run_case("powerlaw", T, j, 512)
    run_case("powerlaw strided", T, j, 1024, ld_extra=4)


def test_mttkrp_strided_output_with_rows_that_have_no_slice():
    """Rows of A without a slice (compressed first level) and empty tensors are cleared inside the row
    stride only: the padding columns keep what they held."""
    for name, fps, lpf, dims, ci in tensors():
        if name not in ("compressed_i", "all_empty"):
            continue
        T = wl.csf3_from_lengths(fps, lpf, dims, seed=35, compressed_i=ci)
        say("mttkrp strided", name)
        run_case(name, T, 48, 512, ld_extra=16)
        I = T.dims[0]
        Afull = torch.full((I, 64), 5.0, device="cuda")
        C = dev(wl.dense_uniform(T.dims[1] * 48, 7, wl.S_B).reshape(-1, 48))
        D = dev(wl.dense_uniform(T.dims[2] * 48, 8, wl.S_B).reshape(-1, 48))
        psk.psk_mttkrp_csf3(T.dims, dev(T.crd_i), dev(T.pos_k), dev(T.crd_k), dev(T.pos_l), dev(T.crd_l), dev(T.vals),
                            C, D, Afull[:, :48])
        torch.cuda.synchronize()
        assert torch.all(Afull[:, 48:] == 5.0)


def test_mttkrp_deterministic_and_partition_reuse():
    T = wl.csf3_powerlaw(3000, 700, 900, 5, 1.7, 500, seed=45)
    I, K, L = T.dims
    C = dev(wl.dense_uniform(K * 64, 7, wl.S_B).reshape(K, 64))
    D = dev(wl.dense_uniform(L * 64, 8, wl.S_B).reshape(L, 64))
    args = (T.dims, None, dev(T.pos_k), dev(T.crd_k), dev(T.pos_l), dev(T.crd_l), dev(T.vals), C, D)
    ws = psk.workspace(psk.PSK_OP_MTTKRP_CSF3, T.nslices, T.nnz, k=64)
    A1 = torch.empty((I, 64), device="cuda")
    A2 = torch.empty((I, 64), device="cuda")
    psk.psk_mttkrp_csf3(*args, A1, ws=ws)
    psk.psk_mttkrp_csf3(*args, A2, ws=ws, phases=psk.PSK_PHASE_MAIN | psk.PSK_PHASE_FIXUP)
    torch.cuda.synchronize()
    assert torch.equal(A1, A2)
