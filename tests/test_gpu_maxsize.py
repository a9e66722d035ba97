"""The largest problem the int32 position arrays allow: nnz = 2^31 - 128 (17 GB of crd and vals).  A seeded
block of 2^24 - 1 nonzeros is replicated 128 times down the rows on the device (plain copies with shifted
positions, no arithmetic of the method), so the oracle's result for a row of the block is the reference
for every copy of that row.  Partition bit-exact on sampled table entries, SpMV within the fp32 bar."""
import sys

import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_2001_00532_amd as psk  # noqa: E402

COPIES = 128


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def test_spmv_at_the_int32_limit():
    if torch.cuda.mem_get_info()[0] < 40 * 2 ** 30:
        pytest.skip("needs 40 GB of free device memory")
    # block: power-law rows, trimmed to exactly 2^24 - 1 stored entries
    L = wl.zipf_lengths(600_000, 1.8, 1, 200_000, 4242).astype(np.int64)
    want = 2 ** 24 - 1
    cs = np.cumsum(L)
    rb = int(np.searchsorted(cs, want, side="right"))       # rows that fit entirely
    L = L[:rb + 1].copy()
    L[rb] = want - (cs[rb - 1] if rb else 0)
    cols = 1_000_000
    A = wl.csr_from_lengths(L, cols, seed=4242)
    assert A.nnz == want
    rows_b = A.rows
    x = wl.dense_uniform(cols, 4242, wl.S_X)
    ref, mag = oracle.spmv_csr(A.pos, A.crd, A.vals, x, threads=16)

    rows, nnz = rows_b * COPIES, want * COPIES
    assert nnz == 2 ** 31 - 128
    say("max size: rows", rows, "nnz", nnz)
    dev = torch.device("cuda")
    pos_b = torch.from_numpy(A.pos.astype(np.int64)).to(dev)
    shifts = torch.arange(COPIES, dtype=torch.int64, device=dev) * want
    pos = (pos_b[:-1].unsqueeze(0) + shifts.unsqueeze(1)).reshape(-1)
    pos = torch.cat([pos, torch.tensor([nnz], dtype=torch.int64, device=dev)]).to(torch.int32)
    crd = torch.from_numpy(A.crd).to(dev).repeat(COPIES)
    vals = torch.from_numpy(A.vals).to(dev).repeat(COPIES)
    xd = torch.from_numpy(x).to(dev)
    assert crd.numel() == nnz and int(pos[-1]) == nnz

    for tile, passes in ((2048, 1), (1024, 2)):
        ws = psk.workspace(psk.PSK_OP_SPMV_CSR, rows, nnz, tile=tile)
        # the cut: sampled entries of the table against the definition, evaluated with the block's pos
        say("partition, tile", tile)
        tr = psk.psk_partition_csr(pos, nnz, tile).cpu().numpy().astype(np.int64)
        nt = -(-nnz // tile)
        assert tr.shape[0] == nt + 1 and tr[-1] == rows
        ts = np.unique(np.concatenate([np.arange(0, 2000), np.arange(nt - 2000, nt), np.random.default_rng(1).integers(0, nt, 20000)]))
        first = np.minimum(ts * tile, nnz)
        copy, inside = first // want, first % want
        exp = copy * rows_b + (np.searchsorted(A.pos.astype(np.int64), inside, side="right") - 1)
        assert (tr[ts] == exp).all()
        say("spmv, tile", tile, "passes", passes)
        y = torch.full((rows,), float("nan"), device=dev)
        psk.psk_spmv_csr(rows, cols, nnz, pos, crd, vals, xd, y, tile=tile, col_passes=passes, ws=ws)
        torch.cuda.synchronize()
        got = y.cpu().numpy().reshape(COPIES, rows_b)
        assert not np.isnan(got).any()
        bound = 1e-5 * mag + 1e-30
        worst = (np.abs(got - ref[None, :]) / bound[None, :]).max()
        assert worst <= 1.0, "tile %d passes %d: worst |err|/bound = %.3g" % (tile, passes, worst)
        del y, ws

    # the divided variant at the same size: the last part ends within 2048 positions of 2^31, where a chunk
    # start that is stepped past the end of the part would wrap around (chunks are counted instead)
    say("divided spmv, 2048 parts")
    ws = psk.workspace(psk.PSK_OP_SPMV_CSR, rows, nnz, tile=2048)
    y = torch.full((rows,), float("nan"), device=dev)
    psk.psk_spmv_csr_divide(rows, cols, nnz, pos, crd, vals, xd, y, parts=0, ws=ws)
    torch.cuda.synchronize()
    got = y.cpu().numpy().reshape(COPIES, rows_b)
    assert not np.isnan(got).any()
    worst = (np.abs(got - ref[None, :]) / (1e-5 * mag + 1e-30)[None, :]).max()
    assert worst <= 1.0, "divided: worst |err|/bound = %.3g" % worst
