"""The seeded generators against closed forms and structural invariants."""
import hashlib

import numpy as np
import pytest

import workloads as wl


def check_structure(A):
    pos, crd = A.pos, A.crd
    assert pos.dtype == np.int32 and crd.dtype == np.int32 and A.vals.dtype == np.float32
    assert pos[0] == 0 and pos[-1] == crd.size and (np.diff(pos) >= 0).all()
    assert A.vals.size == crd.size * A.bs * A.bs
    if crd.size:
        assert crd.min() >= 0 and crd.max() < A.cols
        # strictly ascending inside each row: a decrease may only happen at a row start
        dec = np.flatnonzero(np.diff(crd) <= 0) + 1
        starts = set(pos.tolist())
        assert all(int(p) in starts for p in dec)


def test_config1_shape():
    c = wl.config(1)
    A = c["A"]
    check_structure(A)
    assert (A.rows, A.cols, A.nnz) == (1024, 1024, 10240)
    assert (np.diff(A.pos) == 10).all()
    assert c["x"].shape == (1024,) and c["x"].min() >= -1 and c["x"].max() < 1
    assert A.vals.min() >= -1 and A.vals.max() < 1 and abs(float(A.vals.mean())) < 0.05


def test_same_seed_same_bytes_and_seed_matters():
    a, b = wl.config(2, scale=0.001), wl.config(2, scale=0.001)
    for k in ("pos", "crd", "vals"):
        assert hashlib.sha256(getattr(a["A"], k).tobytes()).digest() == hashlib.sha256(
            getattr(b["A"], k).tobytes()).digest()
    assert (a["x"] == b["x"]).all()
    other = wl.csr_uniform(100, 100, 5, seed=1)
    again = wl.csr_uniform(100, 100, 5, seed=2)
    assert not (other.crd == again.crd).all()


def test_values_are_exact_24bit_grid():
    v = wl.dense_uniform(10000, 9, wl.S_X)
    scaled = (v.astype(np.float64) + 1.0) * 2.0 ** 23
    assert (scaled == np.round(scaled)).all()


def test_zipf_law():
    L = wl.zipf_lengths(400000, 1.8, 1, 200000, seed=5)
    assert L.min() >= 1 and L.max() <= 200000
    k = np.arange(1, 200001, dtype=np.float64)
    pmf = k ** -1.8
    pmf /= pmf.sum()
    assert abs((L == 1).mean() - pmf[0]) < 0.005
    assert abs((L <= 4).mean() - pmf[:4].sum()) < 0.005
    assert abs((L > 1024).mean() - pmf[1024:].sum()) < 0.0008
    # bounds are honoured
    L2 = wl.zipf_lengths(1000, 1.8, 3, 7, seed=5)
    assert L2.min() >= 3 and L2.max() <= 7


def test_powerlaw_config_small():
    c = wl.config(2, scale=0.01)
    A = c["A"]
    check_structure(A)
    assert A.rows == 20000 and np.diff(A.pos).min() >= 1 and np.diff(A.pos).max() <= 2000


@pytest.mark.parametrize("n", [2, 3, 5, 8])
def test_stencil_closed_forms(n):
    A = wl.csr_stencil27(n, seed=1)
    check_structure(A)
    assert A.nnz == (3 * n - 2) ** 3
    L = np.diff(A.pos)
    if n >= 3:
        hist = {int(k): int(v) for k, v in zip(*np.unique(L, return_counts=True))}
        assert hist == {27: (n - 2) ** 3, 18: 6 * (n - 2) ** 2, 12: 12 * (n - 2), 8: 8} or n == 3 and hist == {
            27: 1, 18: 6, 12: 12, 8: 8}
    rows = np.repeat(np.arange(A.rows), L)
    diag = A.crd == rows
    assert diag.sum() == A.rows and (A.vals[diag] == 27.0).all()
    off = A.vals[~diag]
    assert off.min() >= 0.5 and off.max() < 1.5
    # neighbours differ by at most 1 in each grid coordinate
    r, c = rows, A.crd
    for div in (1, n, n * n):
        assert (np.abs((r // div) % n - (c // div) % n) <= 1).all()
    # symmetric pattern
    pairs = set(zip(r.tolist(), c.tolist()))
    assert all((j, i) in pairs for i, j in list(pairs)[:2000])


def test_full_stencil_nnz_formula():
    assert (3 * 160 - 2) ** 3 == 109_215_352


def test_config4_and_5_small():
    c = wl.config(4, scale=0.001)
    A = c["A"]
    check_structure(A)
    assert (np.diff(A.pos) == 16).all() and c["B"].shape == (1000, 128) and c["k"] == 128
    c = wl.config(5, scale=0.001)
    A = c["A"]
    check_structure(A)
    assert A.bs == 4 and (np.diff(A.pos) == 8).all() and A.vals.size == A.nnz * 16
    assert c["x"].shape == (A.cols * 4,) and c["B"].shape == (A.cols * 4, 64)


def test_from_lengths_edge_cases():
    A = wl.csr_from_lengths([0, 0, 0], 5, seed=1)
    assert A.nnz == 0 and A.pos.tolist() == [0, 0, 0, 0]
    A = wl.csr_from_lengths([5, 0, 5], 5, seed=1)          # rows as long as the column count
    assert A.crd.tolist() == [0, 1, 2, 3, 4, 0, 1, 2, 3, 4]
    A = wl.csr_from_lengths([100, 3000], 4000, seed=1)     # long rows take the sort/dedupe branch
    check_structure(A)
    with pytest.raises(ValueError):
        wl.csr_from_lengths([6], 5, seed=1)


def test_power_law_configuration_has_the_recorded_bytes():
    """The generators are counter-based: the same seed gives the same bytes on every machine.  The hash is
    the one bench.py prints for its default workload (computed by this repository's generators, not taken
    from anywhere else)."""
    import hashlib

    c = wl.config(2)
    A = c["A"]
    h = hashlib.blake2b(digest_size=8)
    for a in (A.pos, A.crd, A.vals, c["x"]):
        h.update(np.ascontiguousarray(a).view(np.uint8).reshape(-1).data)
    assert h.hexdigest() == "b182aa2126833ff2"
    assert A.nnz == 56_486_638
