"""Seeded synthetic inputs shaped like the evaluated workloads.

Inputs only: sparsity patterns, values, dense operands.  Nothing here computes
a product, a reduction or a position cut, so the CPU oracle and the HIP path
can both be fed from this module without sharing any of the method's logic.

The paper evaluates on SuiteSparse/FROSTT collections and on synthetic
matrices (random nonzeros, skewed row lengths, few long rows: Section 8.1,
8.3-8.5).  The collections are not available offline; the generators below
stand in for them with the same structural classes.

Matrices are returned as a ``CSR`` tuple of numpy arrays (int32 ``pos`` and
``crd``, float32 ``vals``); BCSR matrices use the same container with ``bs``
set, ``pos``/``crd`` indexing blocks and ``vals`` holding ``bs*bs`` floats per
block, row-major inside a block.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gen.c")
_SO = os.path.join(_HERE, "libworkloads.so")

BASE_SEED = 200100532  # config n uses BASE_SEED + n

# stream identifiers (which array a draw belongs to)
S_VALS, S_COLS, S_X, S_B, S_LEN = 1, 2, 3, 4, 5


def build(force: bool = False) -> str:
    """Compile gen.c into libworkloads.so (host code, gcc + OpenMP)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _SO, _SRC, "-lm"]
        )
    return _SO


_lib_handle = None


def _lib():
    global _lib_handle
    if _lib_handle is None:
        lib = ctypes.CDLL(build())
        i64, u64, f32, p = ctypes.c_int64, ctypes.c_uint64, ctypes.c_float, ctypes.c_void_p
        lib.wl_fill_uniform.argtypes = [p, i64, u64, u64, f32, f32]
        lib.wl_fill_uniform.restype = None
        lib.wl_zipf_lengths.argtypes = [p, i64, ctypes.c_double, ctypes.c_int32, ctypes.c_int32, u64, u64]
        lib.wl_zipf_lengths.restype = ctypes.c_int
        lib.wl_csr_columns.argtypes = [p, i64, i64, u64, u64, p]
        lib.wl_csr_columns.restype = ctypes.c_int
        lib.wl_stencil27_nnz.argtypes = [i64]
        lib.wl_stencil27_nnz.restype = i64
        lib.wl_stencil27.argtypes = [i64, u64, u64, p, p, p]
        lib.wl_stencil27.restype = ctypes.c_int
        _lib_handle = lib
    return _lib_handle


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


@dataclass
class CSR:
    rows: int          # rows (block rows when bs > 1)
    cols: int          # columns (block columns when bs > 1)
    pos: np.ndarray    # int32 [rows+1]
    crd: np.ndarray    # int32 [nnz]   (block columns when bs > 1)
    vals: np.ndarray   # float32 [nnz * bs * bs]
    bs: int = 1        # dense block edge (1 = plain CSR)

    @property
    def nnz(self) -> int:
        """Stored positions at the compressed level (blocks when bs > 1)."""
        return int(self.pos[-1])


def dense_uniform(n: int, seed: int, stream: int, lo: float = -1.0, hi: float = 1.0) -> np.ndarray:
    out = np.empty(int(n), dtype=np.float32)
    _lib().wl_fill_uniform(_ptr(out), int(n), seed, stream, lo, hi)
    return out


def dense_uniform_f64(n: int, seed: int, stream: int, lo: float = -1.0, hi: float = 1.0) -> np.ndarray:
    """fp64 values with 48 random significand bits: two 24-bit draws, the second scaled by 2^-24."""
    a = dense_uniform(n, seed, stream, lo, hi).astype(np.float64)
    b = dense_uniform(n, seed ^ 0x5DEECE66D, stream, 0.0, 1.0).astype(np.float64)
    return a + b * (hi - lo) * 2.0 ** -24


def csr_from_lengths(lengths, cols: int, seed: int, lo: float = -1.0, hi: float = 1.0, bs: int = 1) -> CSR:
    """CSR/BCSR with the given number of stored entries per row; columns are
    distinct, uniform over [0, cols) and sorted within each row."""
    lengths = np.ascontiguousarray(lengths, dtype=np.int64)
    rows = int(lengths.shape[0])
    if lengths.size and (lengths.min() < 0 or lengths.max() > cols):
        raise ValueError("row length outside [0, cols]")
    total = int(lengths.sum())
    if total >= 2**31:
        raise ValueError("nnz does not fit int32 positions")
    pos = np.zeros(rows + 1, dtype=np.int32)
    pos[1:] = np.cumsum(lengths, dtype=np.int64).astype(np.int32)
    crd = np.empty(total, dtype=np.int32)
    if _lib().wl_csr_columns(_ptr(pos), rows, int(cols), seed, S_COLS, _ptr(crd)) != 0:
        raise RuntimeError("column generation failed")
    vals = dense_uniform(total * bs * bs, seed, S_VALS, lo, hi)
    return CSR(rows, int(cols), pos, crd, vals, bs)


@dataclass
class DCSR:
    rows: int          # extent of the row dimension
    cols: int
    crd_i: np.ndarray  # int32 [nstored]  coordinates of the stored rows, strictly increasing
    pos: np.ndarray    # int32 [nstored+1]
    crd: np.ndarray    # int32 [nnz]
    vals: np.ndarray   # float32 [nnz]

    @property
    def nstored(self) -> int:
        return int(self.crd_i.shape[0])

    @property
    def nnz(self) -> int:
        return int(self.pos[-1])


def dcsr_from_lengths(rows: int, lengths, cols: int, seed: int) -> DCSR:
    """DCSR with len(lengths) stored rows (a stored row may still be empty) placed at distinct,
    sorted row coordinates drawn uniformly from [0, rows)."""
    A = csr_from_lengths(lengths, cols, seed)
    n = A.rows
    if n > rows:
        raise ValueError("more stored rows than rows")
    if n == rows:
        crd_i = np.arange(rows, dtype=np.int32)
    else:
        # distinct sorted coordinates: stratified draw, one per equal slice of [0, rows)
        u = dense_uniform(n, seed, S_LEN, 0.0, 1.0).astype(np.float64)
        lo = (np.arange(n, dtype=np.int64) * rows) // max(1, n)
        hi = ((np.arange(n, dtype=np.int64) + 1) * rows) // max(1, n)
        crd_i = (lo + np.minimum((u * (hi - lo)).astype(np.int64), hi - lo - 1)).astype(np.int32)
    return DCSR(int(rows), int(cols), crd_i, A.pos, A.crd, A.vals)


def csr_uniform(rows: int, cols: int, per_row: int, seed: int, bs: int = 1) -> CSR:
    """Exactly ``per_row`` stored entries in every row."""
    return csr_from_lengths(np.full(rows, per_row, dtype=np.int64), cols, seed, bs=bs)


def zipf_lengths(rows: int, alpha: float, kmin: int, kmax: int, seed: int) -> np.ndarray:
    out = np.empty(rows, dtype=np.int32)
    if _lib().wl_zipf_lengths(_ptr(out), rows, alpha, kmin, kmax, seed, S_LEN) != 0:
        raise RuntimeError("zipf generation failed")
    return out


def csr_powerlaw(rows: int, cols: int, alpha: float, kmin: int, kmax: int, seed: int) -> CSR:
    """Row lengths i.i.d. from the truncated Zipf law k^-alpha on [kmin, kmax]."""
    return csr_from_lengths(zipf_lengths(rows, alpha, kmin, min(kmax, cols), seed), cols, seed)


@dataclass
class CSF3:
    """Order-3 tensor B(i,k,l) as a three-level coordinate hierarchy: slices (mode i, dense when crd_i is
    None), fibers (mode k), leaves (mode l)."""
    dims: tuple            # (I, K, L)
    crd_i: object          # int32 [nslices] or None
    pos_k: np.ndarray      # int32 [nslices+1]
    crd_k: np.ndarray      # int32 [nfibers]
    pos_l: np.ndarray      # int32 [nfibers+1]
    crd_l: np.ndarray      # int32 [nnz]
    vals: np.ndarray       # float32 [nnz]

    @property
    def nslices(self) -> int:
        return int(self.pos_k.size - 1)

    @property
    def nfibers(self) -> int:
        return int(self.pos_l.size - 1)

    @property
    def nnz(self) -> int:
        return int(self.pos_l[-1])


def csf3_from_lengths(fibers_per_slice, leaves_per_fiber, dims, seed: int, compressed_i: bool = False) -> CSF3:
    """fibers_per_slice[s] fibers in slice s (distinct sorted k), leaves_per_fiber[q] leaves in fiber q
    (distinct sorted l).  With compressed_i the slices get distinct sorted coordinates out of dims[0]."""
    I, K, L = dims
    lk = csr_from_lengths(fibers_per_slice, K, seed)
    if lk.nnz != len(leaves_per_fiber):
        raise ValueError("leaves_per_fiber must have one entry per fiber")
    ll = csr_from_lengths(leaves_per_fiber, L, seed + 7919)
    crd_i = None
    if compressed_i:
        crd_i = csr_from_lengths([lk.rows], I, seed + 104729).crd
    elif lk.rows != I:
        raise ValueError("dense first level needs one entry of fibers_per_slice per i")
    return CSF3((I, K, L), crd_i, lk.pos, lk.crd, ll.pos, ll.crd, ll.vals)


def csf3_powerlaw(I: int, K: int, L: int, mean_fibers: float, alpha: float, max_leaves: int, seed: int) -> CSF3:
    """Synthetic stand-in for a FROSTT-like tensor: about mean_fibers fibers per slice (uniform in
    [0, 2*mean_fibers]), leaves per fiber from the truncated Zipf law k^-alpha on [1, max_leaves]."""
    fps = (dense_uniform(I, seed, S_LEN, 0.0, 1.0) * (2 * mean_fibers + 1)).astype(np.int64)
    fps = np.minimum(fps, K)
    lpf = zipf_lengths(int(fps.sum()), alpha, 1, min(max_leaves, L), seed + 1)
    return csf3_from_lengths(fps, lpf, (I, K, L), seed)


def exponential_lengths(rows: int, total: int, base: float, cols: int, seed: int) -> np.ndarray:
    """Row lengths proportional to base**rank, scaled to about `total` stored entries, capped at
    `cols`, then shuffled (the skew experiment of Section 8.4: nnz fixed, skew set by the base of an
    exponential, rows in random order).  base = 1 gives equal rows."""
    rank = np.arange(rows, dtype=np.float64)
    w = np.exp((rank - (rows - 1)) * np.log(base)) if base > 1.0 else np.ones(rows)
    L = np.minimum(np.floor(w / w.sum() * total + 0.5), cols).astype(np.int64)
    order = np.argsort(dense_uniform(rows, seed, S_LEN), kind="stable")
    return L[order]


def csr_stencil27(n: int, seed: int) -> CSR:
    """27-point stencil on an n^3 grid, clipped at the faces; diagonal 27,
    off-diagonals uniform in [0.5, 1.5)."""
    lib = _lib()
    rows = n ** 3
    nnz = int(lib.wl_stencil27_nnz(n))
    pos = np.empty(rows + 1, dtype=np.int32)
    crd = np.empty(nnz, dtype=np.int32)
    vals = np.empty(nnz, dtype=np.float32)
    if lib.wl_stencil27(n, seed, S_VALS, _ptr(pos), _ptr(crd), _ptr(vals)) != 0:
        raise RuntimeError("stencil generation failed")
    return CSR(rows, rows, pos, crd, vals, 1)


def config(n: int, scale: float = 1.0) -> dict:
    """The n-th evaluated configuration (1..5) as a dict with the matrix ``A``
    and the dense operands (``x`` and/or ``B`` with ``k`` columns).

    ``scale`` < 1 shrinks the row/column counts (and the stencil edge by its
    cube root) for tests; the structure class is unchanged.
    """
    seed = BASE_SEED + n
    s = float(scale)
    if n == 1:
        r = max(16, int(round(1024 * s)))
        A = csr_uniform(r, r, min(10, r), seed)
        return {"name": "csr_spmv_uniform10", "A": A, "x": dense_uniform(r, seed, S_X)}
    if n == 2:
        r = max(16, int(round(2_000_000 * s)))
        A = csr_powerlaw(r, r, 1.8, 1, max(1, int(round(200_000 * s))), seed)
        return {"name": "csr_spmv_powerlaw", "A": A, "x": dense_uniform(r, seed, S_X)}
    if n == 3:
        g = max(2, int(round(160 * s ** (1.0 / 3.0))))
        A = csr_stencil27(g, seed)
        return {"name": "csr_spmv_stencil27", "A": A, "x": dense_uniform(A.cols, seed, S_X), "grid": g}
    if n == 4:
        r = max(16, int(round(1_000_000 * s)))
        A = csr_uniform(r, r, min(16, r), seed)
        k = 128
        return {"name": "csr_spmm_uniform16_k128", "A": A, "k": k,
                "B": dense_uniform(r * k, seed, S_B).reshape(r, k)}
    if n == 5:
        br = max(8, int(round(250_000 * s)))
        A = csr_uniform(br, br, min(8, br), seed, bs=4)
        k = 64
        return {"name": "bcsr4_spmv_spmm_n64", "A": A, "k": k,
                "x": dense_uniform(br * 4, seed, S_X),
                "B": dense_uniform(br * 4 * k, seed, S_B).reshape(br * 4, k)}
    raise ValueError("config must be 1..5")
