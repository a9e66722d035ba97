"""ctypes front end of the CPU oracle (oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports this module
and this module never imports the product package.

Every function takes numpy arrays (int32 index arrays, float32 values and
dense operands) and returns float64 results: the plain definitions
y(i) = A(i,j)*x(j) and C(i,k) = A(i,j)*B(j,k) of the paper's appendix
evaluated over the CSR / BCSR coordinate hierarchy of Section 3, together
with mag = sum |a*x|, and the position cut of Sections 3/5/6.2.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_SO = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile oracle.c (plain C, -O2, OpenMP over rows only)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _SO, _SRC, "-lm"]
        )
    return _SO


_h = None


def _lib():
    global _h
    if _h is None:
        lib = ctypes.CDLL(build())
        i64, i32, p, ci = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int
        lib.oracle_threads.argtypes = [ci]
        lib.oracle_threads.restype = ci
        lib.oracle_spmv_csr.argtypes = [i64, p, p, p, p, p, p, p, i64, ci]
        lib.oracle_spmv_csr.restype = None
        lib.oracle_spmv_csr_f64.argtypes = [i64, p, p, p, p, p, p, p, i64, ci]
        lib.oracle_spmv_csr_f64.restype = None
        lib.oracle_spmv_dcsr.argtypes = [i64, i64, p, p, p, p, p, p, p]
        lib.oracle_spmv_dcsr.restype = None
        lib.oracle_spmm_csr.argtypes = [i64, i64, p, p, p, p, i64, p, p, p, i64, ci]
        lib.oracle_spmm_csr.restype = None
        lib.oracle_spmv_bcsr.argtypes = [i64, i32, p, p, p, p, p, p, p, i64, ci]
        lib.oracle_spmv_bcsr.restype = None
        lib.oracle_spmm_bcsr.argtypes = [i64, i32, i64, p, p, p, p, i64, p, p, p, i64, ci]
        lib.oracle_spmm_bcsr.restype = None
        lib.oracle_mttkrp_csf3.argtypes = [i64, i64, p, p, p, p, p, p, i64, p, i64, p, p, p, i64, ci]
        lib.oracle_mttkrp_csf3.restype = None
        lib.oracle_partition_csf3.argtypes = [i64, i64, i64, p, p, i64, p, p]
        lib.oracle_partition_csf3.restype = None
        lib.oracle_num_tiles.argtypes = [i64, i64]
        lib.oracle_num_tiles.restype = i64
        lib.oracle_partition.argtypes = [i64, i64, p, i64, p]
        lib.oracle_partition.restype = None
        lib.oracle_validate_csr.argtypes = [i64, i64, i64, p, p]
        lib.oracle_validate_csr.restype = ci
        lib.oracle_slab_count.argtypes = [i64, i64, i64, p, p, i64, i64, p]
        lib.oracle_slab_count.restype = ci
        lib.oracle_slab_build.argtypes = [i64, i64, i64, p, p, p, i64, i64, p, p, p, p, p, p, p]
        lib.oracle_slab_build.restype = ci
        lib.oracle_spmv_slab.argtypes = [i64, i64, i64, i64, i64, p, p, p, p, p, p, p, p, p, p]
        lib.oracle_spmv_slab.restype = None
        lib.oracle_slab_build_f64.argtypes = [i64, i64, i64, p, p, p, i64, i64, p, p, p, p, p, p, p]
        lib.oracle_slab_build_f64.restype = ci
        lib.oracle_spmv_slab_f64.argtypes = [i64, i64, i64, i64, i64, p, p, p, p, p, p, p, p]
        lib.oracle_spmv_slab_f64.restype = ci
        _h = lib
    return _h


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _sel(sel):
    if sel is None:
        return None, None, 0
    s = np.ascontiguousarray(sel, dtype=np.int64)
    return s, s.ctypes.data, int(s.size)


def threads_used(threads: int) -> int:
    return int(_lib().oracle_threads(int(threads)))


def spmv_csr(pos, crd, vals, x, sel=None, threads: int = 1):
    """Returns (y, mag) as float64 arrays (one entry per row, or per selected row)."""
    pos, crd, vals, x = _i32(pos), _i32(crd), _f32(vals), _f32(x)
    rows = pos.size - 1
    keep, sp, ns = _sel(sel)
    n = ns if keep is not None else rows
    y = np.empty(n, dtype=np.float64)
    mag = np.empty(n, dtype=np.float64)
    _lib().oracle_spmv_csr(rows, pos.ctypes.data, crd.ctypes.data, vals.ctypes.data, x.ctypes.data,
                           y.ctypes.data, mag.ctypes.data, sp, ns, int(threads))
    return y, mag


def spmv_csr_f64(pos, crd, vals, x, sel=None, threads: int = 1):
    """fp64 operands; sums in extended precision, rounded once.  Returns (y, mag) as float64."""
    pos, crd = _i32(pos), _i32(crd)
    vals = np.ascontiguousarray(vals, dtype=np.float64)
    x = np.ascontiguousarray(x, dtype=np.float64)
    rows = pos.size - 1
    keep, sp, ns = _sel(sel)
    n = ns if keep is not None else rows
    y = np.empty(n, dtype=np.float64)
    mag = np.empty(n, dtype=np.float64)
    _lib().oracle_spmv_csr_f64(rows, pos.ctypes.data, crd.ctypes.data, vals.ctypes.data, x.ctypes.data,
                               y.ctypes.data, mag.ctypes.data, sp, ns, int(threads))
    return y, mag


def spmv_dcsr(rows: int, crd_i, pos, crd, vals, x):
    """DCSR operand: crd_i [nstored] row coordinates, pos [nstored+1].  Returns (y, mag), `rows` float64 each."""
    crd_i, pos, crd, vals, x = _i32(crd_i), _i32(pos), _i32(crd), _f32(vals), _f32(x)
    y = np.empty(int(rows), dtype=np.float64)
    mag = np.empty(int(rows), dtype=np.float64)
    _lib().oracle_spmv_dcsr(int(rows), crd_i.size, crd_i.ctypes.data, pos.ctypes.data, crd.ctypes.data,
                            vals.ctypes.data, x.ctypes.data, y.ctypes.data, mag.ctypes.data)
    return y, mag


def spmm_csr(pos, crd, vals, B, sel=None, threads: int = 1):
    """B is a 2-D row-major float32 array (its row stride is honoured). Returns (C, mag)."""
    pos, crd, vals = _i32(pos), _i32(crd), _f32(vals)
    B = np.asarray(B, dtype=np.float32)
    if B.ndim != 2 or B.strides[1] != 4:
        B = np.ascontiguousarray(B)
    k, ldb = B.shape[1], B.strides[0] // 4
    rows = pos.size - 1
    keep, sp, ns = _sel(sel)
    n = ns if keep is not None else rows
    C = np.empty((n, k), dtype=np.float64)
    mag = np.empty((n, k), dtype=np.float64)
    _lib().oracle_spmm_csr(rows, k, pos.ctypes.data, crd.ctypes.data, vals.ctypes.data, B.ctypes.data, ldb,
                           C.ctypes.data, mag.ctypes.data, sp, ns, int(threads))
    return C, mag


def spmv_bcsr(pos, crd, vals, x, bs: int, sel=None, threads: int = 1):
    """sel lists block rows; outputs have bs entries per (selected) block row."""
    pos, crd, vals, x = _i32(pos), _i32(crd), _f32(vals), _f32(x)
    brows = pos.size - 1
    keep, sp, ns = _sel(sel)
    n = (ns if keep is not None else brows) * bs
    y = np.empty(n, dtype=np.float64)
    mag = np.empty(n, dtype=np.float64)
    _lib().oracle_spmv_bcsr(brows, bs, pos.ctypes.data, crd.ctypes.data, vals.ctypes.data, x.ctypes.data,
                            y.ctypes.data, mag.ctypes.data, sp, ns, int(threads))
    return y, mag


def spmm_bcsr(pos, crd, vals, B, bs: int, sel=None, threads: int = 1):
    pos, crd, vals = _i32(pos), _i32(crd), _f32(vals)
    B = np.asarray(B, dtype=np.float32)
    if B.ndim != 2 or B.strides[1] != 4:
        B = np.ascontiguousarray(B)
    k, ldb = B.shape[1], B.strides[0] // 4
    brows = pos.size - 1
    keep, sp, ns = _sel(sel)
    n = (ns if keep is not None else brows) * bs
    C = np.empty((n, k), dtype=np.float64)
    mag = np.empty((n, k), dtype=np.float64)
    _lib().oracle_spmm_bcsr(brows, bs, k, pos.ctypes.data, crd.ctypes.data, vals.ctypes.data, B.ctypes.data,
                            ldb, C.ctypes.data, mag.ctypes.data, sp, ns, int(threads))
    return C, mag


def mttkrp_csf3(pos_k, crd_k, pos_l, crd_l, vals, C, D, sel=None, threads: int = 1):
    """A(s, j) = sum over the fibers and leaves of slice s of vals * C[k, j] * D[l, j]; returns (A, mag)
    with one row per slice (or per selected slice)."""
    pos_k, crd_k, pos_l, crd_l, vals = _i32(pos_k), _i32(crd_k), _i32(pos_l), _i32(crd_l), _f32(vals)
    C = np.asarray(C, dtype=np.float32)
    D = np.asarray(D, dtype=np.float32)
    if C.ndim != 2 or C.strides[1] != 4:
        C = np.ascontiguousarray(C)
    if D.ndim != 2 or D.strides[1] != 4:
        D = np.ascontiguousarray(D)
    j = C.shape[1]
    assert D.shape[1] == j
    nslices = pos_k.size - 1
    keep, sp, ns = _sel(sel)
    n = ns if keep is not None else nslices
    A = np.empty((n, j), dtype=np.float64)
    mag = np.empty((n, j), dtype=np.float64)
    _lib().oracle_mttkrp_csf3(nslices, j, pos_k.ctypes.data, crd_k.ctypes.data, pos_l.ctypes.data, crd_l.ctypes.data,
                              vals.ctypes.data, C.ctypes.data, C.strides[0] // 4, D.ctypes.data, D.strides[0] // 4,
                              A.ctypes.data, mag.ctypes.data, sp, ns, int(threads))
    return A, mag


def partition_csf3(pos_k, pos_l, tile: int):
    """Leaf-level position cut of a three-level hierarchy: (tile_slice, tile_fiber), num_tiles+1 entries each."""
    pos_k, pos_l = _i32(pos_k), _i32(pos_l)
    nslices, nfibers, nnz = pos_k.size - 1, pos_l.size - 1, int(pos_l[-1])
    nt = num_tiles(nnz, tile)
    ts = np.empty(nt + 1, dtype=np.int32)
    tf = np.empty(nt + 1, dtype=np.int32)
    _lib().oracle_partition_csf3(nslices, nfibers, nnz, pos_k.ctypes.data, pos_l.ctypes.data, int(tile),
                                 ts.ctypes.data, tf.ctypes.data)
    return ts, tf


def num_tiles(nnz: int, tile: int) -> int:
    return int(_lib().oracle_num_tiles(int(nnz), int(tile)))


def partition(pos, tile: int):
    """Position cut: int32 array of num_tiles+1 row indices."""
    pos = _i32(pos)
    rows = pos.size - 1
    nnz = int(pos[-1])
    out = np.empty(num_tiles(nnz, tile) + 1, dtype=np.int32)
    _lib().oracle_partition(rows, nnz, pos.ctypes.data, int(tile), out.ctypes.data)
    return out


def validate_csr(pos, crd, cols: int) -> int:
    pos, crd = _i32(pos), _i32(crd)
    return int(_lib().oracle_validate_csr(pos.size - 1, int(cols), int(crd.size), pos.ctypes.data,
                                          crd.ctypes.data))


def within_tolerance(got, ref, mag, rel: float = 1e-5, floor: float = 1e-30):
    """The acceptance test for fp32 results: |got - ref| <= rel*mag + floor, elementwise.
    Returns (ok, worst_ratio) where worst_ratio = max |got-ref| / (rel*mag+floor)."""
    got = np.asarray(got, dtype=np.float64)
    bound = rel * np.asarray(mag, dtype=np.float64) + floor
    err = np.abs(got - np.asarray(ref, dtype=np.float64))
    bad = ~(err <= bound)  # NaN counts as failure
    worst = float(np.max(err / bound)) if err.size else 0.0
    return (not bool(bad.any())), worst


class Slab:
    """The column-slab hierarchy of a CSR matrix (see oracle.c): arrays svals, scol (uint16), srow, chunk_pair,
    slab_chunk, qpos, qidx and the sizes nslots, npairs, nq, nslabs."""


def slab_build(rows: int, cols: int, pos, crd, vals, W: int = 32736, CH: int = 512, f64: bool = False) -> Slab:
    """fp32 values by default; f64=True keeps the values as doubles (the structure is the same, the values'
    storage order inside a chunk follows the 8-byte rule)."""
    pos, crd = _i32(pos), _i32(crd)
    vals = np.ascontiguousarray(vals, dtype=np.float64) if f64 else _f32(vals)
    nnz = int(crd.size)
    sizes = np.zeros(4, dtype=np.int64)
    if _lib().oracle_slab_count(rows, cols, nnz, pos.ctypes.data, crd.ctypes.data, W, CH, sizes.ctypes.data) != 0:
        raise MemoryError("oracle_slab_count")
    S = Slab()
    S.rows, S.cols, S.nnz, S.W, S.CH = rows, cols, nnz, W, CH
    S.nslots, S.npairs, S.nq, S.nslabs = (int(v) for v in sizes)
    S.f64 = bool(f64)
    S.svals = np.empty(S.nslots, dtype=np.float64 if f64 else np.float32)
    S.scol = np.empty(S.nslots, dtype=np.uint16)
    S.srow = np.empty(S.nslots, dtype=np.int32)
    S.chunk_pair = np.empty(S.nslots // CH + 1, dtype=np.int32)
    S.slab_chunk = np.empty(S.nslabs + 1, dtype=np.int32)
    S.qpos = np.empty(rows + 1, dtype=np.int32)
    S.qidx = np.empty(S.nq, dtype=np.int32)
    build = _lib().oracle_slab_build_f64 if f64 else _lib().oracle_slab_build
    if build(rows, cols, nnz, pos.ctypes.data, crd.ctypes.data, vals.ctypes.data, W, CH, S.svals.ctypes.data,
             S.scol.ctypes.data, S.srow.ctypes.data, S.chunk_pair.ctypes.data, S.slab_chunk.ctypes.data,
             S.qpos.ctypes.data, S.qidx.ctypes.data) != 0:
        raise MemoryError("oracle_slab_build")
    return S


def spmv_slab(S: Slab, x):
    """y and mag (float64, one per row) evaluated over the slab structure: P per pair, then the pairs of each row."""
    if getattr(S, "f64", False):
        x = np.ascontiguousarray(x, dtype=np.float64)
        y = np.empty(S.rows, dtype=np.float64)
        mag = np.empty(S.rows, dtype=np.float64)
        if _lib().oracle_spmv_slab_f64(S.rows, S.cols, S.npairs, S.W, S.CH, S.svals.ctypes.data, S.scol.ctypes.data,
                                       S.slab_chunk.ctypes.data, S.qpos.ctypes.data, S.qidx.ctypes.data,
                                       x.ctypes.data, y.ctypes.data, mag.ctypes.data) != 0:
            raise MemoryError("oracle_spmv_slab_f64")
        return y, mag
    x = _f32(x)
    P = np.empty(max(S.npairs, 1), dtype=np.float64)
    Pm = np.empty(max(S.npairs, 1), dtype=np.float64)
    y = np.empty(S.rows, dtype=np.float64)
    mag = np.empty(S.rows, dtype=np.float64)
    _lib().oracle_spmv_slab(S.rows, S.cols, S.nslots, S.W, S.CH, S.svals.ctypes.data, S.scol.ctypes.data,
                            S.slab_chunk.ctypes.data, S.qpos.ctypes.data, S.qidx.ctypes.data, x.ctypes.data,
                            P.ctypes.data, Pm.ctypes.data, y.ctypes.data, mag.ctypes.data)
    return y, mag
