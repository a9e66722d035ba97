"""Thin ctypes binding of libpsk.so: argument marshalling only.

Function names match include/psk.h.  Tensors are torch CUDA tensors (device memory and streams are
PyTorch's only role); every computation happens inside the library's kernels.  There is no CPU
fallback: a missing library raises at import of this module's first use.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpsk.so")
TRACE_LIB_PATH = os.path.join(_HERE, "libpsk_trace.so")

PSK_OK = 0
PSK_OP_SPMV_CSR, PSK_OP_SPMM_CSR, PSK_OP_SPMV_BCSR, PSK_OP_SPMM_BCSR, PSK_OP_MTTKRP_CSF3 = 0, 1, 2, 3, 4
PSK_OP_SPMV_CSR_F64 = 5
PSK_CUT_POSITIONS, PSK_CUT_ROWS = 0, 1
PSK_SCHEDULE_POSITIONS, PSK_SCHEDULE_ROWS = 0, 1
PSK_PHASE_PARTITION, PSK_PHASE_MAIN, PSK_PHASE_FIXUP, PSK_PHASE_ALL = 1, 2, 4, 7
PSK_ROWSPLIT_THREAD_PER_ROW, PSK_ROWSPLIT_WAVE_PER_ROW = 0, 1

EXPORTS = [
    "psk_status_string", "psk_version", "psk_default_tile", "psk_num_tiles", "psk_workspace_bytes",
    "psk_partition_csr", "psk_analyze_csr", "psk_spmv_csr", "psk_spmm_csr", "psk_spmv_bcsr", "psk_spmm_bcsr",
    "psk_spmv_csr_rowsplit", "psk_spmm_csr_rowsplit", "psk_spmv_csr_atomics", "psk_mttkrp_csf3",
    "psk_partition_csf3", "psk_spmv_csr_notemp", "psk_spmv_csr_f64", "psk_spmv_dcsr", "psk_spmv_csr_divide", "psk_suggest_schedule_csr", "psk_default_tile_bcsr", "psk_validate_csr",
    "psk_spmv_csr_static", "psk_static_scratch_bytes",
    "psk_slab_mem_bytes", "psk_slab_build_workspace_bytes", "psk_slab_spmv_workspace_bytes", "psk_slab_build_csr",
    "psk_spmv_slab", "psk_slab_mem_bytes_f64", "psk_slab_build_workspace_bytes_f64", "psk_slab_build_csr_f64",
    "psk_spmv_slab_f64", "psk_cu_trace_set", "psk_calibrate_stream_read", "psk_calibrate_gather", "psk_calibrate_gather_lds",
]


PSK_SLAB_COLS, PSK_SLAB_CHUNK = 32736, 512


class psk_slab(ctypes.Structure):
    """Mirror of the C struct psk_slab (host memory; the pointers are device addresses)."""
    _fields_ = [(n, ctypes.c_int64) for n in ("rows", "cols", "nnz", "nslabs", "nslots", "nchunks", "npairs", "nq")] + \
               [(n, ctypes.c_int32) for n in ("slab_cols", "chunk", "tile", "value_bytes")] + \
               [(n, ctypes.c_void_p) for n in ("svals", "scol", "chunk_pair", "slab_chunk", "qpos", "qidx", "qtile_row")]


class PskError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__("%s failed: status %d (%s)" % (what, status, status_string(status)))
        self.status = status


_lib = None
_lib_path = LIB_PATH


def use_instrumented_library() -> None:
    """Selects libpsk_trace.so (the build with per-workgroup records, see psk_cu_trace_set) instead of libpsk.so.
    Must be called before the first operation of the process."""
    global _lib_path
    if _lib is not None:
        raise RuntimeError("the library is already loaded")
    _lib_path = TRACE_LIB_PATH


def lib() -> ctypes.CDLL:
    """The loaded library.  Raises if it has not been built (python -m paper_2001_00532_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_lib_path):
            raise RuntimeError("%s is not built; run `python -m paper_2001_00532_amd.build`" % os.path.basename(_lib_path))
        L = ctypes.CDLL(_lib_path)
        i64, i32, p, ci, sz = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        L.psk_status_string.argtypes, L.psk_status_string.restype = [ci], ctypes.c_char_p
        L.psk_version.argtypes, L.psk_version.restype = [], ci
        L.psk_default_tile.argtypes, L.psk_default_tile.restype = [ci], i32
        L.psk_num_tiles.argtypes, L.psk_num_tiles.restype = [i64, i32], i64
        L.psk_workspace_bytes.argtypes, L.psk_workspace_bytes.restype = [ci, i64, i64, i32, i32, i32], sz
        L.psk_partition_csr.argtypes, L.psk_partition_csr.restype = [i64, i64, p, i32, ci, p, p], ci
        L.psk_analyze_csr.argtypes = [i64, i64, i64, p, p, p, sz, ctypes.POINTER(i32), p]
        L.psk_analyze_csr.restype = ci
        L.psk_spmv_csr.argtypes = [i64, i64, i64, p, p, p, p, p, i32, i32, ci, p, sz, p]
        L.psk_spmv_csr.restype = ci
        L.psk_spmv_csr_static.argtypes = [i64, i64, i64, p, p, p, p, p, i32, i32, p]
        L.psk_spmv_csr_static.restype = ci
        L.psk_static_scratch_bytes.argtypes, L.psk_static_scratch_bytes.restype = [], sz
        L.psk_slab_mem_bytes.argtypes, L.psk_slab_mem_bytes.restype = [i64, i64, i64], sz
        L.psk_slab_build_workspace_bytes.argtypes, L.psk_slab_build_workspace_bytes.restype = [i64, i64, i64], sz
        L.psk_slab_spmv_workspace_bytes.argtypes = [ctypes.POINTER(psk_slab)]
        L.psk_slab_spmv_workspace_bytes.restype = sz
        L.psk_slab_build_csr.argtypes = [i64, i64, i64, p, p, p, p, sz, p, sz, ctypes.POINTER(psk_slab), p]
        L.psk_slab_build_csr.restype = ci
        L.psk_spmv_slab.argtypes = [ctypes.POINTER(psk_slab), p, p, ci, p, sz, p]
        L.psk_spmv_slab.restype = ci
        L.psk_slab_mem_bytes_f64.argtypes, L.psk_slab_mem_bytes_f64.restype = [i64, i64, i64], sz
        L.psk_slab_build_workspace_bytes_f64.argtypes, L.psk_slab_build_workspace_bytes_f64.restype = [i64, i64, i64], sz
        L.psk_slab_build_csr_f64.argtypes = [i64, i64, i64, p, p, p, p, sz, p, sz, ctypes.POINTER(psk_slab), p]
        L.psk_slab_build_csr_f64.restype = ci
        L.psk_spmv_slab_f64.argtypes = [ctypes.POINTER(psk_slab), p, p, ci, p, sz, p]
        L.psk_spmv_slab_f64.restype = ci
        L.psk_cu_trace_set.argtypes, L.psk_cu_trace_set.restype = [p, sz], ci
        L.psk_calibrate_stream_read.argtypes, L.psk_calibrate_stream_read.restype = [p, sz, p, p], ci
        L.psk_calibrate_gather.argtypes, L.psk_calibrate_gather.restype = [p, i64, p, i64, p, p], ci
        L.psk_calibrate_gather_lds.argtypes, L.psk_calibrate_gather_lds.restype = [p, i32, p, i64, p, p], ci
        L.psk_spmm_csr.argtypes = [i64, i64, i64, p, p, p, p, i32, i64, p, i64, i32, ci, p, sz, p]
        L.psk_spmm_csr.restype = ci
        L.psk_spmv_bcsr.argtypes = [i64, i64, i64, i32, p, p, p, p, p, i32, ci, p, sz, p]
        L.psk_spmv_bcsr.restype = ci
        L.psk_spmm_bcsr.argtypes = [i64, i64, i64, i32, p, p, p, p, i32, i64, p, i64, i32, ci, p, sz, p]
        L.psk_spmm_bcsr.restype = ci
        L.psk_partition_csf3.argtypes = [i64, i64, i64, p, p, i32, p, p, p]
        L.psk_partition_csf3.restype = ci
        L.psk_mttkrp_csf3.argtypes = [i64, i64, i64, i64, i64, i64, p, p, p, p, p, p, p, i64, p, i64, i32, p, i64, i32,
                                      ci, p, sz, p]
        L.psk_mttkrp_csf3.restype = ci
        L.psk_spmv_csr_atomics.argtypes = [i64, i64, i64, p, p, p, p, p, i32, ci, p, sz, p]
        L.psk_spmv_csr_atomics.restype = ci
        L.psk_spmv_csr_notemp.argtypes = [i64, i64, i64, p, p, p, p, p, i32, ci, p, sz, p]
        L.psk_spmv_csr_notemp.restype = ci
        L.psk_spmv_csr_f64.argtypes = [i64, i64, i64, p, p, p, p, p, i32, i32, ci, p, sz, p]
        L.psk_spmv_csr_f64.restype = ci
        L.psk_spmv_dcsr.argtypes = [i64, i64, i64, i64, p, p, p, p, p, p, ci, i32, i32, ci, p, sz, p]
        L.psk_spmv_dcsr.restype = ci
        L.psk_default_tile_bcsr.argtypes = [ci, i32]
        L.psk_default_tile_bcsr.restype = i32
        L.psk_suggest_schedule_csr.argtypes = [i64, i64, p, p, sz, p, p]
        L.psk_suggest_schedule_csr.restype = ci
        L.psk_validate_csr.argtypes = [i64, i64, i64, p, p, p, sz, p, p]
        L.psk_validate_csr.restype = ci
        L.psk_spmv_csr_divide.argtypes = [i64, i64, i64, p, p, p, p, p, i32, ci, p, sz, p]
        L.psk_spmv_csr_divide.restype = ci
        L.psk_spmv_csr_rowsplit.argtypes = [i64, i64, i64, p, p, p, p, p, ci, p]
        L.psk_spmv_csr_rowsplit.restype = ci
        L.psk_spmm_csr_rowsplit.argtypes = [i64, i64, i64, p, p, p, p, i32, i64, p, i64, p]
        L.psk_spmm_csr_rowsplit.restype = ci
        _lib = L
    return _lib


def _ptr(t, dtype=None):
    """Device pointer of a tensor (None -> NULL).  Checks device, dtype and contiguity of the last dim."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("expected a device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError("expected dtype %s, got %s" % (dtype, t.dtype))
    if t.numel() and t.stride(-1) != 1:
        raise ValueError("innermost dimension must be contiguous")
    return ctypes.c_void_p(t.data_ptr()) if t.numel() else ctypes.c_void_p(t.data_ptr() or 0)


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _temporary_ws_ok(phases: int, what: str):
    """A workspace made for one call holds no table: the main and fix-up steps on their own would read garbage
    row numbers (and run out of bounds), so a partial product must bring the workspace the table was built in."""
    if int(phases) & PSK_PHASE_PARTITION == 0:
        raise ValueError("%s: phases without PSK_PHASE_PARTITION need the workspace (ws=...) that holds the table" % what)


def _check(status: int, what: str):
    if status != PSK_OK:
        raise PskError(status, what)


def status_string(status: int) -> str:
    return lib().psk_status_string(int(status)).decode()


def psk_version() -> int:
    return int(lib().psk_version())


def psk_default_tile(op: int) -> int:
    return int(lib().psk_default_tile(int(op)))


def psk_default_tile_bcsr(op: int, bs: int) -> int:
    return int(lib().psk_default_tile_bcsr(int(op), int(bs)))


def psk_num_tiles(nnz: int, tile: int) -> int:
    return int(lib().psk_num_tiles(int(nnz), int(tile)))


def psk_workspace_bytes(op: int, rows: int, nnz: int, k: int = 1, bs: int = 1, tile: int = 0) -> int:
    return int(lib().psk_workspace_bytes(int(op), int(rows), int(nnz), int(k), int(bs), int(tile)))


def workspace(op: int, rows: int, nnz: int, k: int = 1, bs: int = 1, tile: int = 0, device="cuda", stream=None):
    """A byte tensor of the size the operation needs (torch allocations are 256-byte aligned).

    `stream`: the stream the kernels that use it will run on.  The block is allocated under that stream, so
    torch's caching allocator hands it out again only to work that is ordered after those kernels; a
    temporary workspace dropped right after an asynchronous call stays valid until the call has run."""
    n = psk_workspace_bytes(op, rows, nnz, k, bs, tile)
    if n == 0:
        raise ValueError("invalid arguments for psk_workspace_bytes")
    return _alloc_bytes(n, device, stream)


def _alloc_bytes(n: int, device, stream=None):
    if stream is None:
        return torch.empty(n, dtype=torch.uint8, device=device)
    with torch.cuda.stream(stream):
        return torch.empty(n, dtype=torch.uint8, device=device)


PSK_PARTITION_AUTO, PSK_PARTITION_SEARCH, PSK_PARTITION_SCAN = 0, 1, 2


def psk_partition_csr(pos, nnz: int, tile: int, method: int = 0, tile_row=None, stream=None):
    """tile_row (int32, num_tiles+1) for the position cut of `pos` (int32 device tensor, rows+1)."""
    rows = pos.numel() - 1
    nt = max(psk_num_tiles(nnz, tile), 0)
    if tile_row is None:
        tile_row = torch.empty(nt + 1, dtype=torch.int32, device=pos.device)
    st = lib().psk_partition_csr(rows, int(nnz), _ptr(pos, torch.int32), int(tile), int(method),
                                 _ptr(tile_row, torch.int32), _stream(stream))
    _check(st, "psk_partition_csr")
    return tile_row


def psk_analyze_csr(rows, cols, nnz, pos, crd, ws=None, stream=None) -> int:
    """Suggested col_passes for psk_spmv_csr (synchronises the stream)."""
    if ws is None:
        ws = _alloc_bytes(256, pos.device, stream)
    out = ctypes.c_int32(0)
    st = lib().psk_analyze_csr(int(rows), int(cols), int(nnz), _ptr(pos, torch.int32), _ptr(crd, torch.int32),
                               _ptr(ws), ws.numel(), ctypes.byref(out), _stream(stream))
    _check(st, "psk_analyze_csr")
    return int(out.value)


def psk_validate_csr(rows, cols, nnz, pos, crd, ws=None, stream=None) -> int:
    """0 if the index structure is well formed, else the number (1..4) of the first failing condition
    (synchronises the stream)."""
    if ws is None:
        ws = _alloc_bytes(256, pos.device, stream)
    out = ctypes.c_int32(-1)
    st = lib().psk_validate_csr(int(rows), int(cols), int(nnz), _ptr(pos, torch.int32), _ptr(crd, torch.int32),
                                _ptr(ws), ws.numel(), ctypes.byref(out), _stream(stream))
    _check(st, "psk_validate_csr")
    return int(out.value)


def psk_suggest_schedule_csr(rows, nnz, pos, ws=None, stream=None) -> int:
    """PSK_SCHEDULE_POSITIONS or PSK_SCHEDULE_ROWS for y = A x on this matrix (may synchronise the stream)."""
    if ws is None:
        ws = _alloc_bytes(256, pos.device, stream)
    out = ctypes.c_int32(-1)
    st = lib().psk_suggest_schedule_csr(int(rows), int(nnz), _ptr(pos, torch.int32), _ptr(ws), ws.numel(),
                                        ctypes.byref(out), _stream(stream))
    _check(st, "psk_suggest_schedule_csr")
    return int(out.value)


def psk_spmv_csr(rows, cols, nnz, pos, crd, vals, x, y, tile=0, col_passes=1, phases=PSK_PHASE_ALL, ws=None,
                 stream=None):
    if ws is None:
        _temporary_ws_ok(phases, "psk_spmv_csr")
        ws = workspace(PSK_OP_SPMV_CSR, rows, nnz, tile=tile, device=pos.device, stream=stream)
    st = lib().psk_spmv_csr(int(rows), int(cols), int(nnz), _ptr(pos, torch.int32), _ptr(crd, torch.int32),
                            _ptr(vals, torch.float32), _ptr(x, torch.float32), _ptr(y, torch.float32), int(tile),
                            int(col_passes), int(phases), _ptr(ws), ws.numel(), _stream(stream))
    _check(st, "psk_spmv_csr")
    return y


def psk_static_scratch_bytes() -> int:
    return int(lib().psk_static_scratch_bytes())


def psk_spmv_csr_static(rows, cols, nnz, pos, crd, vals, x, y, tile=0, col_passes=1, stream=None):
    """psk_spmv_csr without a workspace: the library's built-in scratch array is used; nothing is allocated."""
    st = lib().psk_spmv_csr_static(int(rows), int(cols), int(nnz), _ptr(pos, torch.int32), _ptr(crd, torch.int32),
                                   _ptr(vals, torch.float32), _ptr(x, torch.float32), _ptr(y, torch.float32),
                                   int(tile), int(col_passes), _stream(stream))
    _check(st, "psk_spmv_csr_static")
    return y


class PreparedCall:
    """A call whose arguments are already marshalled: calling it only crosses into the library.  For loops that
    repeat one product on the same buffers and are bound by the host side of the call (small matrices)."""

    def __init__(self, fn, what, cargs, keep):
        self._fn, self._what, self._cargs, self._keep = fn, what, cargs, keep      # `keep` holds the tensors alive

    def __call__(self):
        st = self._fn(*self._cargs)
        if st != PSK_OK:
            raise PskError(st, self._what)


def psk_spmv_csr_prepared(rows, cols, nnz, pos, crd, vals, x, y, tile=0, col_passes=1, phases=PSK_PHASE_ALL, ws=None,
                          stream=None) -> PreparedCall:
    """psk_spmv_csr with the marshalling done once; the returned object repeats the call."""
    if ws is None:
        ws = workspace(PSK_OP_SPMV_CSR, rows, nnz, tile=tile, device=pos.device, stream=stream)
    cargs = (int(rows), int(cols), int(nnz), _ptr(pos, torch.int32), _ptr(crd, torch.int32), _ptr(vals, torch.float32),
             _ptr(x, torch.float32), _ptr(y, torch.float32), int(tile), int(col_passes), int(phases), _ptr(ws), ws.numel(),
             _stream(stream))
    return PreparedCall(lib().psk_spmv_csr, "psk_spmv_csr", cargs, (pos, crd, vals, x, y, ws, stream))


def psk_spmm_csr(rows, cols, nnz, pos, crd, vals, B, C, tile=0, phases=PSK_PHASE_ALL, ws=None, stream=None):
    k = B.shape[1]
    if ws is None:
        _temporary_ws_ok(phases, "psk_spmm_csr")
        ws = workspace(PSK_OP_SPMM_CSR, rows, nnz, k=k, tile=tile, device=pos.device, stream=stream)
    st = lib().psk_spmm_csr(int(rows), int(cols), int(nnz), _ptr(pos, torch.int32), _ptr(crd, torch.int32),
                            _ptr(vals, torch.float32), _ptr(B, torch.float32), int(k), int(B.stride(0)),
                            _ptr(C, torch.float32), int(C.stride(0)), int(tile), int(phases), _ptr(ws),
                            ws.numel(), _stream(stream))
    _check(st, "psk_spmm_csr")
    return C


def psk_spmv_bcsr(brows, bcols, nblocks, bs, pos, crd, vals, x, y, tile=0, phases=PSK_PHASE_ALL, ws=None,
                  stream=None):
    if ws is None:
        _temporary_ws_ok(phases, "psk_spmv_bcsr")
        ws = workspace(PSK_OP_SPMV_BCSR, brows, nblocks, bs=bs, tile=tile, device=pos.device, stream=stream)
    st = lib().psk_spmv_bcsr(int(brows), int(bcols), int(nblocks), int(bs), _ptr(pos, torch.int32),
                             _ptr(crd, torch.int32), _ptr(vals, torch.float32), _ptr(x, torch.float32),
                             _ptr(y, torch.float32), int(tile), int(phases), _ptr(ws), ws.numel(), _stream(stream))
    _check(st, "psk_spmv_bcsr")
    return y


def psk_spmm_bcsr(brows, bcols, nblocks, bs, pos, crd, vals, B, C, tile=0, phases=PSK_PHASE_ALL, ws=None,
                  stream=None):
    k = B.shape[1]
    if ws is None:
        _temporary_ws_ok(phases, "psk_spmm_bcsr")
        ws = workspace(PSK_OP_SPMM_BCSR, brows, nblocks, k=k, bs=bs, tile=tile, device=pos.device, stream=stream)
    st = lib().psk_spmm_bcsr(int(brows), int(bcols), int(nblocks), int(bs), _ptr(pos, torch.int32),
                             _ptr(crd, torch.int32), _ptr(vals, torch.float32), _ptr(B, torch.float32), int(k),
                             int(B.stride(0)), _ptr(C, torch.float32), int(C.stride(0)), int(tile), int(phases),
                             _ptr(ws), ws.numel(), _stream(stream))
    _check(st, "psk_spmm_bcsr")
    return C


def psk_partition_csf3(pos_k, pos_l, nnz: int, tile: int, stream=None):
    """(tile_slice, tile_fiber), each int32 with num_tiles+1 entries."""
    nslices, nfibers = pos_k.numel() - 1, pos_l.numel() - 1
    nt = max(psk_num_tiles(nnz, tile), 0)
    ts = torch.empty(nt + 1, dtype=torch.int32, device=pos_k.device)
    tf = torch.empty(nt + 1, dtype=torch.int32, device=pos_k.device)
    st = lib().psk_partition_csf3(nslices, nfibers, int(nnz), _ptr(pos_k, torch.int32), _ptr(pos_l, torch.int32),
                                  int(tile), _ptr(ts, torch.int32), _ptr(tf, torch.int32), _stream(stream))
    _check(st, "psk_partition_csf3")
    return ts, tf


def psk_mttkrp_csf3(dims, crd_i, pos_k, crd_k, pos_l, crd_l, vals, C, D, A, tile=0, phases=PSK_PHASE_ALL, ws=None,
                    stream=None):
    """A (dims[0] x j) = MTTKRP of the three-level tensor with C (dims[1] x j) and D (dims[2] x j)."""
    nslices, nfibers, nnz, j = pos_k.numel() - 1, pos_l.numel() - 1, crd_l.numel(), C.shape[1]
    if ws is None:
        _temporary_ws_ok(phases, "psk_mttkrp_csf3")
        ws = workspace(PSK_OP_MTTKRP_CSF3, nslices, nnz, k=j, tile=tile, device=pos_k.device, stream=stream)
    st = lib().psk_mttkrp_csf3(int(dims[0]), int(dims[1]), int(dims[2]), nslices, nfibers, nnz,
                               _ptr(crd_i, torch.int32), _ptr(pos_k, torch.int32), _ptr(crd_k, torch.int32),
                               _ptr(pos_l, torch.int32), _ptr(crd_l, torch.int32), _ptr(vals, torch.float32),
                               _ptr(C, torch.float32), int(C.stride(0)), _ptr(D, torch.float32), int(D.stride(0)),
                               int(j), _ptr(A, torch.float32), int(A.stride(0)), int(tile), int(phases), _ptr(ws),
                               ws.numel(), _stream(stream))
    _check(st, "psk_mttkrp_csf3")
    return A


def psk_spmv_csr_atomics(rows, cols, nnz, pos, crd, vals, x, y, tile=0, phases=PSK_PHASE_ALL, ws=None, stream=None):
    if ws is None:
        _temporary_ws_ok(phases, "psk_spmv_csr_atomics")
        ws = workspace(PSK_OP_SPMV_CSR, rows, nnz, tile=tile, device=pos.device, stream=stream)
    st = lib().psk_spmv_csr_atomics(int(rows), int(cols), int(nnz), _ptr(pos, torch.int32), _ptr(crd, torch.int32),
                                    _ptr(vals, torch.float32), _ptr(x, torch.float32), _ptr(y, torch.float32),
                                    int(tile), int(phases), _ptr(ws), ws.numel(), _stream(stream))
    _check(st, "psk_spmv_csr_atomics")
    return y


def psk_spmv_csr_f64(rows, cols, nnz, pos, crd, vals, x, y, tile=0, col_passes=1, phases=PSK_PHASE_ALL, ws=None,
                     stream=None):
    if ws is None:
        _temporary_ws_ok(phases, "psk_spmv_csr_f64")
        ws = workspace(PSK_OP_SPMV_CSR_F64, rows, nnz, tile=tile, device=pos.device, stream=stream)
    st = lib().psk_spmv_csr_f64(int(rows), int(cols), int(nnz), _ptr(pos, torch.int32), _ptr(crd, torch.int32),
                                _ptr(vals, torch.float64), _ptr(x, torch.float64), _ptr(y, torch.float64),
                                int(tile), int(col_passes), int(phases), _ptr(ws), ws.numel(), _stream(stream))
    _check(st, "psk_spmv_csr_f64")
    return y


def psk_spmv_dcsr(rows, cols, nnz, crd_i, pos, crd, vals, x, y, cut=PSK_CUT_POSITIONS, tile=0, col_passes=1,
                  phases=PSK_PHASE_ALL, ws=None, stream=None):
    nstored = int(crd_i.numel())
    if ws is None and cut == PSK_CUT_POSITIONS:
        _temporary_ws_ok(phases, "psk_spmv_dcsr")
    if ws is None:
        ws = workspace(PSK_OP_SPMV_CSR, nstored, nnz, tile=tile, device=pos.device, stream=stream)
    st = lib().psk_spmv_dcsr(int(rows), int(cols), nstored, int(nnz), _ptr(crd_i, torch.int32), _ptr(pos, torch.int32),
                             _ptr(crd, torch.int32), _ptr(vals, torch.float32), _ptr(x, torch.float32),
                             _ptr(y, torch.float32), int(cut), int(tile), int(col_passes), int(phases), _ptr(ws),
                             ws.numel(), _stream(stream))
    _check(st, "psk_spmv_dcsr")
    return y


def psk_spmv_csr_divide(rows, cols, nnz, pos, crd, vals, x, y, parts=0, phases=PSK_PHASE_ALL, ws=None, stream=None):
    if ws is None:
        if int(phases) & 6 != 6:      # no table here, but main and fix-up share the carry records
            raise ValueError("psk_spmv_csr_divide: main and fix-up on their own need a workspace that outlives the call")
        ws = workspace(PSK_OP_SPMV_CSR, rows, nnz, tile=2048, device=pos.device, stream=stream)
    st = lib().psk_spmv_csr_divide(int(rows), int(cols), int(nnz), _ptr(pos, torch.int32), _ptr(crd, torch.int32),
                                   _ptr(vals, torch.float32), _ptr(x, torch.float32), _ptr(y, torch.float32),
                                   int(parts), int(phases), _ptr(ws), ws.numel(), _stream(stream))
    _check(st, "psk_spmv_csr_divide")
    return y


def psk_spmv_csr_notemp(rows, cols, nnz, pos, crd, vals, x, y, tile=0, phases=PSK_PHASE_ALL, ws=None, stream=None):
    if ws is None:
        _temporary_ws_ok(phases, "psk_spmv_csr_notemp")
        ws = workspace(PSK_OP_SPMV_CSR, rows, nnz, tile=tile, device=pos.device, stream=stream)
    st = lib().psk_spmv_csr_notemp(int(rows), int(cols), int(nnz), _ptr(pos, torch.int32), _ptr(crd, torch.int32),
                                   _ptr(vals, torch.float32), _ptr(x, torch.float32), _ptr(y, torch.float32),
                                   int(tile), int(phases), _ptr(ws), ws.numel(), _stream(stream))
    _check(st, "psk_spmv_csr_notemp")
    return y


def psk_spmv_csr_rowsplit(rows, cols, nnz, pos, crd, vals, x, y, variant=PSK_ROWSPLIT_WAVE_PER_ROW, stream=None):
    st = lib().psk_spmv_csr_rowsplit(int(rows), int(cols), int(nnz), _ptr(pos, torch.int32), _ptr(crd, torch.int32),
                                     _ptr(vals, torch.float32), _ptr(x, torch.float32), _ptr(y, torch.float32),
                                     int(variant), _stream(stream))
    _check(st, "psk_spmv_csr_rowsplit")
    return y


def psk_spmm_csr_rowsplit(rows, cols, nnz, pos, crd, vals, B, C, stream=None):
    st = lib().psk_spmm_csr_rowsplit(int(rows), int(cols), int(nnz), _ptr(pos, torch.int32), _ptr(crd, torch.int32),
                                     _ptr(vals, torch.float32), _ptr(B, torch.float32), int(B.shape[1]),
                                     int(B.stride(0)), _ptr(C, torch.float32), int(C.stride(0)), _stream(stream))
    _check(st, "psk_spmm_csr_rowsplit")
    return C


class Slab:
    """A built column-slab structure: the C struct (`desc`) plus the device memory that holds its arrays."""

    def __init__(self, desc, mem):
        self.desc, self.mem = desc, mem

    def array(self, name):
        """Device view of one array of the structure (for inspection and tests)."""
        d = self.desc
        dtype, n = {"svals": (torch.float64 if d.value_bytes == 8 else torch.float32, d.nslots), "scol": (torch.int16, d.nslots),
                    "chunk_pair": (torch.int32, d.nchunks + 1), "slab_chunk": (torch.int32, d.nslabs + 1),
                    "qpos": (torch.int32, d.rows + 1), "qidx": (torch.int32, d.nq),
                    "qtile_row": (torch.int32, psk_num_tiles(d.nq, d.tile) + 1)}[name]
        off = int(getattr(d, name)) - self.mem.data_ptr()
        size = n * torch.empty((), dtype=dtype).element_size()
        return self.mem[off:off + size].view(dtype)


def psk_slab_mem_bytes(rows, cols, nnz) -> int:
    return int(lib().psk_slab_mem_bytes(int(rows), int(cols), int(nnz)))


def psk_slab_build_workspace_bytes(rows, cols, nnz) -> int:
    return int(lib().psk_slab_build_workspace_bytes(int(rows), int(cols), int(nnz)))


def psk_slab_build_csr(rows, cols, nnz, pos, crd, vals, mem=None, ws=None, stream=None) -> Slab:
    """Builds the column-slab structure of a CSR matrix on the device (synchronises the stream)."""
    nm, nw = psk_slab_mem_bytes(rows, cols, nnz), psk_slab_build_workspace_bytes(rows, cols, nnz)
    if nm == 0 or nw == 0:
        raise PskError(5, "psk_slab_build_csr (sizes outside the limits of the slab structure)")
    if mem is None:
        mem = _alloc_bytes(nm, pos.device, stream)
    if ws is None:
        ws = _alloc_bytes(nw, pos.device, stream)
    desc = psk_slab()
    st = lib().psk_slab_build_csr(int(rows), int(cols), int(nnz), _ptr(pos, torch.int32), _ptr(crd, torch.int32),
                                  _ptr(vals, torch.float32), _ptr(mem), mem.numel(), _ptr(ws), ws.numel(),
                                  ctypes.byref(desc), _stream(stream))
    _check(st, "psk_slab_build_csr")
    return Slab(desc, mem)


def psk_slab_mem_bytes_f64(rows, cols, nnz) -> int:
    return int(lib().psk_slab_mem_bytes_f64(int(rows), int(cols), int(nnz)))


def psk_slab_build_workspace_bytes_f64(rows, cols, nnz) -> int:
    return int(lib().psk_slab_build_workspace_bytes_f64(int(rows), int(cols), int(nnz)))


def psk_slab_build_csr_f64(rows, cols, nnz, pos, crd, vals, mem=None, ws=None, stream=None) -> Slab:
    """The structure with fp64 values (synchronises the stream)."""
    nm, nw = psk_slab_mem_bytes_f64(rows, cols, nnz), psk_slab_build_workspace_bytes_f64(rows, cols, nnz)
    if nm == 0 or nw == 0:
        raise PskError(5, "psk_slab_build_csr_f64 (sizes outside the limits of the slab structure)")
    if mem is None:
        mem = _alloc_bytes(nm, pos.device, stream)
    if ws is None:
        ws = _alloc_bytes(nw, pos.device, stream)
    desc = psk_slab()
    st = lib().psk_slab_build_csr_f64(int(rows), int(cols), int(nnz), _ptr(pos, torch.int32), _ptr(crd, torch.int32),
                                      _ptr(vals, torch.float64), _ptr(mem), mem.numel(), _ptr(ws), ws.numel(),
                                      ctypes.byref(desc), _stream(stream))
    _check(st, "psk_slab_build_csr_f64")
    return Slab(desc, mem)


def psk_spmv_slab_f64(S: Slab, x, y, phases=PSK_PHASE_ALL, ws=None, stream=None):
    if ws is None:
        if int(phases) != PSK_PHASE_ALL:
            raise ValueError("psk_spmv_slab_f64: a partial product needs the workspace (ws=...) of the earlier steps")
        ws = psk_slab_spmv_workspace(S, x.device if x is not None else y.device, stream)
    st = lib().psk_spmv_slab_f64(ctypes.byref(S.desc), _ptr(x, torch.float64), _ptr(y, torch.float64), int(phases), _ptr(ws),
                                 ws.numel(), _stream(stream))
    _check(st, "psk_spmv_slab_f64")
    return y


def psk_slab_spmv_workspace(S: Slab, device="cuda", stream=None):
    n = int(lib().psk_slab_spmv_workspace_bytes(ctypes.byref(S.desc)))
    return _alloc_bytes(max(n, 256), device, stream)


def psk_spmv_slab(S: Slab, x, y, phases=PSK_PHASE_ALL, ws=None, stream=None):
    if ws is None:
        if int(phases) != PSK_PHASE_ALL:
            raise ValueError("psk_spmv_slab: a partial product needs the workspace (ws=...) of the earlier steps")
        ws = psk_slab_spmv_workspace(S, x.device if x is not None else y.device, stream)
    st = lib().psk_spmv_slab(ctypes.byref(S.desc), _ptr(x, torch.float32), _ptr(y, torch.float32), int(phases), _ptr(ws), ws.numel(),
                             _stream(stream))
    _check(st, "psk_spmv_slab")
    return y


def psk_calibrate_stream_read(src, sink, stream=None):
    st = lib().psk_calibrate_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink, torch.float32), _stream(stream))
    _check(st, "psk_calibrate_stream_read")


def psk_calibrate_gather(table, idx, out, stream=None):
    st = lib().psk_calibrate_gather(_ptr(table, torch.float32), table.numel(), _ptr(idx, torch.int32), idx.numel(),
                                    _ptr(out, torch.float32), _stream(stream))
    _check(st, "psk_calibrate_gather")


def psk_calibrate_gather_lds(table, idx, out, stream=None):
    st = lib().psk_calibrate_gather_lds(_ptr(table, torch.float32), table.numel(), _ptr(idx, torch.int16), idx.numel(),
                                        _ptr(out, torch.float32), _stream(stream))
    _check(st, "psk_calibrate_gather_lds")


def psk_cu_trace_set(records) -> None:
    """records: int64 device tensor with 3 entries per workgroup, more than 1024 records (None switches tracing off).
    Instrumented build only."""
    n = 0 if records is None else records.numel() // 3
    st = lib().psk_cu_trace_set(_ptr(records, torch.int64) if records is not None else None, n)
    _check(st, "psk_cu_trace_set")
