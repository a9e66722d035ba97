"""Do the pins bite?  Plausible mistakes are planted in a COPY of the oracle source (CPU only), the
copy is compiled, and the same kinds of checks the pins make must reject it.  Every mutant must be
caught; the unmodified source must pass the same checks."""
import ctypes
import json
import os
import subprocess

import numpy as np
import pytest

import oracle
import workloads as wl
from conftest import dense_of

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = open(os.path.join(os.path.dirname(HERE), "oracle", "oracle.c")).read()
GOLD = json.load(open(os.path.join(HERE, "golden", "hand_worked.json")))

# (name, text to replace, replacement) -- each occurs exactly once in oracle.c unless count is given
MUTANTS = [
    ("spmv_drops_last_term", "for (int64_t p = pos[i]; p < pos[i + 1]; ++p) {\n            double t = (double)vals[p] * (double)x[crd[p]];",
     "for (int64_t p = pos[i]; p < pos[i + 1] - 1; ++p) {\n            double t = (double)vals[p] * (double)x[crd[p]];"),
    ("spmv_wrong_sign", "            acc += t;\n            m += fabs(t);\n        }\n        y[s] = acc;", "            acc -= t;\n            m += fabs(t);\n        }\n        y[s] = acc;"),
    ("spmv_x_indexed_by_position", "(double)vals[p] * (double)x[crd[p]];", "(double)vals[p] * (double)x[p % 4];"),
    ("spmv_mag_without_abs", "            acc += t;\n            m += fabs(t);\n        }\n        y[s] = acc;", "            acc += t;\n            m += t;\n        }\n        y[s] = acc;"),
    ("spmv_float_accumulation", "        double acc = 0.0, m = 0.0;\n        for (int64_t p = pos[i]; p < pos[i + 1]; ++p) {\n            double t = (double)vals[p] * (double)x[crd[p]];",
     "        float acc = 0.0f; double m = 0.0;\n        for (int64_t p = pos[i]; p < pos[i + 1]; ++p) {\n            double t = (double)vals[p] * (double)x[crd[p]];"),
    ("spmm_b_transposed", "const float *b = B + (int64_t)crd[p] * ldb;\n            for (int64_t kk = 0; kk < k; ++kk) {\n                double t = a * (double)b[kk];",
     "const float *b = B + (int64_t)crd[p];\n            for (int64_t kk = 0; kk < k; ++kk) {\n                double t = a * (double)b[kk * ldb];"),
    ("spmm_ignores_ldb", "const float *b = B + (int64_t)crd[p] * ldb;", "const float *b = B + (int64_t)crd[p] * k;"),
    ("bcsr_block_transposed", "double t = (double)vals[(p * bs + ii) * bs + ji] * (double)x[jb * bs + ji];",
     "double t = (double)vals[(p * bs + ji) * bs + ii] * (double)x[jb * bs + ji];"),
    ("bcsr_x_offset", "(double)x[jb * bs + ji];", "(double)x[jb + ji];"),
    ("bcsr_spmm_row_of_b", "const float *b = B + (jb * bs + ji) * ldb;", "const float *b = B + (jb * bs + ii) * ldb;"),
    ("bcsr_spmm_ignores_ldb", "const float *b = B + (jb * bs + ji) * ldb;", "const float *b = B + (jb * bs + ji) * k;"),
    ("partition_strict_compare", "while (i < rows && (int64_t)pos[i + 1] <= first) ++i;", "while (i < rows && (int64_t)pos[i + 1] < first) ++i;"),
    # (removing the clamp of the last tile's first position to nnz is an equivalent mutant: the walk
    # reaches `rows` either way, so it is not listed)
    ("partition_restarts_every_tile", "    int64_t i = 0;\n    for (int64_t t = 0; t <= ntiles; ++t) {\n        int64_t first = t * tile;",
     "    int64_t i = 0;\n    for (int64_t t = 0; t <= ntiles; ++t) {\n        i = t;\n        int64_t first = t * tile;"),
    ("partition_stops_at_empty_rows", "while (i < rows && (int64_t)pos[i + 1] <= first) ++i;", "if (i < rows && (int64_t)pos[i + 1] <= first) ++i;"),
    ("num_tiles_floor", "(nnz + tile - 1) / tile", "nnz / tile"),
    ("dcsr_writes_by_stored_index", "        y[crd_i[s]] = acc;", "        y[s] = acc;"),
    ("dcsr_absent_rows_not_zeroed", "for (int64_t i = 0; i < rows; ++i) { y[i] = 0.0; if (mag) mag[i] = 0.0; }",
     "for (int64_t i = 0; i < nstored; ++i) { y[i] = 0.0; if (mag) mag[i] = 0.0; }"),
    ("mttkrp_c_indexed_by_leaf", "const float *c = C + (int64_t)crd_k[q] * ldc;", "const float *c = C + (int64_t)crd_l[pos_l[q] < pos_l[q + 1] ? pos_l[q] : 0] * ldc;"),
    ("mttkrp_d_indexed_by_fiber", "const float *d = D + (int64_t)crd_l[p] * ldd;", "const float *d = D + (int64_t)crd_k[q] * ldd;"),
    ("mttkrp_drops_last_leaf", "for (int64_t p = pos_l[q]; p < pos_l[q + 1]; ++p) {\n                const float *d", "for (int64_t p = pos_l[q]; p < pos_l[q + 1] - 1; ++p) {\n                const float *d"),
    ("mttkrp_adds_instead_of_multiplying", "double term = v * (double)c[jj] * (double)d[jj];", "double term = v * ((double)c[jj] + (double)d[jj]);"),
    ("mttkrp_ignores_ldd", "const float *d = D + (int64_t)crd_l[p] * ldd;", "const float *d = D + (int64_t)crd_l[p] * j;"),
    ("mttkrp_ignores_ldc", "const float *c = C + (int64_t)crd_k[q] * ldc;", "const float *c = C + (int64_t)crd_k[q] * j;"),
    ("partition_csf3_slice_from_position", "while (s < nslices && (int64_t)pos_k[s + 1] <= q) ++s;", "while (s < nslices && (int64_t)pos_k[s + 1] <= first) ++s;"),
    ("partition_csf3_strict", "while (q < nfibers && (int64_t)pos_l[q + 1] <= first) ++q;", "while (q < nfibers && (int64_t)pos_l[q + 1] < first) ++q;"),
    ("f64_sums_in_double", "long double acc = 0.0L, m = 0.0L;", "double acc = 0.0, m = 0.0;"),
    ("f64_x_indexed_by_position", "(long double)vals[p] * (long double)x[crd[p]];", "(long double)vals[p] * (long double)x[p % 3];"),
    ("f64_operands_read_as_float", "(long double)vals[p] * (long double)x[crd[p]];", "(long double)(float)vals[p] * (long double)x[crd[p]];"),
]


def compile_variant(tmp_path, name, text):
    c = tmp_path / (name + ".c")
    so = tmp_path / (name + ".so")
    c.write_text(text)
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", str(so), str(c), "-lm"])
    return ctypes.CDLL(str(so))


def pins_pass(lib) -> bool:
    """A condensed version of the pins, run against an arbitrary build of the oracle."""
    saved = oracle._h
    try:
        oracle._h = None
        # route oracle's wrappers to `lib` by registering signatures on it
        real_cdll = ctypes.CDLL
        ctypes.CDLL = lambda *_a, **_k: lib
        try:
            oracle._lib()
        finally:
            ctypes.CDLL = real_cdll
        g = GOLD["csr"]
        y, mag = oracle.spmv_csr(g["pos"], g["crd"], g["vals"], g["x"])
        if y.tolist() != g["y"] or mag.tolist() != g["mag"]:
            return False
        C, Cm = oracle.spmm_csr(g["pos"], g["crd"], g["vals"], np.array(g["B"], dtype=np.float32))
        if C.tolist() != g["C"] or Cm.tolist() != g["Cmag"]:
            return False
        for T, expect in g["partition"].items():
            if oracle.partition(g["pos"], int(T)).tolist() != expect:
                return False
        b = GOLD["bcsr"]
        y, mag = oracle.spmv_bcsr(b["pos"], b["crd"], b["vals"], b["x"], b["bs"])
        if y.tolist() != b["y"] or mag.tolist() != b["mag"]:
            return False
        # dense brute force, CSR and BCSR, including a B with a row stride
        A = wl.csr_from_lengths(np.random.default_rng(1).integers(0, 9, size=31), 47, seed=3)
        x = wl.dense_uniform(47, 3, wl.S_X)
        Bw = wl.dense_uniform(47 * 9, 3, wl.S_B).reshape(47, 9)
        D = dense_of(A)
        y, _ = oracle.spmv_csr(A.pos, A.crd, A.vals, x)
        if not np.allclose(y, D @ x.astype(np.float64), rtol=0, atol=1e-13):
            return False
        C, _ = oracle.spmm_csr(A.pos, A.crd, A.vals, Bw[:, :5])
        if not np.allclose(C, D @ Bw[:, :5].astype(np.float64), rtol=0, atol=1e-13):
            return False
        Ab = wl.csr_from_lengths(np.random.default_rng(2).integers(0, 5, size=17), 13, seed=4, bs=4)
        xb = wl.dense_uniform(13 * 4, 4, wl.S_X)
        Bb = wl.dense_uniform(13 * 4 * 5, 4, wl.S_B).reshape(13 * 4, 5)[:, :3]      # row stride 5, three columns
        Db = dense_of(Ab)
        yb, _ = oracle.spmv_bcsr(Ab.pos, Ab.crd, Ab.vals, xb, 4)
        Cb, _ = oracle.spmm_bcsr(Ab.pos, Ab.crd, Ab.vals, Bb, 4)
        if not (np.allclose(yb, Db @ xb.astype(np.float64), rtol=0, atol=1e-13)
                and np.allclose(Cb, Db @ Bb.astype(np.float64), rtol=0, atol=1e-13)):
            return False
        # fp64 accumulation: 1 + 2^-30 + ... is lost in fp32
        pos = np.array([0, 3], dtype=np.int32)
        y, _ = oracle.spmv_csr(pos, np.array([0, 1, 2], np.int32), np.array([1.0, 2.0 ** -30, -1.0], np.float32),
                               np.ones(3, np.float32))
        if y[0] != 2.0 ** -30:
            return False
        # fp64 operands: cancellation that needs more than a double sum, exact rationals on a small case
        y, _ = oracle.spmv_csr_f64(pos, np.array([0, 1, 2], np.int32), np.array([2.0 ** 60, 1.0, -(2.0 ** 60)]), np.ones(3))
        if y[0] != 1.0:
            return False
        from fractions import Fraction
        v64 = wl.dense_uniform_f64(A.nnz, 9, wl.S_VALS)
        x64 = wl.dense_uniform_f64(47, 9, wl.S_X)
        y64, _ = oracle.spmv_csr_f64(A.pos, A.crd, v64, x64)
        for i in range(A.rows):
            ex = sum((Fraction(float(v64[q])) * Fraction(float(x64[A.crd[q]])) for q in range(A.pos[i], A.pos[i + 1])),
                     Fraction(0))
            if abs(Fraction(float(y64[i])) - ex) > Fraction(1, 2 ** 50):
                return False
        # DCSR: hand-worked case (rows 1 and 4 of a 6 x 3 matrix), output buffers pre-filled with garbage
        real_empty = np.empty
        np.empty = lambda *a, **k: np.full(*a, 7.5, **k) if k.get("dtype") == np.float64 else real_empty(*a, **k)
        try:
            y, mag = oracle.spmv_dcsr(6, [1, 4], [0, 2, 3], [0, 2, 1], [2.0, -1.0, 3.0], [1.0, 2.0, 3.0])
        finally:
            np.empty = real_empty
        if y.tolist() != [0.0, -1.0, 0.0, 0.0, 6.0, 0.0] or mag.tolist() != [0.0, 5.0, 0.0, 0.0, 6.0, 0.0]:
            return False
        # MTTKRP: hand-worked case, a strided D, and the two-level cut against brute force
        Cm = np.array([[1.0, 10.0, 7.0], [2.0, 20.0, 7.0]], dtype=np.float32)[:, :2]      # row stride 3
        Dm = np.array([[1.0, 1.0, 9.0], [0.5, 2.0, 9.0], [3.0, -1.0, 9.0]], dtype=np.float32)[:, :2]
        Am, Mm = oracle.mttkrp_csf3([0, 2], [1, 0], [0, 2, 3], [0, 2, 1], [2.0, -1.0, 4.0], Cm, Dm)
        if Am.tolist() != [[0.0, 140.0]] or Mm.tolist() != [[12.0, 140.0]]:
            return False
        Tt = wl.csf3_from_lengths([2, 0, 3, 1], [2, 0, 3, 1, 1, 4], (4, 5, 6), seed=8)
        for tile in (1, 2, 3):
            ts, tf = oracle.partition_csf3(Tt.pos_k, Tt.pos_l, tile)
            nt = -(-Tt.nnz // tile)
            for t in range(nt + 1):
                first = min(t * tile, Tt.nnz)
                qq = max(q for q in range(Tt.nfibers + 1) if Tt.pos_l[q] <= first)
                ss = max(z for z in range(Tt.nslices + 1) if Tt.pos_k[z] <= qq)
                if (tf[t], ts[t]) != (qq, ss):
                    return False
        # partition: closed form, last-tile clamp, empty rows
        p = (np.arange(51) * 7).astype(np.int32)
        if oracle.partition(p, 13).tolist() != [min(t * 13, 350) // 7 for t in range(27)] + [50]:
            return False
        if oracle.partition(np.array([0, 0, 0, 5, 5, 9, 9], np.int32), 4).tolist() != [2, 2, 4, 6]:
            return False
        if oracle.num_tiles(9, 8) != 2:
            return False
        return True
    finally:
        oracle._h = saved


def test_unmodified_source_passes(tmp_path):
    assert pins_pass(compile_variant(tmp_path, "pristine", SRC))


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(tmp_path, name, old, new):
    assert SRC.count(old) >= 1, "mutation site not found: the oracle source changed, update this test"
    mutated = SRC.replace(old, new, 1)
    assert mutated != SRC
    assert not pins_pass(compile_variant(tmp_path, name, mutated)), "mutant survived: " + name
