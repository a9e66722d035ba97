"""Pins of the oracle's column-slab hierarchy (oracle_slab_build, oracle_spmv_slab): a hand-worked case,
the definition checked by independent numpy code, invariants of the structure, the product over the
structure against the CSR definition, and planted mistakes that these checks must reject."""
import ctypes
import json
import os
import subprocess

import numpy as np
import pytest

import oracle
import workloads as wl
from conftest import ADVERSARIAL_KINDS, adversarial_lengths, dense_of

HERE = os.path.dirname(os.path.abspath(__file__))
GOLD = json.load(open(os.path.join(HERE, "golden", "slab_hand_worked.json")))
SRC = open(os.path.join(os.path.dirname(HERE), "oracle", "oracle.c")).read()


def hand_case_ok() -> bool:
    g = GOLD
    for f64 in (False, True):            # chunks of 2 slots: values in slot order for either value type
        S = oracle.slab_build(g["rows"], g["cols"], g["pos"], g["crd"], g["vals"], W=g["W"], CH=g["CH"], f64=f64)
        if (S.nslots, S.npairs, S.nq, S.nslabs) != (g["nslots"], g["npairs"], g["nq"], g["nslabs"]):
            return False
        if S.svals.dtype != (np.float64 if f64 else np.float32):
            return False
        for name in ("svals", "scol", "srow", "chunk_pair", "slab_chunk", "qpos", "qidx"):
            if getattr(S, name).tolist() != g[name]:
                return False
        y, mag = oracle.spmv_slab(S, g["x"])
        if not (y.tolist() == g["y"] and mag.tolist() == g["mag"]):
            return False
    return True


def decode(S):
    """(row, column, value) of every real slot, plus per-slot slab and pair, from the arrays alone."""
    slab_of_chunk = np.repeat(np.arange(S.nslabs), np.diff(S.slab_chunk))
    slab = np.repeat(slab_of_chunk, S.CH)
    col = slab.astype(np.int64) * S.W + (S.scol & 0x7FFF)
    end = (S.scol >> 15).astype(bool)
    start = np.ones(S.nslots, dtype=bool)
    start[1:] = end[:-1]
    pair = np.cumsum(start) - 1
    return slab, col, end, start, pair


def value_index(S):
    """Storage index of every slot's value: inside a chunk whose size is a multiple of 8, slot 8*l + k sits at
    (k // 4) * (CH // 2) + 4 * l + k % 4 for 4-byte values and at (k // 2) * (CH // 4) + 2 * l + k % 2 for 8-byte
    values (groups of 16 bytes, lane after lane); otherwise values are stored in slot order."""
    j = np.arange(S.nslots, dtype=np.int64)
    if S.CH % 8:
        return j
    c, o = j // S.CH, j % S.CH
    l, k = o // 8, o % 8
    if S.svals.dtype == np.float64:
        return c * S.CH + (k // 2) * (S.CH // 4) + 2 * l + k % 2
    return c * S.CH + (k // 4) * (S.CH // 2) + 4 * l + k % 4


def structure_ok(A, S) -> bool:
    """Everything the definition fixes, checked without the oracle's own code."""
    rows_of = np.repeat(np.arange(A.rows), np.diff(A.pos))
    if S.nslots % S.CH or S.slab_chunk[0] != 0 or S.slab_chunk[-1] * S.CH != S.nslots:
        return False
    if S.nslots == 0:
        return S.npairs == 0 and S.nq == 0 and not S.qpos.any()
    slab, col, end, start, pair = decode(S)
    real = S.srow >= 0
    # the real slots are exactly the stored entries: stable bucketing by slab
    order = np.argsort(A.crd // S.W, kind="stable")
    if real.sum() != A.nnz:
        return False
    vals_by_slot = S.svals[value_index(S)]
    want_vals = A.vals[order].astype(S.svals.dtype)          # fp32 -> fp64 is exact
    if not (np.array_equal(S.srow[real], rows_of[order]) and np.array_equal(col[real], A.crd[order])
            and vals_by_slot[real].tobytes() == want_vals.tobytes()):
        return False
    # every slab holds its entries first, then fewer than CH pad slots (value 0, column 0)
    counts = np.bincount(A.crd // S.W, minlength=S.nslabs)
    if not np.array_equal(np.diff(S.slab_chunk) * S.CH, (counts + S.CH - 1) // S.CH * S.CH):
        return False
    for s in range(S.nslabs):
        lo, hi = S.slab_chunk[s] * S.CH, S.slab_chunk[s + 1] * S.CH
        if not (real[lo:lo + counts[s]].all() and not real[lo + counts[s]:hi].any()):
            return False
    if vals_by_slot[~real].any() or (S.scol[~real] & 0x7FFF).any():
        return False
    # pairs: a new pair starts exactly where the row changes or a chunk begins; the last slot is an end
    want_start = np.ones(S.nslots, dtype=bool)
    want_start[1:] = S.srow[1:] != S.srow[:-1]
    want_start[::S.CH] = True
    if not (np.array_equal(start, want_start) and end[-1]) or pair[-1] + 1 != S.npairs:
        return False
    if not np.array_equal(S.chunk_pair[:-1], pair[::S.CH]) or S.chunk_pair[-1] != S.npairs:
        return False
    # rows list each of their pairs once, in the order of the pairs' first slots in the CSR; pad pairs are listed by nobody
    slot_of = np.empty(A.nnz, dtype=np.int64)
    slot_of[order] = np.nonzero(real)[0]
    firsts = start[slot_of]                                   # per CSR position: is its slot the first of a pair
    if not np.array_equal(S.qidx, pair[slot_of[firsts]]):
        return False
    want_qpos = np.concatenate([[0], np.cumsum(np.bincount(rows_of[firsts], minlength=A.rows))])
    return np.array_equal(S.qpos, want_qpos) and S.nq == int(firsts.sum())


CASES = [("mixed", 97, 13), ("empty rows", 1000, 8), ("one long row", 333, 4), ("mixed", 32736, 512), ("mixed", 500, 16),
         ("single entries", 5, 2), ("mixed", 1, 1)]


def matrices():
    rng = np.random.default_rng(77)
    for kind, W, CH in CASES:
        k = kind if kind in ADVERSARIAL_KINDS else "mixed"
        cols = 70_000 if W > 10_000 else 2501
        yield kind, wl.csr_from_lengths(adversarial_lengths(rng, 611, cols, k), cols, seed=len(kind) + W), W, CH


def properties_ok() -> bool:
    for kind, A, W, CH in matrices():
        S = oracle.slab_build(A.rows, A.cols, A.pos, A.crd, A.vals, W=W, CH=CH)
        if not structure_ok(A, S):
            return False
        x = wl.dense_uniform(A.cols, 5, wl.S_X)
        y, mag = oracle.spmv_slab(S, x)
        ref, rmag = oracle.spmv_csr(A.pos, A.crd, A.vals, x)
        if not (np.allclose(y, ref, rtol=0, atol=1e-12) and np.allclose(mag, rmag, rtol=1e-12, atol=0)):
            return False
        # 8-byte values: same structure, other storage order of the values, product in extended precision
        v64 = A.vals.astype(np.float64) * (1.0 + 2.0 ** -40)            # not representable in fp32
        x64 = x.astype(np.float64) * (1.0 - 2.0 ** -41)
        S64 = oracle.slab_build(A.rows, A.cols, A.pos, A.crd, v64, W=W, CH=CH, f64=True)
        for name in ("scol", "srow", "chunk_pair", "slab_chunk", "qpos", "qidx"):
            if not np.array_equal(getattr(S64, name), getattr(S, name)):
                return False
        if S64.svals[value_index(S64)][S64.srow >= 0].tobytes() != v64[np.argsort(A.crd // W, kind="stable")].tobytes():
            return False
        y64, mag64 = oracle.spmv_slab(S64, x64)
        ref64, rmag64 = oracle.spmv_csr_f64(A.pos, A.crd, v64, x64)
        if not (np.allclose(y64, ref64, rtol=0, atol=1e-15 * max(1.0, float(rmag64.max(initial=0.0))))
                and np.allclose(mag64, rmag64, rtol=1e-15, atol=0)):
            return False
    # unsorted and repeated columns inside a row: the order of the CSR is kept inside a slab
    pos = np.array([0, 5, 5, 7], dtype=np.int32)
    crd = np.array([9, 1, 9, 0, 4, 8, 8], dtype=np.int32)
    vals = np.arange(1, 8, dtype=np.float32)
    S = oracle.slab_build(3, 10, pos, crd, vals, W=4, CH=2)

    class M:
        pass
    A = M()
    A.rows, A.cols, A.nnz, A.pos, A.crd, A.vals = 3, 10, 7, pos, crd, vals
    if not structure_ok(A, S):
        return False
    y, _ = oracle.spmv_slab(S, np.arange(10, dtype=np.float32))
    if y.tolist() != [1 * 9 + 2 * 1 + 3 * 9 + 0 + 5 * 4, 0.0, 6 * 8 + 7 * 8]:
        return False
    # empty matrix, and a matrix without columns
    S = oracle.slab_build(4, 9, np.zeros(5, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32), W=4, CH=2)
    if (S.nslots, S.npairs, S.nq, S.nslabs) != (0, 0, 0, 3) or S.qpos.tolist() != [0] * 5 or S.slab_chunk.tolist() != [0] * 4:
        return False
    return True


def test_hand_worked_case():
    assert hand_case_ok()


def test_definition_and_invariants():
    assert properties_ok()


def test_dense_brute_force():
    A = wl.csr_from_lengths(np.random.default_rng(3).integers(0, 12, size=40), 53, seed=9)
    x = wl.dense_uniform(53, 9, wl.S_X)
    S = oracle.slab_build(A.rows, A.cols, A.pos, A.crd, A.vals, W=7, CH=4)
    y, _ = oracle.spmv_slab(S, x)
    assert np.allclose(y, dense_of(A) @ x.astype(np.float64), rtol=0, atol=1e-13)


MUTANTS = [
    ("slab_unstable_order", "int64_t j = base[s] + fill[s]++;", "int64_t j = base[s + 1] - 1 - fill[s]++;"),
    ("slab_no_padding", "int64_t padded = (base[s + 1] + CH - 1) / CH * CH;", "int64_t padded = base[s + 1];"),
    ("slab_pair_ignores_chunks", "return j % CH == 0 || slot_row[j] != slot_row[j - 1];", "return j == 0 || slot_row[j] != slot_row[j - 1];"),
    ("slab_pair_ignores_rows", "return j % CH == 0 || slot_row[j] != slot_row[j - 1];", "return j % CH == 0;"),
    ("slab_column_not_local", "scol[j] = p >= 0 ? (uint16_t)(crd[p] % W) : 0;", "scol[j] = p >= 0 ? (uint16_t)(crd[p]) : 0;"),
    ("slab_end_flag_one_late", "if (j == N - 1 || slab_is_start(srow, CH, j + 1)) scol[j] |= 0x8000u;",
     "if (j == N - 1 || slab_is_start(srow, CH, j)) scol[j] |= 0x8000u;"),
    ("slab_rows_list_every_slot", "if (slab_is_start(srow, CH, j)) qidx[nq++] = pair_of[j];", "qidx[nq++] = pair_of[j];"),
    ("slab_chunk_pair_off_by_one", "if (j % CH == 0) chunk_pair[j / CH] = pair_of[j];", "if (j % CH == 0) chunk_pair[j / CH] = pair_of[j] + 1;"),
    ("slab_spmv_wrong_slab_offset", "int64_t col = s * W + (scol[j] & 0x7fff);", "int64_t col = s * CH + (scol[j] & 0x7fff);"),
    ("slab_spmv_drops_pair", "for (int64_t q = qpos[i]; q < qpos[i + 1]; ++q) { acc += P[qidx[q]];", "for (int64_t q = qpos[i] + 1; q < qpos[i + 1]; ++q) { acc += P[qidx[q]];"),
    ("slab_values_by_slot", "((float *)svals)[at] = p >= 0 ? ((const float *)vals)[p] : 0.0f;",
     "((float *)svals)[at] = p >= 0 ? ((const float *)vals)[j < nnz ? j : 0] : 0.0f;"),
    ("slab_values_not_permuted", "int64_t at = slab_value_index_g(CH, j, g);", "int64_t at = j;"),
    ("slab_permutation_swaps_groups", "return c * CH + (k / g) * (CH / 8 * g) + g * l + k % g;",
     "return c * CH + (8 / g - 1 - k / g) * (CH / 8 * g) + g * l + k % g;"),
    ("slab_f64_values_by_slot", "((double *)svals)[at] = p >= 0 ? ((const double *)vals)[p] : 0.0;",
     "((double *)svals)[at] = p >= 0 ? ((const double *)vals)[j < nnz ? j : 0] : 0.0;"),
    ("slab_f64_values_rounded_to_fp32", "((double *)svals)[at] = p >= 0 ? ((const double *)vals)[p] : 0.0;",
     "((double *)svals)[at] = p >= 0 ? (float)((const double *)vals)[p] : 0.0;"),
    ("slab_f64_groups_of_four", "int64_t g = 16 / vbytes;", "int64_t g = 4;"),
    ("slab_f64_spmv_reads_fp32_order", "(long double)svals[slab_value_index_g(CH, j, 2)] * (long double)x[col];",
     "(long double)svals[slab_value_index_g(CH, j, 4)] * (long double)x[col];"),
    ("slab_f64_spmv_drops_pair", "for (int64_t q = qpos[i]; q < qpos[i + 1]; ++q) { acc += P[qidx[q]]; m += Pmag[qidx[q]]; }\n        y[i] = (double)acc;",
     "for (int64_t q = qpos[i] + 1; q < qpos[i + 1]; ++q) { acc += P[qidx[q]]; m += Pmag[qidx[q]]; }\n        y[i] = (double)acc;"),
    ("slab_f64_spmv_in_double_products_of_floats", "long double t = (long double)svals[slab_value_index_g(CH, j, 2)] * (long double)x[col];",
     "long double t = (long double)((float)svals[slab_value_index_g(CH, j, 2)] * (float)x[col]);"),
]


def with_library(lib, fn):
    saved = oracle._h
    try:
        oracle._h = None
        real_cdll = ctypes.CDLL
        ctypes.CDLL = lambda *_a, **_k: lib
        try:
            oracle._lib()
        finally:
            ctypes.CDLL = real_cdll
        return fn()
    finally:
        oracle._h = saved


def compile_variant(tmp_path, name, text):
    c, so = tmp_path / (name + ".c"), tmp_path / (name + ".so")
    c.write_text(text)
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", str(so), str(c), "-lm"])
    return ctypes.CDLL(str(so))


def pins_pass(lib) -> bool:
    def run():
        try:
            return hand_case_ok() and properties_ok() and value_order_16_ok()
        except (IndexError, ValueError):
            return False          # a mutant may produce arrays that do not even decode
    return with_library(lib, run)


def test_unmodified_source_passes(tmp_path):
    assert pins_pass(compile_variant(tmp_path, "pristine", SRC))


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(tmp_path, name, old, new):
    assert SRC.count(old) >= 1, "mutation site not found: the oracle source changed, update this test"
    mutated = SRC.replace(old, new)
    assert not pins_pass(compile_variant(tmp_path, name, mutated)), "mutant survived: " + name


def value_order_16_ok() -> bool:
    """Listed by hand: with chunks of 16 slots two lanes own slots 0-7 and 8-15.  4-byte values are stored as the
    first halves of both lanes' slots, then the second halves: s0 s1 s2 s3 | s8 s9 s10 s11 | s4 s5 s6 s7 | s12 s13 s14
    s15; 8-byte values as the lanes' first, second, third and fourth pairs of slots: s0 s1 | s8 s9 | s2 s3 | s10 s11 |
    s4 s5 | s12 s13 | s6 s7 | s14 s15."""
    pos = np.array([0, 16], dtype=np.int32)
    crd = np.arange(16, dtype=np.int32)
    vals = np.arange(100, 116, dtype=np.float32)
    S = oracle.slab_build(1, 40, pos, crd, vals, W=40, CH=16)
    if S.svals.tolist() != [100, 101, 102, 103, 108, 109, 110, 111, 104, 105, 106, 107, 112, 113, 114, 115]:
        return False
    if (S.scol & 0x7FFF).tolist() != list(range(16)):           # columns stay in slot order
        return False
    y, _ = oracle.spmv_slab(S, np.arange(40, dtype=np.float32))
    if y.tolist() != [float(sum((100 + i) * i for i in range(16)))]:
        return False
    S = oracle.slab_build(1, 40, pos, crd, vals, W=40, CH=16, f64=True)
    if S.svals.tolist() != [100, 101, 108, 109, 102, 103, 110, 111, 104, 105, 112, 113, 106, 107, 114, 115]:
        return False
    if (S.scol & 0x7FFF).tolist() != list(range(16)):
        return False
    y, _ = oracle.spmv_slab(S, np.arange(40, dtype=np.float64))
    return y.tolist() == [float(sum((100 + i) * i for i in range(16)))]


def test_value_order_inside_a_chunk_of_16():
    assert value_order_16_ok()


def test_f64_product_rounds_once():
    """A row whose exact sum needs more than 53 bits on the way: 1 + 2^-60 - 1 over three slabs.  Sums kept in
    extended precision give 2^-60; a double accumulator would give 0."""
    pos = np.array([0, 3], dtype=np.int32)
    crd = np.array([0, 5, 9], dtype=np.int32)
    vals = np.array([1.0, 2.0 ** -60, -1.0])
    S = oracle.slab_build(1, 12, pos, crd, vals, W=4, CH=2, f64=True)
    y, mag = oracle.spmv_slab(S, np.ones(12))
    assert y.tolist() == [2.0 ** -60]
    assert mag.tolist() == [2.0]                 # 2 + 2^-60 rounded to double
