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
    S = oracle.slab_build(g["rows"], g["cols"], g["pos"], g["crd"], g["vals"], W=g["W"], CH=g["CH"])
    if (S.nslots, S.npairs, S.nq, S.nslabs) != (g["nslots"], g["npairs"], g["nq"], g["nslabs"]):
        return False
    for name in ("svals", "scol", "srow", "chunk_pair", "slab_chunk", "qpos", "qidx"):
        if getattr(S, name).tolist() != g[name]:
            return False
    y, mag = oracle.spmv_slab(S, g["x"])
    return y.tolist() == g["y"] and mag.tolist() == g["mag"]


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
    (k // 4) * (CH // 2) + 4 * l + k % 4; otherwise values are stored in slot order."""
    j = np.arange(S.nslots, dtype=np.int64)
    if S.CH % 8:
        return j
    c, o = j // S.CH, j % S.CH
    l, k = o // 8, o % 8
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
    if not (np.array_equal(S.srow[real], rows_of[order]) and np.array_equal(col[real], A.crd[order])
            and np.array_equal(vals_by_slot[real].view(np.uint32), A.vals[order].view(np.uint32))):
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
    ("slab_values_by_slot", "svals[slab_value_index(CH, j)] = p >= 0 ? vals[p] : 0.0f;", "svals[slab_value_index(CH, j)] = p >= 0 ? vals[j < nnz ? j : 0] : 0.0f;"),
    ("slab_values_not_permuted", "svals[slab_value_index(CH, j)] = p >= 0 ? vals[p] : 0.0f;", "svals[j] = p >= 0 ? vals[p] : 0.0f;"),
    ("slab_permutation_swaps_halves", "return c * CH + (k / 4) * (CH / 2) + 4 * l + k % 4;", "return c * CH + (1 - k / 4) * (CH / 2) + 4 * l + k % 4;"),
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
            return hand_case_ok() and properties_ok()
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


def test_value_order_inside_a_chunk_of_16():
    """Listed by hand: with chunks of 16 slots two lanes own slots 0-7 and 8-15; the values are stored as the first
    halves of both lanes' slots, then the second halves: s0 s1 s2 s3 | s8 s9 s10 s11 | s4 s5 s6 s7 | s12 s13 s14 s15."""
    pos = np.array([0, 16], dtype=np.int32)
    crd = np.arange(16, dtype=np.int32)
    vals = np.arange(100, 116, dtype=np.float32)
    S = oracle.slab_build(1, 40, pos, crd, vals, W=40, CH=16)
    assert S.svals.tolist() == [100, 101, 102, 103, 108, 109, 110, 111, 104, 105, 106, 107, 112, 113, 114, 115]
    assert (S.scol & 0x7FFF).tolist() == list(range(16))        # columns stay in slot order
    y, _ = oracle.spmv_slab(S, np.arange(40, dtype=np.float32))
    assert y.tolist() == [float(sum((100 + i) * i for i in range(16)))]
