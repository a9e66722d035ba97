import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """GPU tests are skipped (not failed) where no GPU is visible."""
    have = None
    for item in items:
        if "gpu" in item.keywords:
            if have is None:
                try:
                    import torch

                    have = torch.cuda.is_available()
                except Exception:
                    have = False
            if not have:
                item.add_marker(pytest.mark.skip(reason="no GPU visible"))


def dense_of(A):
    """Dense float64 image of a workloads.CSR (CSR or BCSR); duplicates add up."""
    bs = A.bs
    D = np.zeros((A.rows * bs, A.cols * bs), dtype=np.float64)
    v = A.vals.astype(np.float64).reshape(-1, bs, bs)
    for i in range(A.rows):
        for p in range(A.pos[i], A.pos[i + 1]):
            j = A.crd[p]
            D[i * bs:(i + 1) * bs, j * bs:(j + 1) * bs] += v[p]
    return D


def adversarial_lengths(rng, rows, cols, kind):
    """Row-length vectors for the structural edge cases of a position cut."""
    L = np.zeros(rows, dtype=np.int64)
    if kind == "all_empty":
        pass
    elif kind == "one_row_has_all":
        L[rows // 2] = cols
    elif kind == "empty_head_tail":
        L[rows // 3: 2 * rows // 3] = rng.integers(1, min(cols, 9), size=2 * rows // 3 - rows // 3)
    elif kind == "mostly_empty":
        idx = rng.choice(rows, size=max(1, rows // 50), replace=False)
        L[idx] = rng.integers(1, min(cols, 300), size=idx.size)
    elif kind == "mixed":
        L[:] = rng.integers(0, 6, size=rows)
        idx = rng.choice(rows, size=max(1, rows // 100), replace=False)
        L[idx] = rng.integers(min(cols, 100), min(cols, 5000) + 1, size=idx.size)
    elif kind == "single_long_rows":
        L[:] = 0
        L[::max(1, rows // 7)] = min(cols, 3000)
    elif kind == "ones":
        L[:] = 1
    else:
        raise ValueError(kind)
    return np.minimum(L, cols)


ADVERSARIAL_KINDS = ["all_empty", "one_row_has_all", "empty_head_tail", "mostly_empty", "mixed",
                     "single_long_rows", "ones"]
