import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def read_golden(name):
    """Parse a tests/golden/*.txt fixture into {block name: float64 array}."""
    blocks, cur, rows, want = {}, None, [], 0
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            tok = line.split()
            if cur is None or len(rows) == want:
                if cur is not None:
                    blocks[cur] = np.array(rows, dtype=np.float64)
                cur, want, rows = tok[0], int(tok[1]), []
                continue
            rows.append([float(t) for t in tok])
    if cur is not None:
        blocks[cur] = np.array(rows, dtype=np.float64)
    return blocks


def dense_to_csr(A):
    """Dense matrix -> (rowptr int64, colidx int32, values float32) keeping stored zeros out."""
    A = np.asarray(A)
    rp = [0]
    ci, av = [], []
    for i in range(A.shape[0]):
        for j in range(A.shape[1]):
            if A[i, j] != 0:
                ci.append(j)
                av.append(A[i, j])
        rp.append(len(ci))
    return (np.array(rp, dtype=np.int64), np.array(ci, dtype=np.int32), np.array(av, dtype=np.float32))


def csr_to_dense(rp, ci, av, n):
    A = np.zeros((n, n), dtype=np.float64)
    for i in range(n):
        for e in range(rp[i], rp[i + 1]):
            A[i, ci[e]] += float(av[e])
    return A


@pytest.fixture(scope="session")
def golden():
    return read_golden
