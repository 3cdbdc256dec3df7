import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _have_gpu() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _have_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


_GRAPH_CACHE = {}


def cached_rmat(V, E, seed=1, with_in=False):
    """R-MAT CSR (and CSC) as NumPy arrays, built once per test session."""
    import torch  # noqa: F401
    from workloads import rmat_csr, transpose_csr
    key = (V, E, seed)
    if key not in _GRAPH_CACHE:
        rp, col = rmat_csr(V, E, seed)
        _GRAPH_CACHE[key] = {"out": (rp.numpy(), col.numpy())}
    ent = _GRAPH_CACHE[key]
    if with_in and "in" not in ent:
        import torch
        rpt, colt = transpose_csr(torch.from_numpy(ent["out"][0]), torch.from_numpy(ent["out"][1]))
        ent["in"] = (rpt.numpy(), colt.numpy())
    return ent


@pytest.fixture(scope="session")
def rmat16k():
    return cached_rmat(16384, 262144, 1, with_in=True)


@pytest.fixture(scope="session")
def rmat1m():
    return cached_rmat(1 << 20, 1 << 24, 1)


def random_small_graph(rng: np.random.Generator, n: int, avg_deg: float):
    """Random directed graph on n nodes as (rowptr, col) with sorted, duplicate-free rows."""
    rows = []
    for u in range(n):
        d = min(n, rng.poisson(avg_deg))
        rows.append(np.sort(rng.choice(n, size=d, replace=False)).astype(np.int32))
    rowptr = np.zeros(n + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum([len(r) for r in rows])
    col = np.concatenate(rows).astype(np.int32) if rowptr[-1] else np.zeros(0, dtype=np.int32)
    return rowptr, col


def transpose_np(rowptr, col):
    n = len(rowptr) - 1
    src = np.repeat(np.arange(n), np.diff(rowptr))
    order = np.lexsort((src, col))
    rp = np.zeros(n + 1, dtype=np.int64)
    rp[1:] = np.cumsum(np.bincount(col, minlength=n))
    return rp, src[order].astype(np.int32)
