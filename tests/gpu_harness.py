"""Helpers shared by the GPU parity tests: run the HIP path and the oracle on the same inputs."""
import numpy as np
import torch

import oracle
import paper_2202_02365_amd as dn

DENSE_FIELDS = ("node_id_offsets", "node_ids", "nbr_offsets", "nbrs", "repr_map")


class DeviceGraph:
    def __init__(self, rowptr, col, rowptr_in=None, col_in=None):
        dev = torch.device("cuda:0")
        t = lambda a: None if a is None else torch.as_tensor(a).to(dev)
        self.graph = dn.Graph(t(rowptr), t(col), t(rowptr_in), t(col_in))
        self.num_nodes = len(rowptr) - 1
        self.oracle = oracle.Graph(self.num_nodes, np.asarray(rowptr), np.asarray(col),
                                   None if rowptr_in is None else np.asarray(rowptr_in),
                                   None if col_in is None else np.asarray(col_in))


def gpu_sample(dg: DeviceGraph, batch: dn.Batch, targets: np.ndarray, seed: int):
    t = torch.from_numpy(np.ascontiguousarray(targets, dtype=np.int32)).to("cuda:0")
    dn.dense_sample(batch, dg.graph, t, seed)
    return {k: v.cpu().numpy() for k, v in batch.view().items()}


def assert_dense_equal(view: dict, d: "oracle.Dense"):
    for name in DENSE_FIELDS:
        got = view[name].astype(np.int64)
        want = np.asarray(getattr(d, name), dtype=np.int64)
        assert got.shape == want.shape, "%s: shape %s vs oracle %s" % (name, got.shape, want.shape)
        if not np.array_equal(got, want):
            bad = np.nonzero(got != want)[0]
            raise AssertionError("%s differs from the oracle at %d of %d entries, first at %d: %d vs %d"
                                 % (name, len(bad), len(want), bad[0], got[bad[0]], want[bad[0]]))


def row_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max over rows of (max abs error in the row / L2 norm of the oracle's row)."""
    if want.size == 0:
        return 0.0
    got = got.astype(np.float64).reshape(want.shape)
    if want.ndim == 1:
        want = want[None, :]
        got = got[None, :]
    norm = np.linalg.norm(want, axis=1)
    err = np.abs(got - want).max(axis=1)
    return float((err / np.maximum(norm, 1e-30))[norm > 0].max()) if (norm > 0).any() else float(err.max())


def to_dev(arrs):
    return [torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda:0") for a in arrs]
