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
    # a row whose oracle norm is zero (an untouched gradient row, an all-zero input column) must be zero on the device
    # too: any non-zero value there counts as an error of its full absolute size, far above every tolerance in use
    zero_rows = float(err[norm == 0].max()) if (norm == 0).any() else 0.0
    rel = float((err / np.maximum(norm, 1e-30))[norm > 0].max()) if (norm > 0).any() else 0.0
    return max(rel, zero_rows)


def exact_distance_report(name, got: dict, bf16: dict, exact: dict, fwd_key="fwd", d_out=None, layers=1, tol=1e-4):
    """Distance of the device's results from the oracle's fp64 `exact` mode (the paper's arithmetic is fp32, Section 6;
    the shipped path rounds matrix-core operands to bfloat16).  Printed for every quantity; checked two ways:
      - triangle inequality: device-vs-exact <= oracle(bf16)-vs-exact + the parity tolerance, for every quantity;
      - forward output: one bfloat16 rounding moves an operand element by up to 2^-9 of its binade, uniformly, i.e. with
        standard deviation 2^-8 / sqrt(12) of the value at the binade's lower end; two rounded operands per product
        give an element of Z the relative deviation sigma = sqrt(2) * 2^-8 / sqrt(12) = 0.41 * 2^-8 of the element's
        rms, or sigma / sqrt(d_out) of the row norm; single-term roundings enter once per layer chain (later layers
        carry the error on, their own operands have 16 bits), so k layers give sqrt(k) of it.  The bound allows 16
        sigma sqrt(k): the maximum over 10^4..10^5 elements sits at 4-5 sigma and rows with a small norm relative to
        their operands (cancellation) roughly double it (measured 9-10 sigma sqrt(k) at the two small workloads)."""
    dev_exact = {k: row_rel_err(np.asarray(got[k]), exact[k]) for k in got}
    orc_exact = {k: row_rel_err(np.asarray(bf16[k], dtype=np.float64), exact[k]) for k in got}
    print(name, "device vs exact:", {k: float("%.2e" % v) for k, v in dev_exact.items()},
          "| oracle bf16 vs exact:", {k: float("%.2e" % v) for k, v in orc_exact.items()})
    for k in got:
        assert dev_exact[k] <= orc_exact[k] + tol, (k, dev_exact[k], orc_exact[k])
    if d_out is not None and fwd_key in got:
        sigma = 0.41 * 2.0 ** -8 / np.sqrt(d_out)
        bound = 16.0 * sigma * np.sqrt(layers)
        print(name, "forward vs exact %.2e = %.1f sigma sqrt(k); bound %.2e" %
              (dev_exact[fwd_key], dev_exact[fwd_key] / (sigma * np.sqrt(layers)), bound))
        assert dev_exact[fwd_key] <= bound, (dev_exact[fwd_key], bound)
    return dev_exact


def to_dev(arrs):
    return [torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda:0") for a in arrs]
