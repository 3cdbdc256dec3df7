"""CPU oracle for the DENSE hot path.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It shares no code with the HIP path and never imports it.

  dense_oracle.c  plain C: Philox4x32-10, Floyd one-hop sampling, Algorithm 1
                  (multi-hop sampling into DENSE), repr_map, H^0 gather.
  sage.py         NumPy fp64: GraphSage-mean forward / backward over DENSE
                  (Algorithms 2 and 3 of the paper with mean aggregation).
  distmult.py     NumPy fp64: DistMult decoder with shared negatives, forward / backward.
  heads.py        NumPy: softmax cross-entropy head (fp64), Adagrad update of learnable rows (fp32).
"""
import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dense_oracle.c")
_LIB = os.path.join(_HERE, "libdense_oracle.so")
_lib = None


_LIB_OMP = os.path.join(_HERE, "libdense_oracle_omp.so")
_lib_omp = None
_use_openmp = False
GCC_FLAGS = ["-O2", "-std=c11", "-Wall", "-Wextra", "-Wno-unknown-pragmas", "-shared", "-fPIC"]


def build(force: bool = False) -> str:
    """Compile dense_oracle.c with gcc into libdense_oracle.so beside it (single-threaded) and, from the same file
    with -fopenmp, libdense_oracle_omp.so, whose per-node sampling loop runs on all cores."""
    for lib, extra in ((_LIB, []), (_LIB_OMP, ["-fopenmp"])):
        stale = (not os.path.exists(lib)) or os.path.getmtime(lib) < os.path.getmtime(_SRC)
        if force or stale:
            tmp = lib + ".tmp.%d" % os.getpid()
            subprocess.check_call(["gcc"] + GCC_FLAGS + extra + [_SRC, "-o", tmp])
            os.replace(tmp, lib)
    return _LIB


def use_openmp(on: bool) -> None:
    """Route the C entry points to the OpenMP build (same source, same results; threads from OMP_NUM_THREADS)."""
    global _use_openmp
    _use_openmp = bool(on)


def _bind(path):
    lib = ctypes.CDLL(path)
    i64p = ctypes.POINTER(ctypes.c_int64)
    i32p = ctypes.POINTER(ctypes.c_int32)
    u32p = ctypes.POINTER(ctypes.c_uint32)
    lib.orc_philox4x32_10.argtypes = [u32p, u32p, u32p]
    lib.orc_philox4x32_10.restype = None
    lib.orc_floyd_positions.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64, ctypes.c_uint32,
                                        ctypes.c_uint32, ctypes.c_uint32, i64p]
    lib.orc_floyd_positions.restype = None
    lib.orc_onehop.argtypes = [i64p, i32p, i64p, i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                               ctypes.c_uint64, ctypes.c_uint32, i32p]
    lib.orc_onehop.restype = ctypes.c_int32
    lib.orc_dense_sample.argtypes = [ctypes.c_int64, i64p, i32p, i64p, i32p, ctypes.c_int32,
                                     i32p, ctypes.c_int32, ctypes.c_int32, i32p, ctypes.c_uint64,
                                     ctypes.c_int64, ctypes.c_int64,
                                     i64p, i32p, i64p, i32p, i32p, i64p]
    lib.orc_dense_sample.restype = ctypes.c_int
    lib.orc_dense_gather.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, i32p, ctypes.c_int64,
                                     ctypes.c_void_p]
    lib.orc_dense_gather.restype = None
    return lib


def _load():
    global _lib, _lib_omp
    if _lib is None:
        build()
        _lib = _bind(_LIB)
    if _use_openmp:
        if _lib_omp is None:
            _lib_omp = _bind(_LIB_OMP)
        return _lib_omp
    return _lib


def _p(a: Optional[np.ndarray], ctype):
    if a is None:
        return ctypes.cast(None, ctypes.POINTER(ctype))
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def philox4x32_10(ctr: Sequence[int], key: Sequence[int]) -> np.ndarray:
    c = np.array(ctr, dtype=np.uint32)
    k = np.array(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    _load().orc_philox4x32_10(_p(c, ctypes.c_uint32), _p(k, ctypes.c_uint32), _p(out, ctypes.c_uint32))
    return out


def floyd_positions(deg: int, f: int, seed: int, node: int, hop: int, dirbit: int = 0) -> np.ndarray:
    picks = np.zeros(f, dtype=np.int64)
    _load().orc_floyd_positions(deg, f, seed, node, hop, dirbit, _p(picks, ctypes.c_int64))
    return picks


@dataclass
class Graph:
    """Adjacency by source (rowptr_out/col_out) and, optionally, by destination."""
    num_nodes: int
    rowptr_out: np.ndarray
    col_out: np.ndarray
    rowptr_in: Optional[np.ndarray] = None
    col_in: Optional[np.ndarray] = None

    def __post_init__(self):
        self.rowptr_out = _i64(self.rowptr_out)
        self.col_out = _i32(self.col_out)
        if self.rowptr_in is not None:
            self.rowptr_in = _i64(self.rowptr_in)
            self.col_in = _i32(self.col_in)


@dataclass
class Dense:
    """The DENSE arrays of Section 4.1 plus repr_map of Section 4.2."""
    node_id_offsets: np.ndarray   # int64[k+2]
    node_ids: np.ndarray          # int32[N]
    nbr_offsets: np.ndarray       # int64[N - n_0 + 1]
    nbrs: np.ndarray              # int32[E]
    repr_map: np.ndarray          # int32[E]

    @property
    def num_layers(self) -> int:
        return len(self.node_id_offsets) - 2


def onehop(g: Graph, v: int, f: int, seed: int, hop: int, direction: int = 0) -> np.ndarray:
    out = np.zeros(2 * f + 1, dtype=np.int32)
    if direction != 0 and g.rowptr_in is None:
        raise ValueError("direction needs the in-edge adjacency")
    c = _load().orc_onehop(_p(g.rowptr_out, ctypes.c_int64), _p(g.col_out, ctypes.c_int32),
                           _p(g.rowptr_in, ctypes.c_int64), _p(g.col_in, ctypes.c_int32),
                           direction, v, f, seed, hop, _p(out, ctypes.c_int32))
    return out[:c].copy()


def dense_sample(g: Graph, targets, fanouts, seed: int, direction: int = 0) -> Dense:
    """Algorithm 1: k-hop sample of `targets` (unique ids) with fanouts ordered away from the targets."""
    targets = _i32(targets)
    fan = _i32(fanouts)
    k = len(fan)
    if direction != 0 and g.rowptr_in is None:
        raise ValueError("direction needs the in-edge adjacency")
    mult = 2 if direction == 2 else 1
    level, cap_nodes, cap_nbrs = len(targets), len(targets), 0
    for f in fan:
        level = level * int(f) * mult
        cap_nbrs += level
        cap_nodes += min(level, g.num_nodes)
    cap_nodes = min(cap_nodes, g.num_nodes)
    node_id_offsets = np.zeros(k + 2, dtype=np.int64)
    node_ids = np.zeros(cap_nodes, dtype=np.int32)
    nbr_offsets = np.zeros(cap_nodes + 1, dtype=np.int64)
    nbrs = np.zeros(max(cap_nbrs, 1), dtype=np.int32)
    repr_map = np.zeros(max(cap_nbrs, 1), dtype=np.int32)
    counts = np.zeros(2, dtype=np.int64)
    rc = _load().orc_dense_sample(g.num_nodes, _p(g.rowptr_out, ctypes.c_int64), _p(g.col_out, ctypes.c_int32),
                                  _p(g.rowptr_in, ctypes.c_int64), _p(g.col_in, ctypes.c_int32), direction,
                                  _p(targets, ctypes.c_int32), len(targets), k, _p(fan, ctypes.c_int32), seed,
                                  cap_nodes, cap_nbrs,
                                  _p(node_id_offsets, ctypes.c_int64), _p(node_ids, ctypes.c_int32),
                                  _p(nbr_offsets, ctypes.c_int64), _p(nbrs, ctypes.c_int32),
                                  _p(repr_map, ctypes.c_int32), _p(counts, ctypes.c_int64))
    if rc == -1:
        raise ValueError("bad argument: id out of range, duplicate target, k < 1 or fanout < 1")
    if rc != 0:
        raise RuntimeError("oracle capacity exceeded")
    n, e = int(counts[0]), int(counts[1])
    n_with_nbrs = n - int(node_id_offsets[1])
    return Dense(node_id_offsets, node_ids[:n].copy(), nbr_offsets[:n_with_nbrs + 1].copy(),
                 nbrs[:e].copy(), repr_map[:e].copy())


def dense_sample_edges(g: Graph, src, dst, neg, fanouts, seed: int, direction: int = 0):
    """Link-prediction front end (Section 2: a training example is a pair of target nodes; Algorithm 1
    takes "unique node IDs"): the targets are the distinct ids among the edge endpoints and the negative
    nodes, in ascending id (a reading: the paper does not order them); returns the DENSE sample of those
    targets and, for src / dst / neg, the index of each id in the target list."""
    src, dst, neg = _i32(src), _i32(dst), _i32(neg)
    targets = np.unique(np.concatenate([src, dst, neg]))              # sorted, distinct
    d = dense_sample(g, targets, fanouts, seed, direction)
    return d, np.searchsorted(targets, src), np.searchsorted(targets, dst), np.searchsorted(targets, neg)


def embedding_sgd(table: np.ndarray, node_ids: np.ndarray, d_h0: np.ndarray, lr: float) -> np.ndarray:
    """Learnable base representations (Section 2: their updates are applied to the lookup table):
    table[node_ids[r]] -= lr * d_h0[r] in fp32, product and difference rounded separately.  Plain SGD is
    a reading; the paper does not name the optimiser.  Returns the updated copy."""
    out = np.array(table, dtype=np.float32, copy=True)
    step = np.float32(lr) * np.asarray(d_h0, dtype=np.float32)
    out[node_ids] = out[node_ids] - step
    return out


def dense_gather(table: np.ndarray, node_ids: np.ndarray) -> np.ndarray:
    """H^0[r] = table[node_ids[r]] (Section 4.2), any fixed-size row dtype."""
    assert table.ndim == 2 and table.flags.c_contiguous
    node_ids = _i32(node_ids)
    out = np.empty((len(node_ids), table.shape[1]), dtype=table.dtype)
    row_bytes = table.shape[1] * table.itemsize
    _load().orc_dense_gather(table.ctypes.data, row_bytes, row_bytes, _p(node_ids, ctypes.c_int32),
                             len(node_ids), out.ctypes.data)
    return out


from .sage import (round_bf16, bf16_terms, dense_layer_view, sage_forward, sage_backward, SageParams,  # noqa: E402
                   ForwardState)
from .distmult import distmult_forward, distmult_backward, DistMultState  # noqa: E402
from .heads import softmax_xent, mean_xent_grad, embedding_adagrad  # noqa: E402

__all__ = ["build", "use_openmp", "GCC_FLAGS", "philox4x32_10", "floyd_positions", "Graph", "Dense", "onehop", "dense_sample",
           "dense_sample_edges", "embedding_sgd",
           "dense_gather", "round_bf16", "dense_layer_view", "sage_forward", "sage_backward",
           "SageParams", "ForwardState", "distmult_forward", "distmult_backward", "DistMultState",
           "softmax_xent", "mean_xent_grad", "embedding_adagrad", "bf16_terms"]
