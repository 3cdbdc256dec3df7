"""GraphSage-mean encoder over DENSE, forward and backward, in NumPy fp64.
TEST INFRASTRUCTURE ONLY (see the package docstring).

What it follows (MariusGNN paper, Section 4.2):
  - Step 1 / Algorithm 3: a layer's output rows are the nodes of node_ids after
    node_id_offsets[1]; neighbour rows are selected through repr_map, reduced per node
    over the sequential segments delimited by nbr_offsets, and combined with the node's
    own row (self_repr = H[node_id_offsets[1]:]).
  - Step 2 / Algorithm 2: after each layer the first Delta and the neighbours of the
    second Delta are dropped and every array is rebased, so the same layer code serves
    every layer.
  - Section 2: h_v^i = AGG(h_v^{i-1}, {h_u^{i-1} : u in N_v}) with learnable parameters.

Readings of points the paper leaves open:
  - the GraphSage layer itself is not written out in the paper; the mean variant is used:
        Z^i = H_self W_s^i + mean_nbrs(H) W_n^i + b^i,   H^i = ReLU(Z^i) for i < k, H^k = Z^k,
    an empty neighbourhood contributes a zero mean; no dropout, no output normalisation.
    aggregation="sum" with identity weights reproduces Algorithm 3 as printed.
  - precision: mode "exact" is fp64 throughout.  Mode "bf16" models matrix-core operands:
    every GEMM operand is a sum of bfloat16 terms (round-to-nearest-even), products and
    sums stay fp64.  Operands that derive from the caller's inputs by arithmetic both
    sides can repeat bit for bit (H^0 rows, the layer-1 neighbour mean, weights, the
    upstream gradient dL/dH^k) are ONE term, bf16(x).  Operands computed on the device
    through a matrix-core accumulation, whose last bits depend on the accumulation order
    (activations H^i for i >= 1, neighbour means of them, back-propagated dZ^i for i < k),
    are TWO terms, bf16(x) + bf16(x - bf16(x)): a rounding decision has to be taken in one
    precision on both sides, and with a second term the sum no longer depends on which
    way the first one was rounded.  The value that gets split is produced in the
    arithmetic the device uses at that point: the neighbour mean is an fp32 sum in
    ascending slot order followed by an fp32 division, activations and gradients are
    stored as fp32.
  - backward: the gradient of the layer above with respect to Z passes where Z > 0;
    dW = operand^T dZ, db = column sums of dZ, and the gradient with respect to the input
    rows is the self part plus, for every neighbour slot, dM[owner] / count[owner].
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np


def bf16_terms(x: np.ndarray, terms: int) -> np.ndarray:
    """x as a sum of `terms` bfloat16 values (1 or 2), returned in fp64."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    hi = round_bf16(x32)
    if terms == 1:
        return hi.astype(np.float64)
    lo = round_bf16(x32 - hi)            # x32 - hi is exact in fp32
    return hi.astype(np.float64) + lo.astype(np.float64)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 -> nearest bfloat16 (ties to even) -> fp32.  Inf stays Inf, NaN stays NaN."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    u = x32.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    r = ((u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)).astype(np.uint32)
    is_nan = np.isnan(x32)
    r = np.where(is_nan, (x32.view(np.uint32) | np.uint32(0x00400000)) & np.uint32(0xFFFF0000), r)
    return r.astype(np.uint32).view(np.float32).reshape(x32.shape)


@dataclass
class DenseView:
    """The five arrays as one layer sees them."""
    node_id_offsets: np.ndarray
    node_ids: np.ndarray
    nbr_offsets: np.ndarray
    nbrs: np.ndarray
    repr_map: np.ndarray


def dense_update(d: DenseView) -> DenseView:
    """Algorithm 2: drop the first Delta and the second Delta's neighbours, rebase the rest."""
    n_prev = int(d.node_id_offsets[1])                               # len(Delta_{i-1})
    n_cur = int(d.node_id_offsets[2] - d.node_id_offsets[1])         # len(Delta_i)
    e_cur = int(d.nbr_offsets[n_cur])                                # len(Delta_i_nbrs)
    return DenseView(node_id_offsets=d.node_id_offsets[1:] - n_prev,
                     node_ids=d.node_ids[n_prev:],
                     nbr_offsets=d.nbr_offsets[n_cur:] - e_cur,
                     nbrs=d.nbrs[e_cur:],
                     repr_map=d.repr_map[e_cur:] - n_prev)


def dense_layer_view(dense, layer: int) -> DenseView:
    """DENSE as layer `layer` (1-based) sees it: Algorithm 2 applied layer-1 times."""
    v = DenseView(np.asarray(dense.node_id_offsets, dtype=np.int64), np.asarray(dense.node_ids),
                  np.asarray(dense.nbr_offsets, dtype=np.int64), np.asarray(dense.nbrs),
                  np.asarray(dense.repr_map, dtype=np.int64))
    for _ in range(layer - 1):
        v = dense_update(v)
    return v


@dataclass
class SageParams:
    w_self: List[np.ndarray]          # layer i-1: [d_{i-1} x d_i]
    w_nbr: List[np.ndarray]
    bias: List[np.ndarray]
    aggregation: str = "mean"         # "mean" | "sum"
    final_relu: bool = False


@dataclass
class LayerState:
    view: DenseView
    counts: np.ndarray                # neighbours per output row
    self_op: np.ndarray               # GEMM operand (rounded in bf16 mode), fp64
    nbr_op: np.ndarray
    z: np.ndarray                     # pre-activation, fp64
    relu: bool


@dataclass
class ForwardState:
    layers: List[LayerState] = field(default_factory=list)
    h: List[np.ndarray] = field(default_factory=list)   # H^0 .. H^k as the next layer reads them
    out: Optional[np.ndarray] = None


def _segment_reduce(h: np.ndarray, view: DenseView, aggregation: str, acc_dtype) -> np.ndarray:
    """Algorithm 3 lines 1-2: index_select by repr_map, then reduce each node's sequential
    segment.  Sums run over a segment's slots in ascending order in acc_dtype."""
    starts = view.nbr_offsets[:-1]
    counts = np.diff(view.nbr_offsets)
    acc = np.zeros((len(counts), h.shape[1]), dtype=acc_dtype)
    hh = h.astype(acc_dtype)
    for t in range(int(counts.max()) if len(counts) else 0):
        rows = np.nonzero(counts > t)[0]
        acc[rows] = acc[rows] + hh[view.repr_map[starts[rows] + t]]
    if aggregation == "mean":
        nz = counts > 0
        acc[nz] = acc[nz] / counts[nz].astype(acc_dtype)[:, None]
    elif aggregation != "sum":
        raise ValueError(aggregation)
    return acc


def sage_forward(dense, h0: np.ndarray, params: SageParams, mode: str = "exact") -> ForwardState:
    """H^0 -> H^k over DENSE.  Returns every layer's operands and outputs; .out = H^k (rows = targets)."""
    if mode not in ("exact", "bf16"):
        raise ValueError(mode)
    k = len(params.w_self)
    rb = round_bf16 if mode == "bf16" else (lambda a: a)
    store = (lambda a: a.astype(np.float32)) if mode == "bf16" else (lambda a: a.astype(np.float64))

    def operand(a, layer):
        if mode != "bf16":
            return a.astype(np.float64)
        return bf16_terms(a, 1 if layer == 1 else 2)

    view = dense_layer_view(dense, 1)
    h = store(np.asarray(h0))
    st = ForwardState()
    st.h.append(h)
    for i in range(1, k + 1):
        n_prev = int(view.node_id_offsets[1])
        counts = np.diff(view.nbr_offsets)
        nbr_aggr = _segment_reduce(h, view, params.aggregation, np.float32 if mode == "bf16" else np.float64)
        self_repr = h[n_prev:]
        a_self = operand(self_repr, i)
        a_nbr = operand(nbr_aggr, i)
        w_s = rb(params.w_self[i - 1]).astype(np.float64)
        w_n = rb(params.w_nbr[i - 1]).astype(np.float64)
        z = a_self @ w_s + a_nbr @ w_n + params.bias[i - 1].astype(np.float64)[None, :]
        relu = (i < k) or params.final_relu
        h = store(np.maximum(z, 0.0) if relu else z)
        st.layers.append(LayerState(view, counts, a_self, a_nbr, z, relu))
        st.h.append(h)
        view = dense_update(view)                                   # Step 2
    st.out = h
    return st


@dataclass
class Gradients:
    d_w_self: List[np.ndarray]
    d_w_nbr: List[np.ndarray]
    d_bias: List[np.ndarray]
    d_h0: np.ndarray
    d_z: List[np.ndarray]


def sage_backward(st: ForwardState, params: SageParams, grad_out: np.ndarray, mode: str = "exact") -> Gradients:
    """Gradients of <grad_out, H^k> with respect to every weight, bias and H^0."""
    k = len(params.w_self)
    rb = round_bf16 if mode == "bf16" else (lambda a: a)
    store = (lambda a: a.astype(np.float32).astype(np.float64)) if mode == "bf16" else (lambda a: a)
    g = store(np.asarray(grad_out, dtype=np.float64))
    d_ws, d_wn, d_b, d_zs = [None] * k, [None] * k, [None] * k, [None] * k
    for i in range(k, 0, -1):
        ls = st.layers[i - 1]
        view = ls.view
        if ls.relu:
            d_z = g * (ls.z > 0.0)
        else:
            d_z = g
        d_zs[i - 1] = d_z
        d_zb = d_z if mode != "bf16" else bf16_terms(d_z, 1 if i == k else 2)
        w_s = rb(params.w_self[i - 1]).astype(np.float64)
        w_n = rb(params.w_nbr[i - 1]).astype(np.float64)
        d_ws[i - 1] = ls.self_op.T @ d_zb
        d_wn[i - 1] = ls.nbr_op.T @ d_zb
        d_b[i - 1] = d_z.sum(axis=0)
        d_self = d_zb @ w_s.T
        d_m = d_zb @ w_n.T
        n_prev = int(view.node_id_offsets[1])
        g_prev = np.zeros((len(view.node_ids), d_self.shape[1]), dtype=np.float64)
        g_prev[n_prev:] += d_self
        owner = np.repeat(np.arange(len(ls.counts)), ls.counts)       # slot -> output row
        if params.aggregation == "mean":
            contrib = d_m[owner] / ls.counts[owner].astype(np.float64)[:, None]
        else:
            contrib = d_m[owner]
        np.add.at(g_prev, view.repr_map, contrib)
        g = store(g_prev)
    return Gradients(d_ws, d_wn, d_b, g, d_zs)
