"""ctypes binding of include/dense.h.  Same entry-point names; marshalling only."""
import ctypes
import os
import re
from typing import List, Optional, Sequence

import torch

DN_F32, DN_BF16 = 0, 1
DN_DIR_OUT, DN_DIR_IN, DN_DIR_BOTH = 0, 1, 2
DN_MAX_LAYERS = 6
DN_AGG_MEAN, DN_AGG_SUM = 0, 1

_PKG = os.path.dirname(os.path.abspath(__file__))
_HEADER = os.path.join(os.path.dirname(_PKG), "include", "dense.h")
_lib = None


class DenseError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__("libdense_mi355x error %d: %s" % (code, message))
        self.code = code


class _KernelTime(ctypes.Structure):
    _fields_ = [("tag", ctypes.c_char * 48), ("total_ms", ctypes.c_double), ("launches", ctypes.c_int64),
                ("p10_ms", ctypes.c_double), ("p50_ms", ctypes.c_double), ("p90_ms", ctypes.c_double)]


class _TrainStep(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_void_p), ("model", ctypes.c_void_p), ("graph", ctypes.c_void_p),
                ("targets", ctypes.c_void_p), ("n_targets", ctypes.c_int32), ("seed", ctypes.c_uint64),
                ("table", ctypes.c_void_p), ("ld_elems", ctypes.c_int64), ("out", ctypes.c_void_p),
                ("labels", ctypes.c_void_p), ("grad_scale", ctypes.c_float), ("loss", ctypes.c_void_p),
                ("grad_out", ctypes.c_void_p), ("dw_self", ctypes.POINTER(ctypes.c_void_p)),
                ("dw_nbr", ctypes.POINTER(ctypes.c_void_p)), ("dbias", ctypes.POINTER(ctypes.c_void_p)),
                ("dh0", ctypes.c_void_p), ("forward_only", ctypes.c_int32)]


class _View(ctypes.Structure):
    _fields_ = [("node_id_offsets", ctypes.c_void_p), ("node_ids", ctypes.c_void_p),
                ("nbr_offsets", ctypes.c_void_p), ("nbrs", ctypes.c_void_p), ("repr_map", ctypes.c_void_p)]


def library_path() -> str:
    return os.path.join(_PKG, "libdense_mi355x.so")


def declared_symbols() -> List[str]:
    """Names of every entry point include/dense.h declares."""
    text = open(_HEADER).read()
    return re.findall(r"DN_API\s+[\w\s\*]+?\b(\w+)\s*\(", text)


def load_library():
    """Loads the HIP library built in-tree.  Raises if it has not been built: there is no fallback."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise FileNotFoundError("%s is missing: run `python -c 'import __graft_entry__ as g; g.build()'`" % path)
    lib = ctypes.CDLL(path)
    vp, i32, i64, u64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64, ctypes.c_size_t
    pp = ctypes.POINTER(ctypes.c_void_p)
    sig = {
        "dn_last_error": (ctypes.c_char_p, []),
        "dn_graph_create": (ctypes.c_int, [pp, i64, vp, vp, vp, vp]),
        "dn_graph_destroy": (None, [vp]),
        "dn_batch_workspace_size": (ctypes.c_int, [i64, i32, i32, ctypes.POINTER(i32), i32, ctypes.POINTER(sz)]),
        "dn_batch_create": (ctypes.c_int, [pp, i64, i32, i32, ctypes.POINTER(i32), i32, vp, sz, vp]),
        "dn_batch_destroy": (None, [vp]),
        "dn_batch_capacity": (ctypes.c_int, [vp, ctypes.POINTER(i64), ctypes.POINTER(i64)]),
        "dense_sample": (ctypes.c_int, [vp, vp, vp, i32, u64, vp]),
        "dense_sample_noalloc": (ctypes.c_int, [vp, vp, i32, i32, ctypes.POINTER(i32), i32, u64, vp, vp, vp, i64, vp, vp, i64, vp, vp]),
        "dn_train_steps": (ctypes.c_int, [ctypes.POINTER(_TrainStep), i32, i32, vp]),
        "dense_sample_edges": (ctypes.c_int, [vp, vp, vp, vp, i32, vp, i32, u64, vp, vp, vp, vp]),
        "dn_embedding_sgd": (ctypes.c_int, [vp, vp, i32, i64, vp, ctypes.c_float, vp]),
        "dn_embedding_adagrad": (ctypes.c_int, [vp, vp, vp, i32, i64, vp, ctypes.c_float, ctypes.c_float, vp]),
        "dn_softmax_xent": (ctypes.c_int, [vp, i64, vp, i64, i32, ctypes.c_float, vp, vp, i64, vp]),
        "dn_batch_view": (ctypes.c_int, [vp, ctypes.POINTER(_View)]),
        "dn_batch_prepare_backward": (ctypes.c_int, [vp, i32, vp]),
        "dn_batch_counts": (ctypes.c_int, [vp, ctypes.POINTER(i64), vp]),
        "dense_gather": (ctypes.c_int, [vp, vp, i32, i32, i64, vp, vp]),
        "dn_model_workspace_size": (ctypes.c_int, [vp, i32, ctypes.POINTER(i32), i32, ctypes.POINTER(sz)]),
        "dn_model_create": (ctypes.c_int, [pp, vp, i32, ctypes.POINTER(i32), i32, vp, sz, vp]),
        "dn_model_set_weights": (ctypes.c_int, [vp, pp, pp, pp, vp]),
        "dn_model_destroy": (None, [vp]),
        "dn_model_status": (ctypes.c_int, [vp, ctypes.POINTER(i32), vp]),
        "dn_profile_enable": (ctypes.c_int, [i32]),
        "dn_profile_calibration_copy": (ctypes.c_int, [vp, vp, sz, vp]),
        "dn_profile_empty_bracket": (ctypes.c_int, [vp]),
        "dn_profile_step_stream_overlap": (ctypes.c_int, [ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_double)]),
        "dn_profile_collect": (ctypes.c_int, [ctypes.POINTER(_KernelTime), i32, ctypes.POINTER(i32)]),
        "dn_decoder_workspace_size": (ctypes.c_int, [i64, i32, i32, i32, i64, i64, ctypes.POINTER(sz)]),
        "dn_decoder_create": (ctypes.c_int, [pp, i64, i32, i32, i32, i64, i64, vp, sz, vp]),
        "dn_decoder_destroy": (None, [vp]),
        "distmult_forward": (ctypes.c_int, [vp, vp, i64, i64, vp, i64, vp, vp, vp, i64, vp, vp, vp, vp]),
        "distmult_backward": (ctypes.c_int, [vp, vp, i64, vp, i64, vp]),
        "dn_decoder_scores": (ctypes.c_int, [vp, i32, pp, ctypes.POINTER(i64), ctypes.POINTER(i64), vp]),
        "dn_decoder_status": (ctypes.c_int, [vp, ctypes.POINTER(i32), vp]),
        "sage_forward": (ctypes.c_int, [vp, vp, vp, vp, vp]),
        "sage_forward_table": (ctypes.c_int, [vp, vp, vp, i64, vp, vp]),
        "dn_model_set_aggregation": (ctypes.c_int, [vp, i32]),
        "sage_backward": (ctypes.c_int, [vp, vp, vp, pp, pp, pp, vp, vp]),
        "sage_backward_sgd": (ctypes.c_int, [vp, vp, vp, pp, pp, pp, vp, i64, ctypes.c_float, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise DenseError(rc, load_library().dn_last_error().decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev_ptr(t: Optional[torch.Tensor], dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous CUDA tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError("expected dtype %s, got %s" % (dtype, t.dtype))
    return t.data_ptr()


def _i32_array(values: Sequence[int]):
    return (ctypes.c_int32 * len(values))(*[int(v) for v in values])


def _ptr_array(tensors: Sequence[torch.Tensor]):
    return (ctypes.c_void_p * len(tensors))(*[_dev_ptr(t, torch.float32) for t in tensors])


def _alloc_workspace(nbytes: int, device) -> torch.Tensor:
    ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
    shift = (-ws.data_ptr()) % 256
    return ws[shift:shift + nbytes]


class Graph:
    """CSR by source (out-edges) and optionally by destination (in-edges), resident in HBM."""

    def __init__(self, rowptr_out: Optional[torch.Tensor], col_out: Optional[torch.Tensor],
                 rowptr_in: Optional[torch.Tensor] = None, col_in: Optional[torch.Tensor] = None):
        lib = load_library()
        ref = rowptr_out if rowptr_out is not None else rowptr_in
        self.num_nodes = ref.numel() - 1
        self._keep = (rowptr_out, col_out, rowptr_in, col_in)
        h = ctypes.c_void_p()
        _check(lib.dn_graph_create(ctypes.byref(h), self.num_nodes,
                                   _dev_ptr(rowptr_out, torch.int64), _dev_ptr(col_out, torch.int32),
                                   _dev_ptr(rowptr_in, torch.int64), _dev_ptr(col_in, torch.int32)))
        self.handle = h

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.dn_graph_destroy(self.handle)
            self.handle = None


class Batch:
    """One mini-batch slot: workspace sized for max_targets targets and the given fanouts."""

    def __init__(self, num_nodes: int, max_targets: int, fanouts: Sequence[int], direction: int = DN_DIR_OUT,
                 device="cuda"):
        lib = load_library()
        self.k = len(fanouts)
        self.fanouts = list(fanouts)
        self.direction = direction
        fan = _i32_array(fanouts)
        nbytes = ctypes.c_size_t()
        _check(lib.dn_batch_workspace_size(num_nodes, max_targets, self.k, fan, direction, ctypes.byref(nbytes)))
        self.workspace = _alloc_workspace(nbytes.value, device)
        h = ctypes.c_void_p()
        _check(lib.dn_batch_create(ctypes.byref(h), num_nodes, max_targets, self.k, fan, direction,
                                   self.workspace.data_ptr(), nbytes.value, _stream()))
        self.handle = h
        nc, sc = ctypes.c_int64(), ctypes.c_int64()
        _check(lib.dn_batch_capacity(h, ctypes.byref(nc), ctypes.byref(sc)))
        self.node_capacity, self.slot_capacity = nc.value, sc.value
        self._targets = None

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.dn_batch_destroy(self.handle)
            self.handle = None

    def prepare_backward(self, need_input_grad: bool = False) -> None:
        """Build the transpose index of the current sample now (on the current stream)."""
        _check(load_library().dn_batch_prepare_backward(self.handle, 1 if need_input_grad else 0, _stream()))

    def counts(self) -> List[int]:
        """[node_id_offsets[0..k+1]..., E]; waits for the stream."""
        buf = (ctypes.c_int64 * (self.k + 3))()
        _check(load_library().dn_batch_counts(self.handle, buf, _stream()))
        return list(buf)

    def _wrap(self, ptr: int, count: int) -> torch.Tensor:
        off = ptr - self.workspace.data_ptr()
        return self.workspace[off:off + 4 * count].view(torch.int32)

    def view(self):
        """The five DENSE arrays as int32 CUDA tensors aliasing the workspace (calls counts())."""
        c = self.counts()
        n, e, n0 = c[self.k + 1], c[self.k + 2], c[1]
        v = _View()
        _check(load_library().dn_batch_view(self.handle, ctypes.byref(v)))
        return {"node_id_offsets": self._wrap(v.node_id_offsets, self.k + 2),
                "node_ids": self._wrap(v.node_ids, n),
                "nbr_offsets": self._wrap(v.nbr_offsets, n - n0 + 1),
                "nbrs": self._wrap(v.nbrs, e),
                "repr_map": self._wrap(v.repr_map, e)}


class Model:
    """GraphSage-mean encoder bound to a batch's capacities."""

    def __init__(self, batch: Batch, dims: Sequence[int], in_dtype: int = DN_F32, device="cuda"):
        lib = load_library()
        self.k = len(dims) - 1
        self.dims = list(dims)
        self.in_dtype = in_dtype
        d = _i32_array(dims)
        nbytes = ctypes.c_size_t()
        _check(lib.dn_model_workspace_size(batch.handle, self.k, d, in_dtype, ctypes.byref(nbytes)))
        self.workspace = _alloc_workspace(nbytes.value, device)
        h = ctypes.c_void_p()
        _check(lib.dn_model_create(ctypes.byref(h), batch.handle, self.k, d, in_dtype, self.workspace.data_ptr(),
                                   nbytes.value, _stream()))
        self.handle = h

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.dn_model_destroy(self.handle)
            self.handle = None

    def set_aggregation(self, aggregation: int) -> None:
        """DN_AGG_MEAN (default) or DN_AGG_SUM (Algorithm 3 as printed)."""
        _check(load_library().dn_model_set_aggregation(self.handle, aggregation))

    def status(self):
        """(sign fix-ups of the last ReLU layer, queue-overflow flag); waits for the stream."""
        buf = (ctypes.c_int32 * 2)()
        _check(load_library().dn_model_status(self.handle, buf, _stream()))
        return int(buf[0]), int(buf[1])

    def set_weights(self, w_self: Sequence[torch.Tensor], w_nbr: Sequence[torch.Tensor], bias: Sequence[torch.Tensor]):
        for i in range(self.k):
            assert tuple(w_self[i].shape) == (self.dims[i], self.dims[i + 1]) == tuple(w_nbr[i].shape)
            assert tuple(bias[i].shape) == (self.dims[i + 1],)
        _check(load_library().dn_model_set_weights(self.handle, _ptr_array(w_self), _ptr_array(w_nbr),
                                                   _ptr_array(bias), _stream()))


class Decoder:
    """DistMult decoder with shared negatives: workspace for at most max_edges edges per call."""

    def __init__(self, max_edges: int, chunk: int, num_neg: int, dim: int, max_rows: int, num_rel: int, device="cuda"):
        lib = load_library()
        self.max_edges, self.chunk, self.num_neg, self.dim = max_edges, chunk, num_neg, dim
        self.max_rows, self.num_rel = max_rows, num_rel
        nbytes = ctypes.c_size_t()
        _check(lib.dn_decoder_workspace_size(max_edges, chunk, num_neg, dim, max_rows, num_rel, ctypes.byref(nbytes)))
        self.workspace = _alloc_workspace(nbytes.value, device)
        h = ctypes.c_void_p()
        _check(lib.dn_decoder_create(ctypes.byref(h), max_edges, chunk, num_neg, dim, max_rows, num_rel,
                                     self.workspace.data_ptr(), nbytes.value, _stream()))
        self.handle = h
        self._keep = None
        self._n_edges = 0

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.dn_decoder_destroy(self.handle)
            self.handle = None

    def status(self) -> int:
        """Flags of the last forward (1 = node index out of range, 2 = relation out of range); waits for the stream."""
        f = ctypes.c_int32()
        _check(load_library().dn_decoder_status(self.handle, ctypes.byref(f), _stream()))
        return int(f.value)

    def scores(self, side: int) -> torch.Tensor:
        """Negatives' scores of the last forward as a [n_edges x num_neg] view-copy (side 0: corrupted destination);
        the library computes them on this call (the forward pass keeps only each row's log-sum-exp)."""
        ptr, cs, rs = ctypes.c_void_p(), ctypes.c_int64(), ctypes.c_int64()
        _check(load_library().dn_decoder_scores(self.handle, side, ctypes.byref(ptr), ctypes.byref(cs), ctypes.byref(rs),
                                                _stream()))
        n_chunks = (self._n_edges + self.chunk - 1) // self.chunk
        off = ptr.value - self.workspace.data_ptr()
        flat = self.workspace[off:off + 4 * n_chunks * cs.value].view(torch.float32)
        full = flat.view(n_chunks, cs.value // rs.value, rs.value)[:, :self.chunk, :self.num_neg]
        return full.reshape(n_chunks * self.chunk, self.num_neg)[:self._n_edges]


def distmult_forward(dec: Decoder, h: torch.Tensor, r: torch.Tensor, src: torch.Tensor, rel: torch.Tensor,
                     dst: torch.Tensor, neg: torch.Tensor, pos: torch.Tensor, loss: torch.Tensor) -> None:
    """pos[e], loss[e] of the edges (src, rel, dst) with per-chunk shared negatives neg [chunks x num_neg]."""
    ne = src.numel()
    assert rel.numel() == ne and dst.numel() == ne and pos.numel() >= ne and loss.numel() >= ne
    assert h.dtype == torch.float32 and r.dtype == torch.float32 and h.stride(1) == 1 and r.stride(1) == 1
    assert h.shape[1] == dec.dim and r.shape[1] == dec.dim and r.shape[0] == dec.num_rel
    assert neg.numel() == ((ne + dec.chunk - 1) // dec.chunk) * dec.num_neg
    dec._keep = (h, r, src, rel, dst, neg)
    dec._n_edges = ne
    _check(load_library().distmult_forward(dec.handle, h.data_ptr(), h.stride(0), h.shape[0], r.data_ptr(), r.stride(0),
                                           _dev_ptr(src, torch.int32), _dev_ptr(rel, torch.int32),
                                           _dev_ptr(dst, torch.int32), ne, _dev_ptr(neg, torch.int32),
                                           _dev_ptr(pos, torch.float32), _dev_ptr(loss, torch.float32), _stream()))


def distmult_backward(dec: Decoder, d_h: torch.Tensor, d_r: torch.Tensor) -> None:
    """Gradients of sum(loss) of the last distmult_forward with respect to h and r."""
    assert d_h.dtype == torch.float32 and d_r.dtype == torch.float32 and d_h.stride(1) == 1 and d_r.stride(1) == 1
    assert d_h.shape == dec._keep[0].shape and tuple(d_r.shape) == (dec.num_rel, dec.dim)
    _check(load_library().distmult_backward(dec.handle, d_h.data_ptr(), d_h.stride(0), d_r.data_ptr(), d_r.stride(0),
                                            _stream()))


def profile_enable(on: bool) -> None:
    """Bracket every kernel launch of the library with HIP events (benchmark use)."""
    _check(load_library().dn_profile_enable(1 if on else 0))


def profile_calibration_copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    """Plain streaming copy of src into dst with the library's reference copy kernel."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(load_library().dn_profile_calibration_copy(_dev_ptr(dst), _dev_ptr(src), nbytes, _stream()))


def profile_step_stream_overlap(n_streams: int, kernel_us: int = 20) -> float:
    """Microseconds per round of one kernel_us-long single-wave kernel on each of dn_train_steps' first n_streams streams."""
    out = ctypes.c_double(0.0)
    _check(load_library().dn_profile_step_stream_overlap(n_streams, kernel_us, ctypes.byref(out)))
    return out.value


def profile_empty_bracket() -> None:
    """One event pair around nothing (tag "empty_bracket"): the cost of a bracket itself."""
    _check(load_library().dn_profile_empty_bracket(_stream()))


def profile_collect():
    """{tag: (total_ms, launches)} since profile_enable(True); waits for the device."""
    return {tag: (v[0], v[1]) for tag, v in profile_collect_percentiles().items()}


def profile_collect_percentiles():
    """{tag: (total_ms, launches, p10_ms, p50_ms, p90_ms)} since profile_enable(True); waits for the device."""
    buf = (_KernelTime * 128)()
    n = ctypes.c_int32()
    _check(load_library().dn_profile_collect(buf, 128, ctypes.byref(n)))
    return {buf[i].tag.decode(): (buf[i].total_ms, int(buf[i].launches), buf[i].p10_ms, buf[i].p50_ms, buf[i].p90_ms)
            for i in range(min(n.value, 128))}


def dense_sample(batch: Batch, graph: Graph, targets: torch.Tensor, seed: int) -> None:
    """Algorithm 1 on the device; results stay in the batch (see Batch.view / Batch.counts)."""
    n = targets.numel()
    batch._targets = targets
    _check(load_library().dense_sample(batch.handle, graph.handle, _dev_ptr(targets, torch.int32) if n else None,
                                       n, seed & 0xFFFFFFFFFFFFFFFF, _stream()))


def dense_sample_noalloc(graph: Graph, targets: torch.Tensor, fanouts: Sequence[int], direction: int, seed: int,
                         node_id_offsets: torch.Tensor, node_ids: torch.Tensor, nbr_offsets: torch.Tensor,
                         nbrs: torch.Tensor, repr_map: torch.Tensor, counts: torch.Tensor) -> None:
    """dense_sample into caller-provided int32 tensors, with the library's static scratch array as workspace."""
    n = targets.numel()
    assert node_id_offsets.numel() >= len(fanouts) + 2 and counts.numel() >= 3
    assert nbr_offsets.numel() >= node_ids.numel() + 1 and repr_map.numel() >= nbrs.numel()
    _check(load_library().dense_sample_noalloc(graph.handle, _dev_ptr(targets, torch.int32) if n else None, n, len(fanouts),
                                               _i32_array(fanouts), direction, seed & 0xFFFFFFFFFFFFFFFF,
                                               _dev_ptr(node_id_offsets, torch.int32), _dev_ptr(node_ids, torch.int32),
                                               _dev_ptr(nbr_offsets, torch.int32), node_ids.numel(),
                                               _dev_ptr(nbrs, torch.int32), _dev_ptr(repr_map, torch.int32), nbrs.numel(),
                                               _dev_ptr(counts, torch.int32), _stream()))


class TrainSteps:
    """A marshalled list of training steps for dn_train_steps (built once, run many times).  Each entry is a dict with
    batch, model, graph, targets, seed, table, out, labels, grad_scale, loss, grad_out, dws, dwn, dbs, dh0 (optional)."""

    def __init__(self, entries, forward_only: bool = False):
        self._keep = []
        self.array = (_TrainStep * len(entries))()
        for a, e in zip(self.array, entries):
            dws, dwn, dbs = _ptr_array(e["dws"]), _ptr_array(e["dwn"]), _ptr_array(e["dbs"])
            self._keep.append((e, dws, dwn, dbs))
            a.batch, a.model, a.graph = e["batch"].handle, e["model"].handle, e["graph"].handle
            a.targets, a.n_targets, a.seed = _dev_ptr(e["targets"], torch.int32), e["targets"].numel(), e["seed"] & 0xFFFFFFFFFFFFFFFF
            a.table, a.ld_elems = e["table"].data_ptr(), e["table"].stride(0)
            a.out, a.labels = _dev_ptr(e["out"], torch.float32), _dev_ptr(e["labels"], torch.int32)
            a.grad_scale, a.loss, a.grad_out = e["grad_scale"], _dev_ptr(e["loss"], torch.float32), _dev_ptr(e["grad_out"], torch.float32)
            a.dw_self = ctypes.cast(dws, ctypes.POINTER(ctypes.c_void_p))
            a.dw_nbr = ctypes.cast(dwn, ctypes.POINTER(ctypes.c_void_p))
            a.dbias = ctypes.cast(dbs, ctypes.POINTER(ctypes.c_void_p))
            a.dh0 = _dev_ptr(e.get("dh0"), torch.float32)
            a.forward_only = 1 if forward_only else 0

    def run(self, n_streams: int, first: int = 0, count: Optional[int] = None) -> None:
        """Steps first .. first+count-1 on n_streams library-owned streams, ordered behind / before the current stream."""
        count = len(self.array) - first if count is None else count
        ptr = ctypes.cast(ctypes.byref(self.array, first * ctypes.sizeof(_TrainStep)), ctypes.POINTER(_TrainStep))
        _check(load_library().dn_train_steps(ptr, count, n_streams, _stream()))


def dense_sample_edges(batch: Batch, graph: Graph, src: torch.Tensor, dst: torch.Tensor, neg: torch.Tensor, seed: int):
    """Targets = ascending distinct ids of src, dst, neg; returns their indices in the target list."""
    ne, nn = src.numel(), neg.numel()
    assert dst.numel() == ne
    batch._targets = (src, dst, neg)
    out = [torch.empty_like(src), torch.empty_like(dst), torch.empty_like(neg)]
    _check(load_library().dense_sample_edges(batch.handle, graph.handle,
                                             _dev_ptr(src, torch.int32) if ne else None,
                                             _dev_ptr(dst, torch.int32) if ne else None, ne,
                                             _dev_ptr(neg, torch.int32) if nn else None, nn, seed & 0xFFFFFFFFFFFFFFFF,
                                             _dev_ptr(out[0]) if ne else None, _dev_ptr(out[1]) if ne else None,
                                             _dev_ptr(out[2]) if nn else None, _stream()))
    return out


def embedding_sgd(batch: Batch, table: torch.Tensor, d_h0: torch.Tensor, lr: float) -> None:
    """table[node_ids[r]] -= lr * d_h0[r] for the batch's N nodes (fp32 table, rows may be strided)."""
    assert table.dtype == torch.float32 and table.stride(1) == 1 and d_h0.shape[1] == table.shape[1]
    _check(load_library().dn_embedding_sgd(batch.handle, table.data_ptr(), table.shape[1], table.stride(0),
                                           _dev_ptr(d_h0, torch.float32), lr, _stream()))


def embedding_adagrad(batch: Batch, table: torch.Tensor, state: torch.Tensor, d_h0: torch.Tensor, lr: float,
                      eps: float) -> None:
    """Adagrad step on the rows of `table` that the batch touched; `state` has the table's shape and strides."""
    assert table.dtype == torch.float32 and state.dtype == torch.float32 and table.stride(1) == 1
    assert state.shape == table.shape and state.stride() == table.stride() and d_h0.shape[1] == table.shape[1]
    _check(load_library().dn_embedding_adagrad(batch.handle, table.data_ptr(), state.data_ptr(), table.shape[1],
                                               table.stride(0), _dev_ptr(d_h0, torch.float32), lr, eps, _stream()))


def softmax_xent(logits: torch.Tensor, labels: torch.Tensor, loss: torch.Tensor, grad: torch.Tensor,
                 grad_scale: float = 1.0) -> None:
    """loss[i], grad[i, :] of the softmax cross-entropy of logits[i, :] against labels[i]."""
    n, c = logits.shape
    assert logits.dtype == torch.float32 and grad.dtype == torch.float32 and logits.stride(1) == 1 and grad.stride(1) == 1
    assert grad.shape == logits.shape and labels.numel() == n and loss.numel() >= n
    _check(load_library().dn_softmax_xent(logits.data_ptr(), logits.stride(0), _dev_ptr(labels, torch.int32), n, c,
                                          grad_scale, _dev_ptr(loss, torch.float32), grad.data_ptr(), grad.stride(0),
                                          _stream()))


def dense_gather(batch: Batch, table: torch.Tensor, out: torch.Tensor) -> torch.Tensor:
    """out[r] = table[node_ids[r]] for the batch's N nodes; out has node_capacity rows."""
    dtype = {torch.float32: DN_F32, torch.bfloat16: DN_BF16}[table.dtype]
    assert out.dtype == table.dtype and out.shape[1] == table.shape[1] and out.shape[0] >= batch.node_capacity
    assert table.stride(1) == 1
    _check(load_library().dense_gather(batch.handle, table.data_ptr(), dtype, table.shape[1], table.stride(0),
                                       _dev_ptr(out), _stream()))
    return out


def sage_forward(model: Model, batch: Batch, h0: torch.Tensor, out: torch.Tensor) -> torch.Tensor:
    """out[t] = H^k of target t (fp32 [n_targets x dims[k]])."""
    want = torch.float32 if model.in_dtype == DN_F32 else torch.bfloat16
    assert h0.dtype == want and h0.shape[1] == model.dims[0] and h0.shape[0] >= batch.node_capacity
    assert out.shape[1] == model.dims[-1]
    _check(load_library().sage_forward(model.handle, batch.handle, _dev_ptr(h0), _dev_ptr(out, torch.float32), _stream()))
    return out


def sage_forward_table(model: Model, batch: Batch, table: torch.Tensor, out: torch.Tensor) -> torch.Tensor:
    """sage_forward reading the feature table's rows directly (no dense_gather, no H^0 buffer)."""
    want = torch.float32 if model.in_dtype == DN_F32 else torch.bfloat16
    assert table.dtype == want and table.shape[1] == model.dims[0] and table.stride(1) == 1
    assert out.shape[1] == model.dims[-1]
    _check(load_library().sage_forward_table(model.handle, batch.handle, table.data_ptr(), table.stride(0),
                                             _dev_ptr(out, torch.float32), _stream()))
    return out


def sage_backward(model: Model, batch: Batch, grad_out: torch.Tensor, d_w_self: Sequence[torch.Tensor],
                  d_w_nbr: Sequence[torch.Tensor], d_bias: Sequence[torch.Tensor],
                  d_h0: Optional[torch.Tensor] = None) -> None:
    if d_h0 is not None:
        assert d_h0.shape[0] >= batch.node_capacity and d_h0.shape[1] == model.dims[0]
    _check(load_library().sage_backward(model.handle, batch.handle, _dev_ptr(grad_out, torch.float32),
                                        _ptr_array(d_w_self), _ptr_array(d_w_nbr), _ptr_array(d_bias),
                                        _dev_ptr(d_h0, torch.float32), _stream()))


def sage_backward_sgd(model: Model, batch: Batch, grad_out: torch.Tensor, d_w_self: Sequence[torch.Tensor],
                      d_w_nbr: Sequence[torch.Tensor], d_bias: Sequence[torch.Tensor], table: torch.Tensor,
                      lr: float) -> None:
    """sage_backward that applies the SGD step of the learnable input rows to `table` instead of writing dL/dH^0."""
    assert table.dtype == torch.float32 and table.stride(1) == 1 and table.shape[1] == model.dims[0]
    _check(load_library().sage_backward_sgd(model.handle, batch.handle, _dev_ptr(grad_out, torch.float32),
                                            _ptr_array(d_w_self), _ptr_array(d_w_nbr), _ptr_array(d_bias),
                                            table.data_ptr(), table.stride(0), lr, _stream()))
