"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This package holds input generators only: R-MAT graphs in CSR/CSC form, feature tables,
Glorot weights, target batches.  None of the method's arithmetic (sampling, DENSE
assembly, aggregation, linear layers) lives here, and nothing here imports either the
oracle or the HIP binding.

All randomness that decides graph *structure* comes from an integer hash evaluated with
wrapping int64 tensor ops, so the same graph is produced on the host and on the device.
"""
from .configs import CONFIGS, WorkloadConfig, get_config
from .rmat import rmat_csr, transpose_csr, mix64
from .tensors import (feature_table, glorot_weights, target_batch, training_subset,
                      class_labels, decoder_inputs, edge_batch, relation_embeddings)



def make_inputs(cfg, device, n_batches: int = 64, log=None):
    """Graph (CSR, plus CSC when the workload samples in-edges), feature table, Glorot weights and
    `n_batches` target batches of a workload.  Graphs and tables beyond a few million nodes are
    generated on `device` (they need not exist on the host); everything is returned on `device`,
    the target batches and weights as NumPy arrays."""
    import time
    import torch
    t0 = time.time()
    big = cfg.num_nodes > (1 << 22)
    gen_dev = device if big else "cpu"
    rowptr, col = rmat_csr(cfg.num_nodes, cfg.num_edges, cfg.graph_seed, device=gen_dev)
    rowptr_in = col_in = None
    if cfg.direction != 0:
        rowptr_in, col_in = transpose_csr(rowptr, col)
    if big and torch.cuda.is_available():
        torch.cuda.empty_cache()
    if log:
        log("graph: V=%d E=%d (nominal %d) on %s in %.1fs" % (cfg.num_nodes, col.numel(), cfg.num_edges, gen_dev,
                                                              time.time() - t0))
    t0 = time.time()
    table = feature_table(cfg.num_nodes, cfg.feat_dim, cfg.feat_dtype, cfg.feat_seed, device=gen_dev)
    if log:
        log("features: %d x %d %s in %.1fs" % (cfg.num_nodes, cfg.feat_dim, cfg.feat_dtype, time.time() - t0))
    pool = training_subset(cfg.num_nodes, cfg.train_fraction, cfg.target_seed, device=gen_dev)
    targets = [target_batch(pool.numel(), cfg.batch, bi, cfg.target_seed,
                            pool=pool if cfg.train_fraction < 1 else None) for bi in range(n_batches)]
    weights = glorot_weights(cfg.dims, cfg.weight_seed)
    to = lambda t: None if t is None else t.to(device)
    return dict(rowptr=to(rowptr), col=to(col), rowptr_in=to(rowptr_in), col_in=to(col_in), table=to(table),
                targets=targets, weights=weights)


__all__ = ["make_inputs", "CONFIGS", "WorkloadConfig", "get_config", "rmat_csr", "transpose_csr", "mix64",
           "feature_table", "glorot_weights", "target_batch", "training_subset",
           "class_labels", "decoder_inputs", "edge_batch", "relation_embeddings"]
