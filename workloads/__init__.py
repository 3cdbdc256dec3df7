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
                      class_labels, softmax_xent_grad)

__all__ = ["CONFIGS", "WorkloadConfig", "get_config", "rmat_csr", "transpose_csr", "mix64",
           "feature_table", "glorot_weights", "target_batch", "training_subset",
           "class_labels", "softmax_xent_grad"]
