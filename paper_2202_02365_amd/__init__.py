"""MI355X-native DENSE mini-batch construction + GraphSage-mean encoder (arXiv 2202.02365 hot path).

Thin Python binding over libdense_mi355x.so (hand-written HIP for gfx950).  Argument
marshalling only: every step runs in the library's kernels.  PyTorch supplies device memory
and streams.  There is no CPU fallback: if the library is missing, loading raises.
"""
from .binding import (DN_F32, DN_BF16, DN_DIR_OUT, DN_DIR_IN, DN_DIR_BOTH, DenseError, Graph, Batch, Model, Decoder, distmult_forward, distmult_backward,
                      dense_sample, dense_sample_noalloc, TrainSteps, dense_sample_edges, embedding_sgd, embedding_adagrad, softmax_xent, dense_gather, sage_forward, sage_forward_table, sage_backward, sage_backward_sgd, DN_AGG_MEAN, DN_AGG_SUM, library_path, load_library,
                      declared_symbols, profile_enable, profile_collect, profile_collect_percentiles,
                      profile_calibration_copy, profile_empty_bracket, profile_step_stream_overlap)

__all__ = ["DN_F32", "DN_BF16", "DN_DIR_OUT", "DN_DIR_IN", "DN_DIR_BOTH", "DenseError", "Graph", "Batch", "Model", "Decoder", "distmult_forward", "distmult_backward",
           "dense_sample", "dense_sample_noalloc", "TrainSteps", "dense_sample_edges", "embedding_sgd", "embedding_adagrad", "softmax_xent", "dense_gather", "sage_forward", "sage_forward_table", "sage_backward", "sage_backward_sgd", "DN_AGG_MEAN", "DN_AGG_SUM", "library_path", "load_library",
           "declared_symbols", "profile_enable", "profile_collect", "profile_collect_percentiles", "profile_calibration_copy", "profile_empty_bracket", "profile_step_stream_overlap"]
