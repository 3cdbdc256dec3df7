"""Every kernel tag the library brackets for bench.py's per-kernel timing must have an algorithmic byte or flop count
in bench.algorithmic_work, so that the roofline object is chosen over ALL kernels of the step (host logic only)."""
import os
import re
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def source_tags():
    """Tags passed to dn_prof_scope in the library's sources: (tag, has_layer_suffix)."""
    tags = set()
    csrc = os.path.join(ROOT, "paper_2202_02365_amd", "csrc")
    for name in os.listdir(csrc):
        if not name.endswith(".hip"):
            continue
        text = open(os.path.join(csrc, name)).read()
        for m in re.finditer(r'dn_prof_scope ps\(([^;]*)\);', text):
            args = m.group(1)
            layered = not re.search(r',\s*0\s*,\s*st\s*$', args)
            for t in re.findall(r'"(\w+)"', args):
                tags.add((t, layered))
    return tags


def test_every_node_classification_tag_has_a_formula():
    import bench
    from workloads import get_config
    cfg = get_config("rmat1m")
    k = cfg.num_layers
    # one made-up mini-batch: node_id_offsets[0..k+1], E, S_1..S_k (slots owned by Delta_i..Delta_k)
    sizes = [[0, 90000, 105000, 107000, 108000, 120000, 120000, 40000, 3000]]
    assert len(sizes[0]) == k + 3 + k
    # tags that only time the bracket itself, or kernels of the link-prediction decoder / optimiser steps (their step
    # reports per-stage times, not a per-kernel roofline)
    not_in_step = {"empty_bracket", "noop_kernel_bracket", "embedding_sgd", "embedding_adagrad", "mark_ids", "local_ids"}
    missing = []
    tags = source_tags() | {("gemm_fwd", True), ("gemm_dx", True)}      # these two reach dn_prof_scope through a variable
    assert {"sample_hop", "next_delta_hop", "assemble", "transpose_index", "aggregate_bwd", "sage_layer", "gemm_dw_all"} <= {t for t, _ in tags}
    for tag, layered in sorted(tags):
        if tag in not_in_step or tag.startswith("dm_"):
            continue
        names = ["%s_L%d" % (tag, i) for i in range(1, k + 1)] if layered else [tag]
        for n in names:
            bound, work = bench.algorithmic_work(n, sizes, cfg, cfg.dims)
            if work is None or not np.isfinite(work) or work <= 0:
                missing.append(n)
    assert not missing, "no algorithmic work for: %s" % missing
