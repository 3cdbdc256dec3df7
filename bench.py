#!/usr/bin/env python3
"""Benchmark of the DENSE hot path on one MI355X.

One step = one mini-batch through every step of the path: dense_sample (3-hop DENSE
construction) -> gather of H^0 (inside sage_forward_table, or dense_gather with --separate-gather)
-> forward -> softmax cross-entropy head -> sage_backward, on synthetic inputs that
are resident in HBM before the clock starts.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload rmat111m|rmat1m|rmat16k|...]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published
N_BATCHES = 64                  # distinct target batches cycled through, sampling seed = batch index


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


REPEATS = 5     # every timed block of K steps is run this often; the median block is reported


def median_seconds(timed_block, repeats=REPEATS):
    """Median of `repeats` runs of a block that times exactly K steps between two device synchronisations (a single
    block of 20 steps is a 3 ms window; the median of five keeps one slow block from deciding the figure)."""
    import numpy as np
    times = sorted(timed_block() for _ in range(repeats))
    return float(np.median(times)), times


def dw_effective_splits(rows, kx, d_out, zterms, tile=128, max_splits=64, min_chunks=8, target_blocks=256):
    """Reduction splits the weight-gradient GEMM of a layer actually uses for `rows` rows (the library chooses them on
    the device: enough workgroups to fill the chip by capacity, then at least `min_chunks` k-steps of 64 rows per
    split; every bf16 term of dZ has its own splits)."""
    tiles = -(-kx // tile) * -(-d_out // tile) * zterms
    by_capacity = min(max_splits, -(-target_blocks // tiles))
    chunks = -(-int(rows) // 64)
    return max(1, min(by_capacity, chunks // min_chunks))


def algorithmic_work(tag, sizes, cfg, dims):
    """Algorithmic bytes (HBM-bound kernels) or flops (GEMMs) of ONE launch of the kernel `tag`, averaged over the
    batches.  sizes = per batch [node_id_offsets[0..k+1], E, S_1..S_k] with S_i = neighbour slots owned by
    Delta_i..Delta_k (what layer i aggregates over).  Byte counts follow the data each step has to touch once:
    16 B of row offsets per frontier node and direction, 4 B per adjacency entry read, 4 B per array entry written,
    one 8-byte bitmap pair per claimed neighbour, a feature row per row read or written."""
    import numpy as np
    k = cfg.num_layers
    elt0 = 4 if cfg.feat_dtype == "f32" else 2
    ndir = 2 if cfg.direction == 2 else 1
    off = np.array([s[:k + 2] for s in sizes], dtype=np.float64)      # [batches, k+2]
    E = np.array([s[k + 2] for s in sizes], dtype=np.float64)
    S = np.array([list(s[k + 3:k + 3 + k]) + [0.0] for s in sizes], dtype=np.float64)   # S[:, i-1] = S_i, S_{k+1} = 0
    N = off[:, k + 1]
    mean = lambda x: float(np.mean(x))

    def level_nodes(h):                    # level h = Delta_{k-h}
        return off[:, k - h + 1] - off[:, k - h]

    def hop_slots(h):                      # slots owned by level h
        return S[:, k - h - 1] - S[:, k - h]

    def layer_of(t):
        return int(t.split("_L")[1])

    if tag == "gather":
        return "hbm", mean(2 * N * dims[0] * elt0)
    if tag == "init_targets":
        return "hbm", mean(level_nodes(0) * (4 + 16 * ndir + 8 + 12))
    if tag == "init_offsets":
        return "hbm", mean(level_nodes(0) * 8)
    if tag == "init_level0":                  # both steps in one launch (target lists of a few thousand ids)
        return "hbm", mean(level_nodes(0) * (4 + 16 * ndir + 8 + 12 + 4))
    if tag in ("mark_ids", "local_ids") and cfg.lp_edges:
        ids = 2.0 * cfg.lp_edges + cfg.lp_edges // cfg.lp_chunk * cfg.lp_negatives
        return "hbm", ids * 12.0
    if tag.startswith("sample_hop_L"):
        h = layer_of(tag) - 1
        return "hbm", mean(level_nodes(h) * (8 + 16 * ndir) + hop_slots(h) * (4 + 8 + 8))
    if tag.startswith("fresh_count_hop") or tag.startswith("fresh_emit_hop") or tag.startswith("next_delta_hop"):
        # next_delta_hop: count and emit in one launch (the walk's words are read once from memory)
        h = layer_of(tag) if "_L" in tag else 0      # forms level h (0: the link-prediction front end's targets)
        new = level_nodes(h)
        rowptr = 16 * ndir if h < k else 0
        walk = cfg.num_nodes / 1024.0 * 4 + new * 8
        if tag.startswith("fresh_count"):
            return "hbm", mean(walk + new * rowptr)
        return "hbm", mean(walk + new * (8 + 12 + rowptr))
    if tag == "assemble":
        return "hbm", mean(12 * N + 20 * E)
    if tag == "transpose_index":
        need_all = cfg.name.endswith("_lp")
        pairs = E if need_all else (S[:, 1] if k >= 2 else 0 * E)
        cap_nodes = cfg.capacity()[0]
        passes = -(-max(1, int(np.ceil(np.log2(max(cap_nodes, 2))))) // 11)
        return "hbm", mean(pairs * (8 + 16 * passes + 12) + (N + 1) * 4)
    if tag.startswith("aggregate_L") or tag.startswith("aggregate_table_L"):
        # aggregate_table_L1 reads the same rows from the feature table itself (plus 4 B of node id per row read)
        i = layer_of(tag)
        rows = N - off[:, i]
        slots = S[:, i - 1]
        elt = elt0 if i == 1 else 4
        d = dims[i - 1]
        terms = 1 if i == 1 else 2
        ids = 4 * rows if "table" in tag else 0
        return "hbm", mean((slots + rows) * d * elt + slots * 4 + ids + rows * 2 * d * terms * 2)
    if tag.startswith("aggregate_bwd_L"):
        i = layer_of(tag)
        d = dims[i - 1]
        rows_in, rows_out, slots = N - off[:, i - 1], N - off[:, i], S[:, i - 1]
        read = slots * (d * 4 + 12) + rows_out * d * 4 + rows_in * 8
        if i >= 2:
            np_pad = -(-dims[i - 1] // 64) * 64
            write = rows_in * (d * 4 + 2 * np_pad * 2)           # ReLU mask row read, dZ of the layer below as two bf16 terms
        elif cfg.name.endswith("_lp"):
            write = rows_in * (2 * d * 4 + 4)                    # fused SGD: table row read and written, node id
        else:
            write = rows_in * d * 4
        return "hbm", mean(read + write)
    if tag.startswith("dz_L"):
        i = layer_of(tag)
        zt = 1 if i == k else 2
        return "hbm", mean((N - off[:, i]) * dims[i] * (4 + 2 * zt))
    if tag == "bwd_reduce_all":
        total = 0.0
        for i in range(1, k + 1):
            xt, zt = (1 if i == 1 else 2), (1 if i == k else 2)
            kx = 2 * dims[i - 1] * xt
            eff = np.array([dw_effective_splits(r, kx, dims[i], zt) for r in (N - off[:, i])], dtype=np.float64)
            total = total + eff * zt * kx * dims[i] * 4 + 2 * dims[i - 1] * dims[i] * 4
        return "hbm", mean(total)
    if tag == "softmax_xent":
        return "hbm", float(cfg.batch * (dims[-1] * 8 + 8))
    if tag in ("embedding_sgd", "embedding_adagrad"):
        return "hbm", mean(N * dims[0] * 4 * (3 if tag.endswith("sgd") else 5))
    if tag.startswith("gemm_fwd_L") or tag.startswith("sage_layer_L"):
        # sage_layer_L*: aggregation and linear map of a layer above the first in one launch; the contraction is the same
        i = layer_of(tag)
        rows = N - off[:, i]
        terms = 1 if i == 1 else 2
        return "mfma", mean(2 * rows * (2 * dims[i - 1] * terms) * dims[i])
    if tag == "gemm_dw_all":               # the dW GEMMs of all layers share one launch
        total = 0.0
        for i in range(1, k + 1):
            rows = N - off[:, i]
            xt = 1 if i == 1 else 2
            zt = 1 if i == k else 2
            total = total + 2 * rows * (2 * dims[i - 1] * xt) * dims[i] * zt
        return "mfma", mean(total)
    if tag.startswith("gemm_dx_L"):
        i = layer_of(tag)
        rows = N - off[:, i]
        zt = 1 if i == k else 2
        return "mfma", mean(2 * rows * (2 * dims[i - 1]) * dims[i] * zt)
    if tag.startswith("dm_") and cfg.lp_edges:
        pairs = 2.0 * cfg.lp_edges * cfg.lp_negatives            # (edge, negative) pairs of both corrupted sides
        d = dims[-1]
        if tag == "dm_gemm_scores":
            return "mfma", 2.0 * pairs * d
        if tag in ("dm_gemm_dq", "dm_gemm_de"):                  # probabilities enter as two bf16 terms
            return "mfma", 2.0 * pairs * d * 2
        if tag == "dm_probs":                                    # the scores again; writes the probabilities as two bf16 terms
            return "hbm", pairs * 2 * 2
    return "hbm", None


def gemm_algorithmic_bytes(tag, sizes, cfg, dims):
    """Operand + result bytes of one launch of a GEMM kernel (weights left out: a few hundred KB), for the
    arithmetic intensity that tells whether the MFMA or the HBM roofline is the lower one at this shape."""
    import numpy as np
    k = cfg.num_layers
    off = np.array([s[:k + 2] for s in sizes], dtype=np.float64)
    N = off[:, k + 1]

    def layer(i):
        rows = N - off[:, i]
        xt = 1 if i == 1 else 2                  # bf16 terms of the layer's input operand [self | mean]
        zt = 1 if i == k else 2                  # bf16 terms of dZ
        return rows, 2 * dims[i - 1], dims[i], xt, zt

    if tag.startswith("gemm_fwd_L"):
        rows, kk, n, xt, _ = layer(int(tag.split("_L")[1]))
        return float(np.mean(rows * kk * xt * 2 + rows * n * 4))
    if tag.startswith("sage_layer_L"):
        # input rows read per slot and per output row, slot list, X written for the backward pass, output rows, weights
        i = int(tag.split("_L")[1])
        rows, kk, n, xt, _ = layer(i)
        slots = np.array([s[k + 2 + i] for s in sizes], dtype=np.float64)
        return float(np.mean((slots + rows) * dims[i - 1] * 4 + slots * 4 + rows * kk * xt * 2 + rows * n * 4 + n * kk * 2))
    if tag.startswith("gemm_dx_L"):
        rows, kk, n, _, zt = layer(int(tag.split("_L")[1]))
        return float(np.mean(rows * n * zt * 2 + rows * kk * 4))
    if tag == "gemm_dw_all":
        total = 0.0
        for i in range(1, k + 1):
            rows, kk, n, xt, zt = layer(i)
            total = total + rows * kk * xt * 2 + rows * n * zt * 2
        return float(np.mean(total))
    return None


FORWARD_TAGS = ("init_", "sample_hop", "fresh_", "next_delta", "assemble", "mark_ids", "local_ids", "gather", "aggregate_L",
                "aggregate_table_L", "gemm_fwd_L", "sage_layer_L")


def pick_dominant(candidates, forward_chain_timed):
    """The kernel the roofline object is reported for: the one with the largest share of the kernel time of the
    whole run, as the rocprofv3 summary of the same command ranks them.  The run times the forward-only chain
    (sample + gather + forward) as often as the whole step, so a kernel of that chain is launched twice as often as
    one of the backward pass."""
    if not candidates:
        return None
    def weight(c):
        return c[0] * (2.0 if forward_chain_timed and c[1].startswith(FORWARD_TAGS) else 1.0)
    return max(candidates, key=weight)


def measured_traffic(workload, tag):
    """HBM bytes per launch of kernel `tag` from the committed rocprofv3 counter summary (FETCH_SIZE +
    WRITE_SIZE, each scaled by a plain copy of known size), or None if there is none for this workload."""
    path = os.path.join(ROOT, "profiles", "%s_hbm_traffic.txt" % workload)
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 2 and parts[0] == tag:
            return float(parts[1])
    return None


def host_description():
    """CPU model, usable cores and the C oracle's compiler flags, stated beside every oracle timing."""
    import oracle
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    return {"cpu_model": model, "nproc": os.cpu_count(), "usable_cores": usable,
            "omp_num_threads_env": os.environ.get("OMP_NUM_THREADS"),
            "c_oracle_build": "gcc " + " ".join(oracle.GCC_FLAGS) + " (OpenMP leg: the same plus -fopenmp)"}


def blas_threads():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] + [1]))
    except Exception:
        return os.cpu_count() or 1


def cpu_baseline(cfg, inputs, sizes, budget_s=16.0):
    """The oracle as it stands, timed on the host: sample + gather + forward + backward per batch with the
    single-threaded C sampler, then the sampler alone again from the OpenMP build of the same source."""
    import numpy as np
    import torch
    import oracle
    from workloads import class_labels
    t0 = time.time()
    g = oracle.Graph(cfg.num_nodes, inputs["rowptr"].cpu().numpy(), inputs["col"].cpu().numpy(),
                     None if inputs["rowptr_in"] is None else inputs["rowptr_in"].cpu().numpy(),
                     None if inputs["col_in"] is None else inputs["col_in"].cpu().numpy())
    log("cpu_baseline: graph copied to the host in %.1fs" % (time.time() - t0))
    w_self, w_nbr, bias = inputs["weights"]
    params = oracle.SageParams(w_self, w_nbr, bias)
    table = inputs["table"]
    labels = class_labels(cfg.batch, cfg.dims[-1])
    done, edges, spent = 0, 0, 0.0
    stage = {"sample": 0.0, "gather": 0.0, "forward": 0.0, "backward": 0.0}
    while done < N_BATCHES and (done < 2 or spent < budget_s):
        targets = inputs["targets"][done]
        t0 = time.time()
        d = oracle.dense_sample(g, targets, cfg.fanouts, seed=done, direction=cfg.direction)
        t1 = time.time()
        rows = table[torch.from_numpy(d.node_ids.astype(np.int64)).to(table.device)].float().cpu().numpy()
        t2 = time.time()                                 # device->host row fetch stands in for the host-side gather
        st = oracle.sage_forward(d, rows, params, mode="bf16")
        t3 = time.time()
        gout = oracle.mean_xent_grad(st.out, labels[:len(targets)])
        oracle.sage_backward(st, params, gout, mode="bf16")
        t4 = time.time()
        for name, dt in zip(("sample", "gather", "forward", "backward"), (t1 - t0, t2 - t1, t3 - t2, t4 - t3)):
            stage[name] += dt
        spent += t4 - t0
        edges += len(d.nbrs)
        done += 1
        log("cpu_baseline: batch %d, %.2fs so far" % (done, spent))
    # the sampler alone on all cores (Section 4.1 runs the one-hop samples of a level on several threads)
    host = host_description()
    omp_threads = int(os.environ.get("OMP_NUM_THREADS") or host["usable_cores"])
    omp_done, omp_edges, omp_spent = 0, 0, 0.0
    oracle.use_openmp(True)
    try:
        while omp_done < N_BATCHES and (omp_done < 2 or omp_spent < 4.0):
            t0 = time.time()
            d = oracle.dense_sample(g, inputs["targets"][omp_done], cfg.fanouts, seed=omp_done, direction=cfg.direction)
            omp_spent += time.time() - t0
            omp_edges += len(d.nbrs)
            omp_done += 1
    finally:
        oracle.use_openmp(False)
    threads = blas_threads()
    return {"value": edges / spent, "unit": "sampled edges/s", "cores": int(threads), "kind": "oracle",
            "sample": "%d mini-batches of the same workload (sample+gather+forward+backward, %.1f s; C sampler is "
                      "single-threaded, NumPy GEMMs use the BLAS threads counted in cores; feature rows fetched "
                      "from the device table)" % (done, spent),
            "mini_batches_per_s": done / spent,
            "seconds_per_batch_by_stage": {name: t / done for name, t in stage.items()},
            "sampler_alone": {"single_thread_edges_per_s": edges / stage["sample"],
                              "openmp_edges_per_s": omp_edges / omp_spent, "openmp_threads": omp_threads,
                              "openmp_batches": omp_done,
                              "note": "the OpenMP build parallelises the per-node one-hop samples of a level; computing "
                                      "the next Delta and the concatenations stay serial"},
            "host": host,
            "note": "a plain oracle, not a tuned CPU baseline"}


def run_link_prediction(args, cfg):
    """Link-prediction step: dense_sample_edges -> sage_forward_table -> distmult_forward -> distmult_backward ->
    sage_backward_sgd, one batch of positive edges per step (--separate-gather: dense_gather + sage_forward and
    sage_backward with dL/dH^0 + dn_embedding_sgd instead of the two fused calls)."""
    import numpy as np
    import torch
    import paper_2202_02365_amd as dn
    from workloads import make_inputs, edge_batch, relation_embeddings

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    inputs = make_inputs(cfg, dev, 1, log)
    k, dims = cfg.num_layers, cfg.dims
    n_batches = 16
    B, chunk, Nn, num_rel = cfg.lp_edges, cfg.lp_chunk, cfg.lp_negatives, cfg.num_relations
    graph = dn.Graph(inputs["rowptr"], inputs["col"], inputs["rowptr_in"], inputs["col_in"])
    table = inputs["table"]
    w_self, w_nbr, bias = [[torch.from_numpy(a).to(dev) for a in group] for group in inputs["weights"]]
    R = torch.from_numpy(relation_embeddings(num_rel, dims[-1])).to(dev)
    batches = [edge_batch(inputs["rowptr"], inputs["col"], cfg.num_nodes, B, chunk, Nn, num_rel, bi) for bi in range(n_batches)]
    lr = 1e-3

    def make_slot():
        b = dn.Batch(cfg.num_nodes, cfg.batch, cfg.fanouts, cfg.direction)
        m = dn.Model(b, dims, dn.DN_F32)
        m.set_weights(w_self, w_nbr, bias)
        return dict(batch=b, model=m, dec=dn.Decoder(B, chunk, Nn, dims[-1], cfg.batch, num_rel),
                    h0=torch.empty((b.node_capacity, dims[0]), device=dev) if args.separate_gather else None,
                    out=torch.empty((cfg.batch, dims[-1]), device=dev),
                    pos=torch.empty(B, device=dev), loss=torch.empty(B, device=dev),
                    g_out=torch.empty((cfg.batch, dims[-1]), device=dev), g_rel=torch.empty((num_rel, dims[-1]), device=dev),
                    dws=[torch.empty_like(w) for w in w_self], dwn=[torch.empty_like(w) for w in w_nbr],
                    dbs=[torch.empty_like(x) for x in bias],
                    dh0=torch.empty((b.node_capacity, dims[0]), device=dev) if args.separate_gather else None,
                    stream=torch.cuda.Stream())

    def step(o, bi, update=True):
        src, rel, dst, neg = batches[bi % n_batches]
        ls, ld, ln = dn.dense_sample_edges(o["batch"], graph, src, dst, neg.reshape(-1), bi)
        if args.separate_gather:
            dn.dense_gather(o["batch"], table, o["h0"])
            dn.sage_forward(o["model"], o["batch"], o["h0"], o["out"])
        else:
            dn.sage_forward_table(o["model"], o["batch"], table, o["out"])
        dn.distmult_forward(o["dec"], o["out"], R, ls, rel, ld, ln.view(-1, Nn), o["pos"], o["loss"])
        dn.distmult_backward(o["dec"], o["g_out"], o["g_rel"])
        if args.separate_gather:
            dn.sage_backward(o["model"], o["batch"], o["g_out"], o["dws"], o["dwn"], o["dbs"], o["dh0"])
            if update:
                dn.embedding_sgd(o["batch"], table, o["dh0"], lr)
        else:
            # the layer-1 input gradient is applied to the table as it is formed: no dL/dH^0 buffer
            dn.sage_backward_sgd(o["model"], o["batch"], o["g_out"], o["dws"], o["dwn"], o["dbs"], table, lr)

    slot = make_slot()
    sizes = []
    for bi in range(n_batches):
        src, rel, dst, neg = batches[bi]
        dn.dense_sample_edges(slot["batch"], graph, src, dst, neg.reshape(-1), bi)
        c = slot["batch"].counts()
        sizes.append(c + [c[k + 2]])                 # one layer: every slot is aggregated by layer 1
    mean_n = float(np.mean([s[k + 1] for s in sizes]))
    mean_e = float(np.mean([s[k + 2] for s in sizes]))
    log("mini-batch sizes: mean N=%.0f, mean E=%.0f, %d positive edges, %d x %d negatives" % (mean_n, mean_e, B, B // chunk, Nn))

    def timed(n_steps, slots):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(n_steps):
            o = slots[s % len(slots)]
            with torch.cuda.stream(o["stream"]):
                step(o, s)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    steps, warmup = args.steps, args.warmup
    timed(warmup, [slot])
    serial_s, _ = median_seconds(lambda: timed(steps, [slot]), 3)
    total_s, in_flight = serial_s, "1 mini-batch"
    if args.replicas > 1:
        # replicas update the shared embedding table without waiting for each other (rows of concurrent batches
        # rarely coincide; the paper's pipeline applies such updates with bounded staleness too, Section 3)
        slots = [slot] + [make_slot() for _ in range(args.replicas - 1)]
        timed(max(warmup, len(slots)), slots)
        rep_s, _ = median_seconds(lambda: timed(steps, slots), 3)
        log("%d replicas: %.3f ms/step; one at a time: %.3f ms/step" % (len(slots), 1e3 * rep_s / steps, 1e3 * serial_s / steps))
        if rep_s < total_s:
            total_s, in_flight = rep_s, "%d mini-batches, each on a stream of its own, launched eagerly" % len(slots)
        del slots
    edges = sum(sizes[s % n_batches][k + 2] for s in range(steps))
    if slot["model"].status()[1] != 0:
        raise RuntimeError("the ReLU sign fix-up queue overflowed during the timed run")

    roofline, kernels = None, {}
    if not args.no_kernel_times:
        delay_src = torch.empty(256 << 20, dtype=torch.float32, device=dev)
        delay_dst = torch.empty_like(delay_src)
        dn.profile_enable(True)
        torch.cuda.synchronize()
        for s in range(steps):
            dn.profile_calibration_copy(delay_dst, delay_src)
            dn.profile_empty_bracket()
            step(slot, s)
        prof_pct = dn.profile_collect_percentiles()
        prof = {tag: (v[0], v[1]) for tag, v in prof_pct.items()}
        dn.profile_enable(False)
        del delay_src, delay_dst
        empty_ms, empty_n = prof.pop("empty_bracket", (0.0, 1))
        prof.pop("noop_kernel_bracket", None)
        bracket_us = 1e3 * empty_ms / max(empty_n, 1)
        noop_us = 1e3 * (prof_pct["noop_kernel_bracket"][3] - prof_pct["empty_bracket"][3]) if "noop_kernel_bracket" in prof_pct else 0.0
        kernels = {tag: {"avg_us": max(1e3 * ms / n - bracket_us, 0.0), "launches_per_step": n / steps,
                         "p10_p50_p90_us": [max(1e3 * x - bracket_us, 0.0) for x in prof_pct[tag][2:5]]}
                   for tag, (ms, n) in prof.items()}
        step_sum_us = sum(v["avg_us"] * v["launches_per_step"] for v in kernels.values())
        used = [sizes[s % n_batches] for s in range(steps)]
        candidates = []
        for tag, v in kernels.items():
            bound, work = algorithmic_work(tag, used, cfg, dims)
            if work is None:
                continue
            per_step_us = v["avg_us"] * v["launches_per_step"]
            candidates.append((per_step_us, tag, bound, work, v["avg_us"]))
        best = pick_dominant(candidates, False)
        if best is not None:
            _, tag, bound, work, avg_us = best
            if bound == "hbm":
                achieved, peak, unit = work / (avg_us * 1e-6) / 1e9, HBM_PEAK_GBS, "GB/s"
            else:
                achieved, peak, unit = work / (avg_us * 1e-6) / 1e12, MFMA_BF16_PEAK_TFLOPS, "TFLOP/s"
            roofline = {"kernel": tag, "bound": bound, "achieved": achieved, "peak": peak, "unit": unit,
                        "frac": achieved / peak, "traffic": measured_traffic(cfg.name, tag), "avg_us": avg_us,
                        "p10_p50_p90_us": kernels[tag].get("p10_p50_p90_us"),
                        "algorithmic_per_launch": work, "kernel_time_share_of_step": best[0] / step_sum_us,
                        "event_bracket_overhead_us_subtracted": bracket_us,
                        # a bracket around a kernel that does nothing reads this much more than an empty one: the latency
                        # of a launch as such, still contained in avg_us (rocprofv3's own durations do not contain it)
                        "launch_latency_us_not_subtracted": max(noop_us, 0.0)}

    baseline = None
    if not args.no_cpu_baseline:
        baseline = cpu_baseline_link_prediction(cfg, inputs, batches, R)

    print(json.dumps({
        "metric": "sampled edges/s through sample+gather+forward+DistMult decoder+backward+embedding update (link prediction)",
        "value": edges / total_s, "unit": "sampled edges/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": 1e3 * total_s / steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name, "num_nodes": cfg.num_nodes, "num_edges": int(inputs["col"].numel()),
                   "feat_dim": cfg.feat_dim, "dims": dims, "fanouts": list(cfg.fanouts), "direction": "in+out",
                   "positive_edges_per_batch": B, "chunk": chunk, "negatives_per_chunk": Nn, "relations": num_rel,
                   "mean_nodes_per_batch": mean_n, "mean_sampled_edges_per_batch": mean_e},
        "mini_batches_per_s": steps / total_s, "training_edges_per_s": B * steps / total_s, "in_flight": in_flight,
        "replica_note": "with more than one mini-batch in flight the replicas apply their SGD steps to ONE shared embedding table "
                        "without waiting for each other (non-atomic read-modify-write per row): rows that concurrent batches share "
                        "(hub nodes, negatives) can lose an update or be read half-updated, so that mode is not reproducible bit "
                        "for bit; one_in_flight is the reproducible figure",
        "one_in_flight": {"ms_per_step": 1e3 * serial_s / steps, "training_edges_per_s": B * steps / serial_s},
        "roofline": roofline, "kernels": kernels, "cpu_baseline": baseline}))


def cpu_baseline_link_prediction(cfg, inputs, batches, R, budget_s=20.0):
    """The oracle's link-prediction step on the host (sample, gather, encoder, decoder, both backward passes)."""
    import numpy as np
    import torch
    import oracle
    t0 = time.time()
    g = oracle.Graph(cfg.num_nodes, inputs["rowptr"].cpu().numpy(), inputs["col"].cpu().numpy(),
                     inputs["rowptr_in"].cpu().numpy(), inputs["col_in"].cpu().numpy())
    log("cpu_baseline: graph copied to the host in %.1fs" % (time.time() - t0))
    params = oracle.SageParams(*inputs["weights"])
    table, Rn = inputs["table"], R.cpu().numpy()
    done, edges, spent = 0, 0, 0.0
    while done < len(batches) and (done < 1 or spent < budget_s):
        src, rel, dst, neg = [t.cpu().numpy() for t in batches[done]]
        t0 = time.time()
        d, ls, ld, ln = oracle.dense_sample_edges(g, src, dst, neg.reshape(-1), cfg.fanouts, seed=done, direction=cfg.direction)
        rows = table[torch.from_numpy(d.node_ids.astype(np.int64)).to(table.device)].cpu().numpy()
        st = oracle.sage_forward(d, rows, params, mode="bf16")
        ds = oracle.distmult_forward(st.out.astype(np.float32), Rn, ls, rel, ld, ln.reshape(neg.shape), cfg.lp_chunk, mode="bf16")
        d_h, _ = oracle.distmult_backward(ds)
        oracle.sage_backward(st, params, d_h, mode="bf16")
        spent += time.time() - t0
        edges += len(d.nbrs)
        done += 1
        log("cpu_baseline: batch %d, %.2fs so far" % (done, spent))
    threads = blas_threads()
    return {"value": edges / spent, "unit": "sampled edges/s", "cores": int(threads), "kind": "oracle",
            "sample": "%d mini-batches of the same workload (%.1f s; C sampler is single-threaded, NumPy contractions use "
                      "the BLAS threads counted in cores; feature rows fetched from the device table)" % (done, spent),
            "training_edges_per_s": cfg.lp_edges * done / spent, "host": host_description(),
            "note": "a plain oracle, not a tuned CPU baseline"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--workload", default="rmat111m")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-times", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy a few times (reference for hardware byte counters)")
    ap.add_argument("--separate-gather", action="store_true",
                    help="dense_gather into an H^0 buffer, then sage_forward (default: sage_forward_table, whose layer-1 "
                         "aggregation reads the table's rows itself)")
    ap.add_argument("--also-two-step", type=int, default=0,
                    help="run that many untimed steps in the two-step form (dense_gather + sage_forward) first, so that a "
                         "profiler sees those kernels too")
    ap.add_argument("--no-graphs", action="store_true", help="launch every kernel from the host instead of replaying HIP graphs")
    ap.add_argument("--replica-graphs", action="store_true",
                    help="replicas replay one HIP graph per step instead of launching every kernel from the host")
    ap.add_argument("--python-replicas", action="store_true",
                    help="drive the replicas' streams from Python instead of handing the steps to dn_train_steps")
    ap.add_argument("--replicas", type=int, default=4,
                    help="data-parallel replicas on one GPU: that many mini-batches run the whole path concurrently, "
                         "each on a HIP stream of its own (0 = skip this measurement)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2202_02365_amd as dn
    from workloads import get_config

    cfg = get_config(args.workload)
    if cfg.lp_edges:
        if args.steps == 256 and args.warmup == 64:
            args.steps, args.warmup = 32, 4           # a link-prediction step is ~30 times longer
        run_link_prediction(args, cfg)
        return
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    from workloads import make_inputs
    inputs = make_inputs(cfg, dev, N_BATCHES, log)
    k, dims = cfg.num_layers, cfg.dims

    graph = dn.Graph(inputs["rowptr"], inputs["col"], inputs["rowptr_in"], inputs["col_in"])
    batch = dn.Batch(cfg.num_nodes, cfg.batch, cfg.fanouts, cfg.direction)
    in_dtype = dn.DN_F32 if cfg.feat_dtype == "f32" else dn.DN_BF16
    model = dn.Model(batch, dims, in_dtype)
    w_self, w_nbr, bias = [[torch.from_numpy(a).to(dev) for a in group] for group in inputs["weights"]]
    model.set_weights(w_self, w_nbr, bias)
    table = inputs["table"]
    targets = [torch.from_numpy(t).to(dev) for t in inputs["targets"]]
    h0 = torch.empty((batch.node_capacity, dims[0]), dtype=table.dtype, device=dev)
    out = torch.empty((cfg.batch, dims[-1]), dtype=torch.float32, device=dev)
    gen = torch.Generator(device="cpu").manual_seed(11)
    grad_out = torch.empty((cfg.batch, dims[-1]), dtype=torch.float32, device=dev)        # dL/dH^k from the loss head
    loss_buf = torch.empty(cfg.batch, dtype=torch.float32, device=dev)
    from workloads import class_labels
    labels = torch.from_numpy(class_labels(cfg.batch, dims[-1]).astype(np.int32)).to(dev)  # synthetic class per target

    def loss_and_backward(m, b, out_buf, gout_buf, lbuf, dws_, dwn_, dbs_, dh0_):
        # softmax cross-entropy head on the device (mean over the batch), then the encoder's backward pass
        dn.softmax_xent(out_buf, labels, lbuf, gout_buf, 1.0 / cfg.batch)
        dn.sage_backward(m, b, gout_buf, dws_, dwn_, dbs_, dh0_)
    dws = [torch.empty_like(w) for w in w_self]
    dwn = [torch.empty_like(w) for w in w_nbr]
    dbs = [torch.empty_like(b) for b in bias]
    need_dh0 = cfg.name.endswith("_lp")            # learnable base representations need dL/dH^0
    dh0 = torch.empty((batch.node_capacity, dims[0]), dtype=torch.float32, device=dev) if need_dh0 else None

    fused = not args.separate_gather

    def gather(b, h0_buf):
        if not fused:
            dn.dense_gather(b, table, h0_buf)

    def forward(m, b, h0_buf, out_buf):
        if fused:
            dn.sage_forward_table(m, b, table, out_buf)
        else:
            dn.sage_forward(m, b, h0_buf, out_buf)

    def step(bi, backward=True, separate=False):
        dn.dense_sample(batch, graph, targets[bi], bi)
        if separate or not fused:
            dn.dense_gather(batch, table, h0)
            dn.sage_forward(model, batch, h0, out)
        else:
            dn.sage_forward_table(model, batch, table, out)
        if backward:
            loss_and_backward(model, batch, out, grad_out, loss_buf, dws, dwn, dbs, dh0)

    # Two mini-batches in flight: batch t+1 is sampled and gathered on one stream while batch t runs
    # forward/backward on another (mini-batch construction does not read the weights; this is the
    # paper's pipelining of construction with compute, Section 3, on two HIP streams of one GPU).
    slots = [(batch, h0), (dn.Batch(cfg.num_nodes, cfg.batch, cfg.fanouts, cfg.direction), torch.empty_like(h0))]
    s_build, s_compute = torch.cuda.Stream(), torch.cuda.Stream()
    ev_built = [torch.cuda.Event(), torch.cuda.Event()]
    ev_free = [torch.cuda.Event(), torch.cuda.Event()]

    def timed_pipelined(n_steps, backward=True):
        torch.cuda.synchronize()
        for e in ev_free:
            e.record()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(n_steps):
            b_s, h0_s = slots[s & 1]
            bi = s % N_BATCHES
            with torch.cuda.stream(s_build):
                s_build.wait_event(ev_free[s & 1])
                dn.dense_sample(b_s, graph, targets[bi], bi)
                gather(b_s, h0_s)
                if backward:
                    b_s.prepare_backward(need_dh0)
                ev_built[s & 1].record(s_build)
            with torch.cuda.stream(s_compute):
                s_compute.wait_event(ev_built[s & 1])
                forward(model, b_s, h0_s, out)
                if backward:
                    loss_and_backward(model, b_s, out, grad_out, loss_buf, dws, dwn, dbs, dh0)
                ev_free[s & 1].record(s_compute)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    # sizes of every batch (untimed; counts() waits for the device)
    sizes = []
    for bi in range(N_BATCHES):
        dn.dense_sample(batch, graph, targets[bi], bi)
        c = batch.counts()
        nbr_offsets = batch.view()["nbr_offsets"]
        # slots owned by Delta_i .. Delta_k (what layer i aggregates over), i = 1..k
        c += [int(c[k + 2] - int(nbr_offsets[c[i] - c[1]])) for i in range(1, k + 1)]
        sizes.append(c)
    mean_n = float(np.mean([s[k + 1] for s in sizes]))
    mean_e = float(np.mean([s[k + 2] for s in sizes]))
    log("mini-batch sizes: mean N=%.0f, mean E=%.0f" % (mean_n, mean_e))

    def timed(n_steps, backward=True):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(n_steps):
            step(s % N_BATCHES, backward)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    # The same pipeline replayed from HIP graphs, one graph per batch index, captured once, so that
    # the host submits 1 graph launch per step instead of ~40 kernel launches (the step is a chain of small kernels and the host would otherwise
    # be the bottleneck).  Replays launch exactly the kernels of the eager path; one replay is compared
    # with an eager step below.
    graphs = {}

    def capture_graphs(backward):
        # graph bi: forward(+backward) of batch bi on the capture stream, and, forked onto a second
        # stream inside the same graph, sampling + gather of batch bi+1 into the other slot
        for bi in range(N_BATCHES):
            nxt = (bi + 1) % N_BATCHES
            b_cur, h0_cur = slots[bi & 1]
            b_nxt, h0_nxt = slots[nxt & 1]
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=s_compute):
                s_build.wait_stream(s_compute)
                with torch.cuda.stream(s_build):
                    dn.dense_sample(b_nxt, graph, targets[nxt], nxt)
                    gather(b_nxt, h0_nxt)
                    if backward:
                        b_nxt.prepare_backward(need_dh0)
                forward(model, b_cur, h0_cur, out)
                if backward:
                    loss_and_backward(model, b_cur, out, grad_out, loss_buf, dws, dwn, dbs, dh0)
                s_compute.wait_stream(s_build)
            graphs[(bi, backward)] = g
        torch.cuda.synchronize()

    def timed_graphs(n_steps, backward=True):
        # prologue (untimed): construct batch 0 so that the first graph finds its inputs
        with torch.cuda.stream(s_compute):
            dn.dense_sample(slots[0][0], graph, targets[0], 0)
            gather(slots[0][0], slots[0][1])
            if backward:
                slots[0][0].prepare_backward(need_dh0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        with torch.cuda.stream(s_compute):
            for s in range(n_steps):
                graphs[(s % N_BATCHES, backward)].replay()
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    # Data-parallel replicas on one GPU: R mini-batches run the whole path at once, each on its own stream
    # with its own batch and model workspaces, against the same weights; their gradients are what R
    # data-parallel workers would sum.  The step is a chain of ~40 short kernels, most of them far too
    # small to fill 256 compute units, so concurrent chains fill the gaps.
    stream_overlap = {}

    def timed_replicas(n_steps, n_rep, backward=True):
        reps = []
        for r in range(n_rep):
            b = dn.Batch(cfg.num_nodes, cfg.batch, cfg.fanouts, cfg.direction)
            m = dn.Model(b, dims, in_dtype)
            m.set_weights(w_self, w_nbr, bias)
            reps.append(dict(batch=b, model=m, h0=torch.empty_like(h0), out=torch.empty_like(out),
                             gout=torch.empty_like(grad_out), loss=torch.empty_like(loss_buf),
                             dws=[torch.empty_like(w) for w in w_self], dwn=[torch.empty_like(w) for w in w_nbr],
                             dbs=[torch.empty_like(x) for x in bias],
                             dh0=None if dh0 is None else torch.empty_like(dh0), stream=torch.cuda.Stream()))

        def one_step(o, bi):
            dn.dense_sample(o["batch"], graph, targets[bi], bi)
            gather(o["batch"], o["h0"])
            forward(o["model"], o["batch"], o["h0"], o["out"])
            if backward:
                loss_and_backward(o["model"], o["batch"], o["out"], o["gout"], o["loss"], o["dws"], o["dwn"], o["dbs"], o["dh0"])

        rep_graphs = {}
        if args.replica_graphs:
            # one HIP graph per (replica, batch it runs): the host then hands over a whole step with one call
            assert N_BATCHES % n_rep == 0
            for bi in range(N_BATCHES):
                o = reps[bi % n_rep]
                one_step(o, bi)                              # eager once (lazy initialisation stays out of the capture)
                torch.cuda.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=o["stream"]):
                    one_step(o, bi)
                rep_graphs[bi] = g
            torch.cuda.synchronize()

        lib_steps = None
        if fused and not rep_graphs and not args.python_replicas:
            # the library schedules the replicas itself (dn_train_steps): step s on its internal stream s % n_rep (every
            # call starts at step 0 and the call joins its streams at the end, so a replica's steps stay in order)
            lib_steps = dn.TrainSteps([dict(batch=reps[bi % n_rep]["batch"], model=reps[bi % n_rep]["model"], graph=graph,
                                            targets=targets[bi], seed=bi, table=table, out=reps[bi % n_rep]["out"],
                                            labels=labels, grad_scale=1.0 / cfg.batch, loss=reps[bi % n_rep]["loss"],
                                            grad_out=reps[bi % n_rep]["gout"], dws=reps[bi % n_rep]["dws"],
                                            dwn=reps[bi % n_rep]["dwn"], dbs=reps[bi % n_rep]["dbs"],
                                            dh0=reps[bi % n_rep]["dh0"]) for bi in range(N_BATCHES)],
                                      forward_only=not backward)

        def run(n):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            if lib_steps is not None:
                for first in range(0, n, N_BATCHES):
                    lib_steps.run(n_rep, 0, min(N_BATCHES, n - first))
            else:
                for s in range(n):
                    o = reps[s % n_rep]
                    bi = s % N_BATCHES
                    with torch.cuda.stream(o["stream"]):
                        if rep_graphs:
                            rep_graphs[bi].replay()
                        else:
                            one_step(o, bi)
            queued = time.perf_counter() - t0               # the host has handed over every launch
            torch.cuda.synchronize()
            spent = time.perf_counter() - t0
            log("%d replicas, %s: host queued %d steps in %.3f ms/step, GPU finished them in %.3f ms/step" %
                (n_rep, "whole step" if backward else "forward only", n, 1e3 * queued / n, 1e3 * spent / n))
            return spent
        run(max(args.warmup, n_rep))
        if lib_steps is not None and backward:
            # do the library's step streams run side by side?  (a busy-wait kernel of 20 us on each of them at once)
            overlap = {n: dn.profile_step_stream_overlap(n, 20) for n in range(1, n_rep + 1)}
            log("step streams: 20 us busy-wait kernels on 1..%d streams at once take %s us per round" %
                (n_rep, ", ".join("%.1f" % overlap[n] for n in sorted(overlap))))
            stream_overlap.update(overlap)
        # one read-back of the sizes per batch object, as a training loop does when it logs them: the library picks the
        # form of the transpose-index build from the largest counts read back so far (a matter of speed only)
        for o in reps:
            o["batch"].counts()
        spent, _ = median_seconds(lambda: run(n_steps))
        if backward:
            # with every replica busy, the one that runs batch 5 must give the gradients of the one-at-a-time step
            for r, o in enumerate(reps):
                bi = 5 if r == 0 else 6 + r
                with torch.cuda.stream(o["stream"]):
                    dn.dense_sample(o["batch"], graph, targets[bi], bi)
                    gather(o["batch"], o["h0"])
                    forward(o["model"], o["batch"], o["h0"], o["out"])
                    loss_and_backward(o["model"], o["batch"], o["out"], o["gout"], o["loss"], o["dws"], o["dwn"], o["dbs"], o["dh0"])
            torch.cuda.synchronize()
            o = reps[0]
            if not all(torch.equal(a, b) for a, b in zip(eager, o["dws"] + o["dwn"] + o["dbs"] + [o["out"]])):
                raise RuntimeError("a replica's step differs from the one-at-a-time step")
        return spent

    edges = sum(sizes[s % N_BATCHES][k + 2] for s in range(args.steps))
    for s in range(args.also_two_step):
        step(s % N_BATCHES, separate=True)
    timed(args.warmup)
    serial_s, serial_all = median_seconds(lambda: timed(args.steps))
    serial_fwd_s, _ = median_seconds(lambda: timed(args.steps, backward=False))
    # one-at-a-time reference for batch 5, to compare a graph replay and a replica's step with
    step(5)
    torch.cuda.synchronize()
    eager = [t.clone() for t in dws + dwn + dbs + [out]]
    if args.no_graphs:
        timed_pipelined(args.warmup)
        total_s, _ = median_seconds(lambda: timed_pipelined(args.steps))
        fwd_only_s, _ = median_seconds(lambda: timed_pipelined(args.steps, backward=False))
    else:
        assert N_BATCHES % 2 == 0
        capture_graphs(True)
        capture_graphs(False)
        timed_graphs(args.warmup)
        total_s, _ = median_seconds(lambda: timed_graphs(args.steps))
        fwd_only_s, _ = median_seconds(lambda: timed_graphs(args.steps, backward=False))
        with torch.cuda.stream(s_compute):
            graphs[(4, True)].replay()           # constructs batch 5
            graphs[(5, True)].replay()           # forward + backward of batch 5
        torch.cuda.synchronize()
        if not all(torch.equal(a, b) for a, b in zip(eager, dws + dwn + dbs + [out])):
            raise RuntimeError("a graph replay differs from the eager step")
    log("timed %d steps, two mini-batches in flight: %.3f ms/step (sample+gather+fwd only: %.3f ms); "
        "one in flight: %.3f ms/step (%.3f ms)" %
        (args.steps, 1e3 * total_s / args.steps, 1e3 * fwd_only_s / args.steps,
         1e3 * serial_s / args.steps, 1e3 * serial_fwd_s / args.steps))
    pipelined = {"ms_per_step": 1e3 * total_s / args.steps, "mini_batches_per_s": args.steps / total_s,
                 "sampled_edges_per_s": edges / total_s,
                 "sample_gather_fwd_ms_per_step": 1e3 * fwd_only_s / args.steps,
                 "launch": "eager" if args.no_graphs else
                           "hipGraph replay (1 graph per step, construction forked onto a second stream)"}
    in_flight = "2 mini-batches: sample+gather of batch t+1 on one stream, forward+backward of batch t on another"
    if args.replicas > 1:
        rep_s = timed_replicas(args.steps, args.replicas)
        rep_fwd_s = timed_replicas(args.steps, args.replicas, backward=False)
        log("%d replicas on %d streams: %.3f ms/step (sample+gather+fwd only: %.3f ms)" %
            (args.replicas, args.replicas, 1e3 * rep_s / args.steps, 1e3 * rep_fwd_s / args.steps))
        if rep_s < total_s:
            total_s, fwd_only_s = rep_s, rep_fwd_s
            in_flight = ("%d mini-batches, each running sample+gather+forward+backward on a stream of its own "
                         "(data-parallel replicas on one GPU, same weights, gradients per replica), %s"
                         % (args.replicas, "scheduled by the library (dn_train_steps)"
                            if fused and not args.replica_graphs and not args.python_replicas else "launched from Python"))

    # one mini-batch at a time, but scheduled by the library (dn_train_steps on one stream)
    one_lib_s = None
    if fused and not args.python_replicas:
        one_lib_s = timed_replicas(args.steps, 1)
        log("one mini-batch at a time through dn_train_steps: %.3f ms/step" % (1e3 * one_lib_s / args.steps))

    if model.status()[1] != 0:
        raise RuntimeError("the ReLU sign fix-up queue overflowed during the timed run")

    # per-kernel durations: the same K steps again, every launch bracketed by HIP events on its stream
    roofline, kernels, copy_gbs, whole_step = None, {}, None, None
    if not args.no_kernel_times:
        # The event pairs time what the GPU does only if the host is ahead of it: every step is preceded by
        # a ~1 ms streaming copy (not bracketed) during which the host queues the whole step.
        delay_src = torch.empty(256 << 20, dtype=torch.float32, device=dev)
        delay_dst = torch.empty_like(delay_src)
        # what a plain streaming copy reaches on this machine (1 GiB read + 1 GiB written per call): context for the peak
        dn.profile_calibration_copy(delay_dst, delay_src)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            dn.profile_calibration_copy(delay_dst, delay_src)
        torch.cuda.synchronize()
        copy_gbs = 10 * 2 * delay_src.numel() * 4 / (time.perf_counter() - t0) / 1e9
        dn.profile_enable(True)
        torch.cuda.synchronize()
        for s in range(args.steps):
            dn.profile_calibration_copy(delay_dst, delay_src)
            dn.profile_empty_bracket()
            step(s % N_BATCHES)
        prof_pct = dn.profile_collect_percentiles()
        prof = {tag: (v[0], v[1]) for tag, v in prof_pct.items()}
        dn.profile_enable(False)
        prof_two_step = {}
        if fused:
            # the two-step form too, so that dense_gather and the aggregation over H^0 have their own figures
            dn.profile_enable(True)
            for s in range(min(args.steps, 32)):
                dn.profile_calibration_copy(delay_dst, delay_src)
                step(s % N_BATCHES, separate=True)
            prof_two_step = dn.profile_collect()
            dn.profile_enable(False)
        del delay_src, delay_dst
        # an event pair around nothing already reads a few microseconds: subtract that from every bracket
        empty_ms, empty_n = prof.pop("empty_bracket", (0.0, 1))
        prof.pop("noop_kernel_bracket", None)
        bracket_us = 1e3 * empty_ms / max(empty_n, 1)
        # launch latency as such: median bracket around a kernel that does nothing, less the median empty bracket (the
        # first launch of that kernel loads its code object, which a mean would carry)
        noop_us = 1e3 * (prof_pct["noop_kernel_bracket"][3] - prof_pct["empty_bracket"][3]) if "noop_kernel_bracket" in prof_pct else 0.0
        kernels = {tag: {"avg_us": max(1e3 * ms / n - bracket_us, 0.0), "launches_per_step": n / args.steps}
                   for tag, (ms, n) in prof.items()}
        for tag, v in kernels.items():
            # percentiles of the single brackets (the same bracket cost subtracted): the spread behind avg_us
            v["p10_p50_p90_us"] = [max(1e3 * x - bracket_us, 0.0) for x in prof_pct[tag][2:5]]
        for tag in ("gather", "aggregate_L1"):
            if tag in prof_two_step:
                ms, n = prof_two_step[tag]
                kernels[tag] = {"avg_us": max(1e3 * ms / n - bracket_us, 0.0), "launches_per_step": 0.0,
                                "note": "two-step form (dense_gather + sage_forward) only"}
        step_sum_us = sum(v["avg_us"] * v["launches_per_step"] for v in kernels.values())
        used = [sizes[s % N_BATCHES] for s in range(args.steps)]
        candidates = []
        for tag, v in kernels.items():
            bound, work = algorithmic_work(tag, used, cfg, dims)
            if work is None:
                continue
            # every kernel with a formula carries its own fraction of the peak that bounds it
            rate = work / (v["avg_us"] * 1e-6)
            v["bound"] = bound
            v["frac_of_peak"] = rate / (HBM_PEAK_GBS * 1e9 if bound == "hbm" else MFMA_BF16_PEAK_TFLOPS * 1e12)
            gemm_bytes = gemm_algorithmic_bytes(tag, used, cfg, dims) if bound == "mfma" else None
            if gemm_bytes:
                # at these shapes flops / byte sits below the ridge (peak flops / peak bytes), so the HBM roofline
                # is the lower of the two: the fraction of min(MFMA peak, intensity x HBM peak) goes beside it
                intensity = work / gemm_bytes
                attainable = min(MFMA_BF16_PEAK_TFLOPS * 1e12, intensity * HBM_PEAK_GBS * 1e9)
                v["flop_per_byte"] = intensity
                v["attainable_TFLOPs"] = attainable / 1e12
                v["frac_of_attainable"] = rate / attainable
            v["algorithmic_per_launch"] = work
            traffic = measured_traffic(cfg.name, tag)
            if traffic is not None:
                v["traffic_bytes_per_launch"] = traffic
                moved = work if bound == "hbm" else gemm_bytes
                if moved:
                    v["traffic_over_algorithmic"] = traffic / moved
            per_step_us = v["avg_us"] * v["launches_per_step"]
            candidates.append((per_step_us, tag, bound, work, v["avg_us"]))
        # the whole step against the HBM roofline: algorithmic bytes of every launch of a step (a GEMM counts with its
        # operand and result bytes) over the measured step time
        step_bytes = 0.0
        for tag, v in kernels.items():
            if v["launches_per_step"] <= 0 or "bound" not in v:
                continue
            b = v["algorithmic_per_launch"] if v["bound"] == "hbm" else (gemm_algorithmic_bytes(tag, used, cfg, dims) or 0.0)
            step_bytes += b * v["launches_per_step"]
        whole_step = {"algorithmic_bytes_per_step": step_bytes,
                      "hbm_frac_one_in_flight": step_bytes / (serial_s / args.steps) / (HBM_PEAK_GBS * 1e9),
                      "hbm_frac_reported_mode": step_bytes / (total_s / args.steps) / (HBM_PEAK_GBS * 1e9),
                      "kernel_time_sum_us": step_sum_us,
                      "untagged_kernels": sorted(t for t, v in kernels.items() if "bound" not in v)}
        best = pick_dominant(candidates, True)
        if best is not None:
            _, tag, bound, work, avg_us = best
            if bound == "hbm":
                achieved, peak, unit = work / (avg_us * 1e-6) / 1e9, HBM_PEAK_GBS, "GB/s"
            else:
                achieved, peak, unit = work / (avg_us * 1e-6) / 1e12, MFMA_BF16_PEAK_TFLOPS, "TFLOP/s"
            roofline = {"kernel": tag, "bound": bound, "achieved": achieved, "peak": peak, "unit": unit,
                        "frac": achieved / peak, "traffic": measured_traffic(cfg.name, tag), "avg_us": avg_us,
                        "p10_p50_p90_us": kernels[tag].get("p10_p50_p90_us"),
                        "algorithmic_per_launch": work, "kernel_time_share_of_step": best[0] / step_sum_us,
                        "event_bracket_overhead_us_subtracted": bracket_us,
                        # a bracket around a kernel that does nothing reads this much more than an empty one: the latency
                        # of a launch as such, still contained in avg_us (rocprofv3's own durations do not contain it)
                        "launch_latency_us_not_subtracted": max(noop_us, 0.0)}

    if args.copy_calibration:
        src = torch.empty(64 << 20, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(5):
            dn.profile_calibration_copy(dst, src)          # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()

    baseline = None
    if not args.no_cpu_baseline:
        baseline = cpu_baseline(cfg, inputs, sizes)

    result = {
        "metric": "sampled edges/s + mini-batches/s at 1 MI355X, 3-hop DENSE + GraphSage; value = whole step "
                  "(sample+gather+forward+backward), sample_gather_fwd = the forward-only chain; % of HBM / MFMA peak per "
                  "kernel in kernels[*].frac_of_peak and roofline",
        "value": edges / total_s,
        "unit": "sampled edges/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": 1e3 * total_s / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": cfg.name, "num_nodes": cfg.num_nodes, "num_edges_nominal": cfg.num_edges,
                   "num_edges": int(inputs["col"].numel()), "feat_dim": cfg.feat_dim, "feat_dtype": cfg.feat_dtype,
                   "dims": dims, "fanouts": list(cfg.fanouts), "batch": cfg.batch,
                   "mean_nodes_per_batch": mean_n, "mean_sampled_edges_per_batch": mean_e},
        "mini_batches_per_s": args.steps / total_s,
        "in_flight": in_flight,
        "step_streams_busy_wait_us": {"note": "a 20 us single-wave busy-wait kernel on each of the library's first n step streams "
                                              "at once, us per round (about 20 + 2.5 n if the streams run side by side; the 2.5 "
                                              "is the host's launch call)",
                                      **{str(n): v for n, v in sorted(stream_overlap.items())}},
        "forward": "sage_forward_table: the layer-1 aggregation reads the table's rows itself, no H^0 buffer" if fused
                   else "dense_gather into H^0, then sage_forward",
        "two_in_flight": pipelined,
        "sample_gather_fwd": {"ms_per_step": 1e3 * fwd_only_s / args.steps,
                              "mini_batches_per_s": args.steps / fwd_only_s,
                              "sampled_edges_per_s": edges / fwd_only_s},
        "one_in_flight": {"ms_per_step": 1e3 * serial_s / args.steps, "mini_batches_per_s": args.steps / serial_s,
                          "sampled_edges_per_s": edges / serial_s,
                          "sample_gather_fwd_ms_per_step": 1e3 * serial_fwd_s / args.steps,
                          "launch": "every call of the path made from Python on one stream"},
        "one_in_flight_library": None if one_lib_s is None else
                                 {"ms_per_step": 1e3 * one_lib_s / args.steps, "mini_batches_per_s": args.steps / one_lib_s,
                                  "launch": "dn_train_steps with one stream"},
        "repeats": REPEATS,
        "timing": "every figure is the median of %d timed blocks of `steps` steps" % REPEATS,
        "one_in_flight_blocks_ms": [1e3 * t / args.steps for t in serial_all],
        "roofline": roofline,
        "whole_step": whole_step,
        "streaming_copy_GBs": copy_gbs,
        "kernels": kernels,
        "cpu_baseline": baseline,
    }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
