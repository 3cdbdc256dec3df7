"""Feature tables, Glorot weights, target batches, class labels and link-prediction batches."""
import math
import numpy as np
import torch

from .rmat import mix64, _s64


def feature_table(V: int, d: int, dtype: str = "f32", seed: int = 2, device="cpu",
                  rows_per_chunk: int = 1 << 22) -> torch.Tensor:
    """[V x d] N(0,1) table, row-major.  Drawn from torch's generator of `device`, so a
    table made on the GPU is not the table made on the host: consumers on the other side
    read the rows they need from this tensor."""
    tdtype = {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    out = torch.empty((V, d), dtype=tdtype, device=device)
    for lo in range(0, V, rows_per_chunk):
        hi = min(V, lo + rows_per_chunk)
        blk = torch.randn((hi - lo, d), generator=gen, device=device, dtype=torch.float32)
        out[lo:hi] = blk.to(tdtype)
        del blk
    return out


def glorot_weights(dims, seed: int = 3, bias_scale: float = 0.0):
    """Per layer i (1..k): W_self, W_nbr as float32 [d_{i-1} x d_i] drawn U(-a, a) with
    a = sqrt(6 / (d_in + d_out)), and a bias vector (zero unless bias_scale > 0)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    w_self, w_nbr, bias = [], [], []
    for d_in, d_out in zip(dims[:-1], dims[1:]):
        a = math.sqrt(6.0 / (d_in + d_out))
        w_self.append(rng.uniform(-a, a, size=(d_in, d_out)).astype(np.float32))
        w_nbr.append(rng.uniform(-a, a, size=(d_in, d_out)).astype(np.float32))
        bias.append((bias_scale * rng.standard_normal(d_out)).astype(np.float32))
    return w_self, w_nbr, bias


def training_subset(V: int, fraction: float, seed: int = 4, device="cpu", chunk: int = 1 << 26) -> torch.Tensor:
    """Ascending ids of the nodes whose hash falls below `fraction` (all nodes if fraction >= 1)."""
    if fraction >= 1.0:
        return torch.arange(V, dtype=torch.int64, device=device)
    thresh = int(fraction * (1 << 32))
    key = _s64(seed * 0xA24BAED4963EE407)
    parts = []
    for lo in range(0, V, chunk):
        hi = min(V, lo + chunk)
        ids = torch.arange(lo, hi, dtype=torch.int64, device=device)
        h = mix64(ids ^ key) & 0xFFFFFFFF
        parts.append(ids[h < thresh])
    return torch.cat(parts)


def target_batch(pool_size: int, batch: int, batch_index: int, seed: int = 4, pool: torch.Tensor = None) -> np.ndarray:
    """`batch` pairwise-distinct target node ids (int32), uniform over the pool, for mini-batch `batch_index`.

    Distinctness by construction: positions i*stride + offset_i with offset_i < stride are
    distinct, then shuffled; for a pool much larger than the batch this is a stratified
    uniform draw."""
    if batch > pool_size:
        raise ValueError("batch larger than pool")
    rng = np.random.Generator(np.random.PCG64([seed, batch_index]))
    stride = pool_size // batch
    pos = np.arange(batch, dtype=np.int64) * stride + rng.integers(0, stride, size=batch)
    rng.shuffle(pos)
    if pool is not None:
        ids = pool[torch.from_numpy(pos).to(pool.device)].cpu().numpy()
    else:
        ids = pos
    return ids.astype(np.int32)


def class_labels(n: int, num_classes: int, seed: int = 5) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(0, num_classes, size=n).astype(np.int64)


def decoder_inputs(n_rows: int, num_rel: int, dim: int, n_edges: int, chunk: int, num_neg: int, seed: int = 6,
                   zipf_exponent: float = 1.1, scale: float = 0.5):
    """Inputs of a link-prediction decoder in the shape of the Freebase86M-like workload: node representations
    H [n_rows x dim] (N(0, scale^2)), relation embeddings R [num_rel x dim] (N(0,1)), edges as (row of H, relation,
    row of H) with uniform endpoints and relation ids drawn from a Zipf(zipf_exponent) law over num_rel types,
    and per chunk of `chunk` edges one list of num_neg uniform negative rows."""
    rng = np.random.default_rng([seed, n_rows, n_edges])
    H = (scale * rng.standard_normal((n_rows, dim))).astype(np.float32)
    R = rng.standard_normal((num_rel, dim)).astype(np.float32)
    src = rng.integers(0, n_rows, n_edges).astype(np.int32)
    dst = rng.integers(0, n_rows, n_edges).astype(np.int32)
    w = 1.0 / np.arange(1, num_rel + 1, dtype=np.float64) ** zipf_exponent
    rel = rng.choice(num_rel, size=n_edges, p=w / w.sum()).astype(np.int32)
    n_chunks = (n_edges + chunk - 1) // chunk
    neg = rng.integers(0, n_rows, (n_chunks, num_neg)).astype(np.int32)
    return H, R, src, rel, dst, neg


def edge_batch(rowptr: torch.Tensor, col: torch.Tensor, num_nodes: int, n_edges: int, chunk: int, num_neg: int,
               num_rel: int, batch_index: int, seed: int = 17, zipf_exponent: float = 1.1):
    """One link-prediction batch over a CSR graph: n_edges positive edges drawn uniformly from the graph's edges,
    a Zipf(zipf_exponent) relation type per edge, and per chunk of `chunk` edges num_neg uniform negative nodes.
    Returns (src, rel, dst, neg) as int32 tensors on the graph's device (neg is [chunks x num_neg])."""
    rng = np.random.default_rng([seed, batch_index])
    dev = col.device
    e = torch.from_numpy(rng.integers(0, col.numel(), n_edges)).to(dev)
    dst = col[e].to(torch.int32)
    src = (torch.searchsorted(rowptr, e, right=True) - 1).to(torch.int32)
    n_chunks = (n_edges + chunk - 1) // chunk
    neg = torch.from_numpy(rng.integers(0, num_nodes, (n_chunks, num_neg)).astype(np.int32)).to(dev)
    w = 1.0 / np.arange(1, num_rel + 1, dtype=np.float64) ** zipf_exponent
    rel = torch.from_numpy(rng.choice(num_rel, size=n_edges, p=w / w.sum()).astype(np.int32)).to(dev)
    return src, rel, dst, neg


def relation_embeddings(num_rel: int, dim: int, seed: int = 19) -> np.ndarray:
    """N(0,1) relation embeddings [num_rel x dim], fp32."""
    return np.random.default_rng([seed, num_rel, dim]).standard_normal((num_rel, dim)).astype(np.float32)
