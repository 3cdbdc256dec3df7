"""The synthetic input generators: deterministic, well-formed, shaped like the paper's workloads."""
import numpy as np
import torch

from workloads import (CONFIGS, rmat_csr, transpose_csr, target_batch, training_subset, feature_table,
                       glorot_weights)
from conftest import transpose_np


def test_rmat_csr_is_well_formed_and_deterministic(rmat16k):
    rp, col = rmat16k["out"]
    V = len(rp) - 1
    assert V == 16384 and rp[0] == 0 and rp[-1] == len(col) and np.all(np.diff(rp) >= 0)
    assert col.dtype == np.int32 and rp.dtype == np.int64
    assert col.min() >= 0 and col.max() < V
    src = np.repeat(np.arange(V), np.diff(rp))
    keys = src.astype(np.int64) * V + col
    assert np.all(np.diff(keys) > 0)                      # sorted by (u, v), no duplicate edge
    assert 0.8 * 262144 < len(col) <= 262144              # de-duplication removes a modest share
    rp2, col2 = rmat_csr(V, 262144, 1)
    assert np.array_equal(rp2.numpy(), rp) and np.array_equal(col2.numpy(), col)
    rp3, col3 = rmat_csr(V, 262144, 2)
    assert not np.array_equal(rp3.numpy(), rp)


def test_rmat_degrees_are_skewed(rmat16k):
    rp, _ = rmat16k["out"]
    deg = np.diff(rp)
    assert deg.max() > 50 * deg.mean()                    # hubs
    assert (deg == 0).mean() > 0.1                        # and many isolated sources


def test_rmat_accepts_non_power_of_two_node_counts():
    rp, col = rmat_csr(1000, 8000, 3)
    assert rp.numel() == 1001 and int(col.max()) < 1000 and int(rp[-1]) == col.numel()


def test_transpose(rmat16k):
    rp, col = rmat16k["out"]
    rpi, coli = rmat16k["in"]
    rp_np, col_np = transpose_np(rp, col)
    assert np.array_equal(rpi, rp_np) and np.array_equal(coli, col_np)


def test_target_batches_are_distinct_and_differ_by_index():
    a = target_batch(16384, 256, 0)
    b = target_batch(16384, 256, 1)
    assert len(np.unique(a)) == 256 and len(np.unique(b)) == 256 and a.dtype == np.int32
    assert not np.array_equal(a, b)
    assert np.array_equal(a, target_batch(16384, 256, 0))
    pool = training_subset(100000, 0.011)
    assert 800 < pool.numel() < 1400 and bool((pool[1:] > pool[:-1]).all())
    t = target_batch(pool.numel(), 100, 0, pool=pool)
    assert set(t.tolist()) <= set(pool.tolist()) and len(np.unique(t)) == 100


def test_features_and_weights():
    f = feature_table(1000, 16, "f32", seed=2)
    assert f.shape == (1000, 16) and abs(float(f.mean())) < 0.05 and abs(float(f.std()) - 1) < 0.05
    assert torch.equal(f, feature_table(1000, 16, "f32", seed=2))
    assert feature_table(10, 8, "bf16").dtype == torch.bfloat16
    ws, wn, b = glorot_weights([128, 256, 64])
    assert ws[0].shape == (128, 256) and wn[1].shape == (256, 64) and np.all(b[0] == 0)
    a = np.sqrt(6 / (128 + 256))
    assert np.abs(ws[0]).max() <= a and np.abs(ws[0]).max() > 0.95 * a


def test_config_shapes():
    c = CONFIGS[2]
    assert c.dims == [128, 256, 256, 172] and c.capacity() == (916000, 915000)
    assert CONFIGS[0].dims == [32, 32, 10] and CONFIGS[4].dims == [100, 100]
