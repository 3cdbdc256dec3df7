"""dense_sample_noalloc (the entry point for callers that cannot allocate: static scratch array inside the library)
against dense_sample with a caller-supplied workspace: the five arrays must be identical, on two calls in a row, the
second with a smaller input, and again after a call with another graph size has carved the array differently."""
import numpy as np
import pytest
import torch

import oracle
import paper_2202_02365_amd as dn
from workloads import target_batch
from gpu_harness import DeviceGraph, gpu_sample, assert_dense_equal

pytestmark = pytest.mark.gpu


def bound(V, n_targets, fanouts, direction):
    m = 2 if direction == dn.DN_DIR_BOTH else 1
    level = nodes = max(n_targets, 1)             # an empty request is sized like a request of one target
    slots = 0
    for f in fanouts:
        slots += level * f * m
        level = min(V, level * f * m)
        nodes += level
    return min(V, nodes), slots


def sample_noalloc(dg, targets, fanouts, direction, seed, slack=0):
    dev = torch.device("cuda:0")
    k = len(fanouts)
    ncap, scap = bound(dg.num_nodes, len(targets), fanouts, direction)
    ncap, scap = ncap + slack, scap + slack
    # outputs pre-filled with a pattern: everything past the sample must stay untouched or be in bounds
    bufs = dict(node_id_offsets=torch.full((k + 2,), -7, dtype=torch.int32, device=dev),
                node_ids=torch.full((max(ncap, 1),), -7, dtype=torch.int32, device=dev),
                nbr_offsets=torch.full((max(ncap, 1) + 1,), -7, dtype=torch.int32, device=dev),
                nbrs=torch.full((max(scap, 1),), -7, dtype=torch.int32, device=dev),
                repr_map=torch.full((max(scap, 1),), -7, dtype=torch.int32, device=dev))
    counts = torch.full((3,), -7, dtype=torch.int32, device=dev)
    t = torch.from_numpy(np.ascontiguousarray(targets, dtype=np.int32)).to(dev)
    dn.dense_sample_noalloc(dg.graph, t, fanouts, direction, seed, bufs["node_id_offsets"], bufs["node_ids"],
                            bufs["nbr_offsets"], bufs["nbrs"], bufs["repr_map"], counts)
    torch.cuda.synchronize()
    n, e, status = [int(x) for x in counts.cpu()]
    off = bufs["node_id_offsets"].cpu().numpy()
    n0 = int(off[1])
    return dict(node_id_offsets=off, node_ids=bufs["node_ids"][:n].cpu().numpy(),
                nbr_offsets=bufs["nbr_offsets"][:n - n0 + 1].cpu().numpy(), nbrs=bufs["nbrs"][:e].cpu().numpy(),
                repr_map=bufs["repr_map"][:e].cpu().numpy()), status


def reference(dg, targets, fanouts, direction, seed):
    batch = dn.Batch(dg.num_nodes, max(len(targets), 1), fanouts, direction)
    return gpu_sample(dg, batch, targets, seed)


def assert_same(a, b):
    for name in a:
        assert a[name].shape == b[name].shape, name
        assert np.array_equal(a[name], b[name]), name


def test_noalloc_equals_dense_sample_on_consecutive_calls(rmat16k, rmat1m):
    g16 = DeviceGraph(rmat16k["out"][0], rmat16k["out"][1], rmat16k["in"][0], rmat16k["in"][1])
    g1m = DeviceGraph(rmat1m["out"][0], rmat1m["out"][1])
    # first call: 2^20 nodes, 1000 targets, three hops; second call right after it: a smaller input on a smaller graph
    cases = [(g1m, target_batch(g1m.num_nodes, 1000, 0), [15, 10, 5], dn.DN_DIR_OUT, 3),
             (g16, target_batch(g16.num_nodes, 200, 1), [6, 4], dn.DN_DIR_OUT, 4),
             (g16, target_batch(g16.num_nodes, 90, 2), [20], dn.DN_DIR_BOTH, 5),
             (g1m, target_batch(g1m.num_nodes, 300, 3)[:37], [4, 3, 2], dn.DN_DIR_OUT, 6),
             (g16, np.zeros(0, dtype=np.int32), [3, 2], dn.DN_DIR_OUT, 7)]
    got = [sample_noalloc(dg, t, f, d, s) for dg, t, f, d, s in cases]            # back to back on the shared array
    for (dg, t, f, d, s), (view, status) in zip(cases, got):
        assert status == 0
        assert_same(view, reference(dg, t, f, d, s))
        assert_dense_equal(view, oracle.dense_sample(dg.oracle, t, f, s, d))


def test_noalloc_rejects_what_does_not_fit(rmat16k):
    g16 = DeviceGraph(rmat16k["out"][0], rmat16k["out"][1])
    t = target_batch(g16.num_nodes, 64, 0)
    ncap, scap = bound(g16.num_nodes, 64, [5, 5], dn.DN_DIR_OUT)
    dev = torch.device("cuda:0")
    z = lambda n: torch.zeros(n, dtype=torch.int32, device=dev)
    with pytest.raises(dn.DenseError) as e:                                      # output arrays below the bound
        dn.dense_sample_noalloc(g16.graph, torch.from_numpy(t).to(dev), [5, 5], 0, 1, z(4), z(ncap - 1), z(ncap), z(scap), z(scap), z(3))
    assert e.value.code == -2
    # a graph whose per-node tables exceed the static array: 40 million nodes need 170 MB
    big_rowptr = torch.zeros(40_000_001, dtype=torch.int64, device=dev)
    big = dn.Graph(big_rowptr, torch.zeros(1, dtype=torch.int32, device=dev))
    with pytest.raises(dn.DenseError) as e:
        dn.dense_sample_noalloc(big, torch.zeros(1, dtype=torch.int32, device=dev), [2], 0, 1, z(3), z(3), z(4), z(2), z(2), z(3))
    assert e.value.code == -2 and "static" in str(e.value)
    # invalid target sets are reported in counts[2], as dn_batch_counts reports them for dense_sample
    view, status = sample_noalloc(g16, np.array([5, 9, 5], dtype=np.int32), [3], 0, 1)
    assert status & 2
    view, status = sample_noalloc(g16, np.array([5, 16384], dtype=np.int32), [3], 0, 1)
    assert status & 1
    # and the next valid call is not disturbed by them
    t = target_batch(g16.num_nodes, 128, 5)
    view, status = sample_noalloc(g16, t, [10, 5], 0, 11, slack=13)
    assert status == 0
    assert_dense_equal(view, oracle.dense_sample(g16.oracle, t, [10, 5], 11, 0))
