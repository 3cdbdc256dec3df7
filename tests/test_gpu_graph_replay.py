"""The whole step captured in HIP graphs and replayed: every replay must give exactly what the eager step gives.
The library keeps no state on the host that a replay would miss (sizes live in device memory, the sort's
histograms are left zero by the build itself), so graphs of different mini-batches can be replayed in any order,
any number of times, with eager work in between."""
import numpy as np
import pytest
import torch

import paper_2202_02365_amd as dn
from workloads import CONFIGS, target_batch, feature_table, glorot_weights
from gpu_harness import DeviceGraph, to_dev

pytestmark = pytest.mark.gpu


def test_graph_replays_match_eager_in_any_order(rmat16k):
    cfg = CONFIGS[0]
    rp, col = rmat16k["out"]
    dg = DeviceGraph(rp, col)
    dev = torch.device("cuda:0")
    fanouts, dims = [8, 6, 4], [32, 48, 40, 12]
    table = feature_table(cfg.num_nodes, dims[0], "f32", seed=2).to(dev)
    w_self, w_nbr, bias = [to_dev(g) for g in glorot_weights(dims, seed=3, bias_scale=0.1)]
    batch = dn.Batch(cfg.num_nodes, 200, fanouts)
    model = dn.Model(batch, dims)
    model.set_weights(w_self, w_nbr, bias)
    targets = [torch.from_numpy(target_batch(cfg.num_nodes, 200, bi)).to(dev) for bi in range(4)]
    out = torch.empty((200, dims[-1]), device=dev)
    gout = torch.randn((200, dims[-1]), generator=torch.Generator().manual_seed(1)).to(dev)
    dws, dwn, dbs = ([torch.empty_like(t) for t in g] for g in (w_self, w_nbr, bias))
    dh0 = torch.empty((batch.node_capacity, dims[0]), device=dev)

    def step(bi):
        dn.dense_sample(batch, dg.graph, targets[bi], bi)
        batch.prepare_backward(True)
        dn.sage_forward_table(model, batch, table, out)
        dn.sage_backward(model, batch, gout, dws, dwn, dbs, dh0)

    def snapshot():
        torch.cuda.synchronize()
        n = batch.counts()[len(fanouts) + 1]
        return [t.clone() for t in dws + dwn + dbs + [out, dh0[:n]]]

    eager = []
    for bi in range(4):
        step(bi)
        eager.append(snapshot())

    stream = torch.cuda.Stream()
    graphs = []
    for bi in range(4):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            step(bi)
        graphs.append(g)
    torch.cuda.synchronize()

    order = [2, 0, 0, 3, 1, 3, 3, 2, 1, 0]
    for i, bi in enumerate(order):
        if i == 4:
            step(1)                      # eager work between replays
            torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            graphs[bi].replay()
        got = snapshot()
        for a, b in zip(eager[bi], got):
            assert torch.equal(a, b), (i, bi)


def test_backward_graph_without_its_index_build_is_caught_on_the_device(rmat16k):
    """A graph captured from sage_backward right after a graph that recorded prepare_backward for the same sample holds no
    index build.  Replayed after another sample has been drawn into the batch it must not aggregate through the old
    index silently: the device flags it and dn_batch_counts reports DN_ESTATE.  A graph captured from sage_backward
    without a recorded prepare_backward holds the build and replays correctly after any sample."""
    cfg = CONFIGS[0]
    rp, col = rmat16k["out"]
    dg = DeviceGraph(rp, col)
    dev = torch.device("cuda:0")
    fanouts, dims = [6, 4], [16, 24, 8]
    table = feature_table(cfg.num_nodes, dims[0], "f32", seed=2).to(dev)
    w_self, w_nbr, bias = [to_dev(g) for g in glorot_weights(dims, seed=3, bias_scale=0.1)]
    batch = dn.Batch(cfg.num_nodes, 100, fanouts)
    model = dn.Model(batch, dims)
    model.set_weights(w_self, w_nbr, bias)
    targets = [torch.from_numpy(target_batch(cfg.num_nodes, 100, bi)).to(dev) for bi in range(2)]
    out = torch.empty((100, dims[-1]), device=dev)
    gout = torch.randn((100, dims[-1]), generator=torch.Generator().manual_seed(1)).to(dev)
    dws, dwn, dbs = ([torch.empty_like(t) for t in g] for g in (w_self, w_nbr, bias))
    stream = torch.cuda.Stream()

    def eager_grads(bi):
        dn.dense_sample(batch, dg.graph, targets[bi], bi)
        dn.sage_forward_table(model, batch, table, out)
        dn.sage_backward(model, batch, gout, dws, dwn, dbs)
        torch.cuda.synchronize()
        return [t.clone() for t in dws + dwn + dbs]

    want = [eager_grads(0), eager_grads(1)]

    # (a) backward captured with the build inside: correct after any sample
    dn.dense_sample(batch, dg.graph, targets[0], 0)
    dn.sage_forward_table(model, batch, table, out)
    torch.cuda.synchronize()
    g_with = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g_with, stream=stream):
        dn.sage_backward(model, batch, gout, dws, dwn, dbs)
    for bi in (1, 0, 1):
        dn.dense_sample(batch, dg.graph, targets[bi], bi)
        dn.sage_forward_table(model, batch, table, out)
        for t in dws + dwn + dbs:
            t.fill_(7.0)
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            g_with.replay()
        torch.cuda.synchronize()
        batch.counts()                                   # no flag
        for a, b in zip(want[bi], dws + dwn + dbs):
            assert torch.equal(a, b), bi

    # (b) sample + prepare_backward captured in one graph, backward captured in another right after: the second graph
    # holds no build (the first one's covers the sample), so it is only valid behind a replay of the first
    g_prep = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g_prep, stream=stream):
        dn.dense_sample(batch, dg.graph, targets[0], 0)
        batch.prepare_backward(False)
    dn.sage_forward_table(model, batch, table, out)      # (call order: backward needs a forward on the current sample)
    torch.cuda.synchronize()
    g_without = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g_without, stream=stream):
        dn.sage_backward(model, batch, gout, dws, dwn, dbs)
    with torch.cuda.stream(stream):
        g_prep.replay()
        dn.sage_forward_table(model, batch, table, out)
        g_without.replay()                               # the index of sample 0 is in place: fine
    torch.cuda.synchronize()
    batch.counts()
    for a, b in zip(want[0], dws + dwn + dbs):
        assert torch.equal(a, b)
    dn.dense_sample(batch, dg.graph, targets[1], 1)      # another sample, no build for it
    dn.sage_forward_table(model, batch, table, out)
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        g_without.replay()
    torch.cuda.synchronize()
    with pytest.raises(dn.DenseError) as e:
        batch.counts()
    assert e.value.code == -4
    # the next sample clears the flag
    dn.dense_sample(batch, dg.graph, targets[0], 0)
    batch.counts()
