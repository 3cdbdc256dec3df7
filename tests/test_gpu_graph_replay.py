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
