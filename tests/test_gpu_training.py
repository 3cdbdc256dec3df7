"""End to end on the device: a few SGD steps of sample -> forward -> loss head -> backward -> weight update must lower
the loss on a task the model can learn (the label of a node is a fixed function of its own feature row)."""
import numpy as np
import pytest
import torch

import paper_2202_02365_amd as dn
from workloads import CONFIGS, feature_table, glorot_weights, target_batch
from gpu_harness import DeviceGraph, to_dev

pytestmark = pytest.mark.gpu


def test_sgd_steps_lower_the_loss(rmat16k):
    cfg = CONFIGS[0]
    rp, col = rmat16k["out"]
    dg = DeviceGraph(rp, col)
    dev = torch.device("cuda:0")
    fanouts, dims, classes, B = [6, 4], [32, 48, 4], 4, 256
    table = feature_table(cfg.num_nodes, dims[0], "f32", seed=2).to(dev)
    # the class of a node: which of its first four features is the largest
    node_class = torch.argmax(table[:, :classes], dim=1).to(torch.int32)
    w_self, w_nbr, bias = [to_dev(g) for g in glorot_weights(dims, seed=3, bias_scale=0.0)]
    batch = dn.Batch(cfg.num_nodes, B, fanouts)
    model = dn.Model(batch, dims)
    out = torch.empty((B, dims[-1]), device=dev)
    loss = torch.empty(B, device=dev)
    grad_out = torch.empty_like(out)
    grads = [[torch.empty_like(t) for t in g] for g in (w_self, w_nbr, bias)]
    lr, history = 0.5, []
    for step in range(30):
        targets = torch.from_numpy(target_batch(cfg.num_nodes, B, step)).to(dev)
        labels = node_class[targets.long()].contiguous()
        model.set_weights(w_self, w_nbr, bias)
        dn.dense_sample(batch, dg.graph, targets, step)
        dn.sage_forward_table(model, batch, table, out)
        dn.softmax_xent(out, labels, loss, grad_out, 1.0 / B)
        dn.sage_backward(model, batch, grad_out, *grads)
        for params, gs in zip((w_self, w_nbr, bias), grads):
            for p, g in zip(params, gs):
                p.sub_(lr * g)
        history.append(float(loss.mean()))
    first, last = np.mean(history[:3]), np.mean(history[-3:])
    assert np.all(np.isfinite(history))
    assert first > 1.0                      # about log(4) = 1.39 at the start
    assert last < 0.6 * first, history
