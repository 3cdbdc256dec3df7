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


def test_library_scheduled_steps_equal_the_calls_made_one_after_the_other(rmat16k):
    """dn_train_steps: several mini-batches in flight on streams the library owns must give, bit for bit, what the same
    chain of calls gives one mini-batch at a time (each replica has its own batch, model and output buffers)."""
    import paper_2202_02365_amd as dn
    from workloads import feature_table, glorot_weights, target_batch, class_labels
    from gpu_harness import DeviceGraph, to_dev
    rp, col = rmat16k["out"]
    dg = DeviceGraph(rp, col)
    dev = torch.device("cuda:0")
    V, B, fanouts, dims = dg.num_nodes, 96, [6, 4], [32, 40, 10]
    table = feature_table(V, dims[0], "f32", seed=2).to(dev)
    w_self, w_nbr, bias = [to_dev(g) for g in glorot_weights(dims, seed=3, bias_scale=0.1)]
    labels = torch.from_numpy(class_labels(B, dims[-1]).astype(np.int32)).to(dev)
    n_rep, n_steps = 3, 7
    targets = [torch.from_numpy(target_batch(V, B, bi)).to(dev) for bi in range(n_steps)]

    def replica():
        b = dn.Batch(V, B, fanouts)
        m = dn.Model(b, dims)
        m.set_weights(w_self, w_nbr, bias)
        return dict(batch=b, model=m, graph=dg.graph, table=table, labels=labels, grad_scale=1.0 / B,
                    out=torch.empty((B, dims[-1]), device=dev), loss=torch.empty(B, device=dev),
                    grad_out=torch.empty((B, dims[-1]), device=dev), dws=[torch.empty_like(w) for w in w_self],
                    dwn=[torch.empty_like(w) for w in w_nbr], dbs=[torch.empty_like(x) for x in bias])

    # reference: the calls one after the other on one replica
    ref = replica()
    want = []
    for bi in range(n_steps):
        dn.dense_sample(ref["batch"], dg.graph, targets[bi], bi)
        dn.sage_forward_table(ref["model"], ref["batch"], table, ref["out"])
        dn.softmax_xent(ref["out"], labels, ref["loss"], ref["grad_out"], 1.0 / B)
        dn.sage_backward(ref["model"], ref["batch"], ref["grad_out"], ref["dws"], ref["dwn"], ref["dbs"])
        torch.cuda.synchronize()
        want.append([t.clone() for t in [ref["out"], ref["loss"]] + ref["dws"] + ref["dwn"] + ref["dbs"]])

    for n_streams in (1, 3):
        reps = [replica() for _ in range(n_streams)]
        entries = [dict(reps[bi % n_streams], targets=targets[bi], seed=bi) for bi in range(n_steps)]
        steps = dn.TrainSteps(entries)
        # run in rounds of n_streams steps so that every step's outputs can be looked at before its replica is reused
        for first in range(0, n_steps, n_streams):
            count = min(n_streams, n_steps - first)
            steps.run(n_streams, first, count)
            torch.cuda.synchronize()
            for bi in range(first, first + count):
                r = reps[bi % n_streams]
                got = [r["out"], r["loss"]] + r["dws"] + r["dwn"] + r["dbs"]
                for a, b in zip(want[bi], got):
                    assert torch.equal(a, b), (n_streams, bi)
        # and all of them in one call (replicas reused along their streams): the last steps' results must be in place.
        # One replica's sizes are read back first: the library hands them on to the other batch objects of the call, and
        # all of them now build the transpose index in its one-kernel form, which must not change a bit
        reps[0]["batch"].counts()
        steps.run(n_streams)
        torch.cuda.synchronize()
        for bi in range(n_steps - n_streams, n_steps):
            r = reps[bi % n_streams]
            for a, b in zip(want[bi], [r["out"], r["loss"]] + r["dws"] + r["dwn"] + r["dbs"]):
                assert torch.equal(a, b), (n_streams, bi)
    with pytest.raises(dn.DenseError):
        steps.run(17)
    # the diagnostic of the step streams: three 20 us busy-wait kernels side by side take far less than three in a row
    one, three = dn.profile_step_stream_overlap(1, 20), dn.profile_step_stream_overlap(3, 20)
    assert 15.0 < one < 60.0 and three < 3 * one, (one, three)
    with pytest.raises(dn.DenseError):
        dn.profile_step_stream_overlap(16, 20)             # more streams than dn_train_steps has created
