"""GPU parity at the full workload sizes, in the launch configuration bench.py times: the 111M-node
graph with fp32 features, the 122M-node graph with 768-wide bf16 features, and the 86M-node
link-prediction shape sampled over in- and out-edges.  The graph is generated on the device,
copied to the host for the oracle, and the whole DENSE structure, the gathered rows, the
embeddings and the gradients are compared."""
import gc

import numpy as np
import pytest
import torch

import oracle
import paper_2202_02365_amd as dn
from workloads import CONFIGS, make_inputs, class_labels, edge_batch, relation_embeddings
from gpu_harness import assert_dense_equal, row_rel_err, to_dev, exact_distance_report

pytestmark = pytest.mark.gpu
TOL = 1e-4
# Decoder run on the device encoder's output versus oracle decoder run on the oracle encoder's output: the two
# inputs differ in the last bits (fp32 accumulation order), and where such a difference straddles a bfloat16
# rounding boundary one operand element of the score contraction moves by a whole bf16 step, 2^-8 = 4e-3
# relative.  Every score of that edge moves with it, the softmax turns a score change of delta into a relative
# change of up to delta in the probabilities, and a gradient row is a probability-weighted sum, so single rows
# can be off by a few bf16 steps of their own scale (measured: 1.4e-2 on the worst of 150,000 rows, 1.4e-3 on the
# worst edge's loss).  The bound checked here is eight steps, 2^-5 = 3.1e-2: 300 times the parity tolerance.  It is NOT a
# parity bar, only a check that the pieces fit together (index maps, strides, chunking).  The decoder's own parity is held to 1e-4 on identical inputs: here with the
# oracle's decoder run on the DEVICE encoder's output, and on synthetic inputs in test_gpu_decoder.py.
DECODER_CHAIN_WIRING_BOUND = 2.0 ** -5


def run_full(cfg, batches, n_targets=None, want_dh0=False, link_prediction=False):
    dev = torch.device("cuda:0")
    inputs = make_inputs(cfg, dev, n_batches=max(batches) + 1)
    og = oracle.Graph(cfg.num_nodes, inputs["rowptr"].cpu().numpy(), inputs["col"].cpu().numpy(),
                      None if inputs["rowptr_in"] is None else inputs["rowptr_in"].cpu().numpy(),
                      None if inputs["col_in"] is None else inputs["col_in"].cpu().numpy())
    graph = dn.Graph(inputs["rowptr"], inputs["col"], inputs["rowptr_in"], inputs["col_in"])
    batch = dn.Batch(cfg.num_nodes, cfg.batch, cfg.fanouts, cfg.direction)
    in_dtype = dn.DN_F32 if cfg.feat_dtype == "f32" else dn.DN_BF16
    model = dn.Model(batch, cfg.dims, in_dtype)
    w_self, w_nbr, bias = inputs["weights"]
    model.set_weights(to_dev(w_self), to_dev(w_nbr), to_dev(bias))
    params = oracle.SageParams(w_self, w_nbr, bias)
    table = inputs["table"]
    h0 = torch.empty((batch.node_capacity, cfg.dims[0]), dtype=table.dtype, device=dev)
    report = []
    for bi in batches:
        if not link_prediction:
            targets = inputs["targets"][bi] if n_targets is None else inputs["targets"][bi][:n_targets]
            dn.dense_sample(batch, graph, torch.from_numpy(targets).to(dev), bi)
            d = oracle.dense_sample(og, targets, cfg.fanouts, seed=bi, direction=cfg.direction)
        else:
            # link-prediction batch: uniform positive edges of the graph, shared uniform negatives per chunk
            n_edges, chunk, n_neg = cfg.lp_edges, cfg.lp_chunk, cfg.lp_negatives
            src_t, rel_t, dst_t, neg2d = edge_batch(inputs["rowptr"], inputs["col"], cfg.num_nodes, n_edges, chunk, n_neg,
                                                    cfg.num_relations, bi)
            neg_t = neg2d.reshape(-1)
            ls, ld, ln = dn.dense_sample_edges(batch, graph, src_t, dst_t, neg_t, bi)
            src, dst, neg = src_t.cpu().numpy(), dst_t.cpu().numpy(), neg_t.cpu().numpy()
            d, ols, old, oln = oracle.dense_sample_edges(og, src, dst, neg, cfg.fanouts, seed=bi, direction=cfg.direction)
            assert np.array_equal(ls.cpu().numpy(), ols) and np.array_equal(ld.cpu().numpy(), old)
            assert np.array_equal(ln.cpu().numpy(), oln)
            targets = d.node_ids[d.node_id_offsets[-2]:]
        view = {k: v.cpu().numpy() for k, v in batch.view().items()}
        assert_dense_equal(view, d)
        n = len(d.node_ids)
        dn.dense_gather(batch, table, h0)
        ids = torch.from_numpy(d.node_ids.astype(np.int64)).to(dev)
        assert torch.equal(h0[:n], table[ids])                            # gathered rows, bit for bit
        out = torch.empty((len(targets), cfg.dims[-1]), dtype=torch.float32, device=dev)
        dn.sage_forward(model, batch, h0, out)
        st = oracle.sage_forward(d, table[ids].float().cpu().numpy(), params, mode="bf16")
        errs = {"fwd": row_rel_err(out.cpu().numpy(), st.out)}
        # how far the shipped arithmetic (bfloat16 operands) is from the fp64 oracle without operand rounding
        st_exact = oracle.sage_forward(d, table[ids].float().cpu().numpy(), params, mode="exact")
        exact_distance_report("%s batch %d" % (cfg.name, bi), {"fwd": out.cpu().numpy()}, {"fwd": st.out}, {"fwd": st_exact.out},
                              d_out=cfg.dims[-1], layers=cfg.num_layers, tol=TOL)
        del st_exact
        # the form bench.py times: the first layer reads the table itself; the backward pass below follows this forward
        out_two_step = out.clone()
        out.fill_(float("nan"))
        dn.sage_forward_table(model, batch, table, out)
        assert torch.equal(out, out_two_step)
        if not link_prediction:
            gout = oracle.mean_xent_grad(st.out, class_labels(len(targets), cfg.dims[-1]))
        else:
            # link prediction: the DistMult decoder scores the encoder's output rows of the edge endpoints and the
            # shared negatives; its gradient with respect to those rows is the encoder's upstream gradient.
            # The oracle's decoder gradient feeds both encoders' backward passes (same input on both sides);
            # the device decoder runs on the device encoder's output and is compared with a tolerance for a
            # chain of two operators (see the comment at DECODER_CHAIN_WIRING_BOUND).
            num_rel = cfg.num_relations
            rel = rel_t.cpu().numpy()
            R = relation_embeddings(num_rel, cfg.dims[-1])
            ost = oracle.distmult_forward(st.out.astype(np.float32), R, ols, rel, old, oln.reshape(-1, n_neg), chunk, mode="bf16")
            o_dh, o_dr = oracle.distmult_backward(ost)
            gout = o_dh.astype(np.float32)
            dec = dn.Decoder(n_edges, chunk, n_neg, cfg.dims[-1], len(targets), num_rel)
            pos_t, loss_t = torch.empty(n_edges, device=dev), torch.empty(n_edges, device=dev)
            dn.distmult_forward(dec, out, torch.from_numpy(R).to(dev), ls, rel_t, ld,
                                ln.view(-1, n_neg), pos_t, loss_t)
            g_dh = torch.empty_like(out)
            g_dr = torch.empty((num_rel, cfg.dims[-1]), device=dev)
            dn.distmult_backward(dec, g_dh, g_dr)
            assert dec.status() == 0
            # identical inputs: the oracle's decoder on the device encoder's output
            ost_dev = oracle.distmult_forward(out.cpu().numpy(), R, ols, rel, old, oln.reshape(-1, n_neg), chunk, mode="bf16")
            odh_dev, odr_dev = oracle.distmult_backward(ost_dev)
            same = {"dec_loss": float(np.max(np.abs(loss_t.cpu().numpy() - ost_dev.loss) / np.maximum(ost_dev.loss, 1.0))),
                    "dec_dH": row_rel_err(g_dh.cpu().numpy(), odh_dev), "dec_dR": row_rel_err(g_dr.cpu().numpy(), odr_dev)}
            print(cfg.name, "decoder against the oracle's on the same input:", {k: float("%.2e" % v) for k, v in same.items()})
            assert all(v <= TOL for v in same.values()), same
            chain = {"dec_loss": float(np.max(np.abs(loss_t.cpu().numpy() - ost.loss) / np.maximum(ost.loss, 1.0))),
                     "dec_dH": row_rel_err(g_dh.cpu().numpy(), o_dh), "dec_dR": row_rel_err(g_dr.cpu().numpy(), o_dr)}
            print(cfg.name, "decoder on the encoder's output:", {k: float("%.2e" % v) for k, v in chain.items()})
            assert all(v <= DECODER_CHAIN_WIRING_BOUND for v in chain.values()), chain
            del dec
        grads = oracle.sage_backward(st, params, gout, mode="bf16")
        dws = [torch.empty_like(t) for t in to_dev(w_self)]
        dwn = [torch.empty_like(t) for t in to_dev(w_nbr)]
        dbs = [torch.empty_like(t) for t in to_dev(bias)]
        dh0 = torch.empty((batch.node_capacity, cfg.dims[0]), device=dev) if want_dh0 else None
        fused_rows = None
        if want_dh0:
            # the link-prediction step of bench.py: backward with the SGD update of the learnable rows fused in,
            # on a copy of the table; compared below, bit for bit, with backward followed by embedding_sgd
            fused_table = table.clone()
            dws2, dwn2, dbs2 = ([torch.empty_like(t) for t in g] for g in (dws, dwn, dbs))
            dn.sage_backward_sgd(model, batch, torch.from_numpy(gout).to(dev), dws2, dwn2, dbs2, fused_table, 0.01)
            fused_rows = fused_table[ids].clone()
            del fused_table
        dn.sage_backward(model, batch, torch.from_numpy(gout).to(dev), dws, dwn, dbs, dh0)
        torch.cuda.synchronize()
        if want_dh0:
            for a, b in zip(dws + dwn + dbs, dws2 + dwn2 + dbs2):
                assert torch.equal(a, b)
        assert model.status()[1] == 0
        for i in range(cfg.num_layers):
            errs["dws%d" % (i + 1)] = row_rel_err(dws[i].cpu().numpy(), grads.d_w_self[i])
            errs["dwn%d" % (i + 1)] = row_rel_err(dwn[i].cpu().numpy(), grads.d_w_nbr[i])
            errs["db%d" % (i + 1)] = row_rel_err(dbs[i].cpu().numpy(), grads.d_bias[i])
        if want_dh0:
            errs["dh0"] = row_rel_err(dh0[:n].cpu().numpy(), grads.d_h0)
            # learnable inputs: apply the update to a small stand-in table indexed by position, row by row
            probe = torch.from_numpy(d.node_ids[:2000].astype(np.int64)).to(dev)
            before = table[probe].clone()
            dn.embedding_sgd(batch, table, dh0, 0.01)
            want = before.cpu().numpy() - np.float32(0.01) * dh0[:2000].cpu().numpy()
            assert np.array_equal(table[probe].cpu().numpy().view(np.uint32), want.astype(np.float32).view(np.uint32))
            assert torch.equal(table[ids], fused_rows)
        print(cfg.name, "batch", bi, "N=%d E=%d" % (n, len(d.nbrs)), {k: float("%.2e" % v) for k, v in errs.items()})
        bad = {k: v for k, v in errs.items() if not v <= TOL}
        assert not bad, bad
        report.append((n, len(d.nbrs)))
    del inputs, graph, batch, model, table, h0, og
    gc.collect()
    torch.cuda.empty_cache()
    return report


def test_rmat111m_fp32_features():
    report = run_full(CONFIGS[2], batches=[0, 3])
    assert all(n > 20000 for n, _ in report)


def test_rmat122m_bf16_features():
    run_full(CONFIGS[3], batches=[1])


def test_rmat86m_both_directions_with_input_gradient():
    """50,000 positive edges with 1,000 shared negatives per chunk of 1,000 edges (at most 150,000 target
    nodes), 20 in- plus 20 out-neighbours, one layer, gradient with respect to the learnable inputs and
    their SGD update."""
    run_full(CONFIGS[4], batches=[0], want_dh0=True, link_prediction=True)
