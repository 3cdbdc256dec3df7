"""GPU parity, numerics: sage_forward / sage_backward through the C ABI versus the CPU oracle in its
bf16-operand mode.  Bar: max abs error per row <= 1e-4 x the L2 norm of the oracle's row."""
import numpy as np
import pytest
import torch

import oracle
import paper_2202_02365_amd as dn
from workloads import CONFIGS, target_batch, feature_table, glorot_weights, class_labels
from gpu_harness import DeviceGraph, gpu_sample, assert_dense_equal, row_rel_err, to_dev, exact_distance_report

pytestmark = pytest.mark.gpu
TOL = 1e-4


@pytest.fixture(scope="module")
def g16k(rmat16k):
    rp, col = rmat16k["out"]
    rpi, coli = rmat16k["in"]
    return DeviceGraph(rp, col, rpi, coli)


@pytest.fixture(scope="module")
def g1m(rmat1m):
    rp, col = rmat1m["out"]
    return DeviceGraph(rp, col)


def run_case(dg, fanouts, dims, n_targets, seed, batch_index=0, direction=0, feat_dtype="f32", bias_scale=0.1,
             want_dh0=False, targets=None, aggregation="mean", from_table=False, versus_exact=False):
    V = dg.num_nodes
    if targets is None:
        targets = target_batch(V, n_targets, batch_index)
    batch = dn.Batch(V, len(targets), fanouts, direction)
    view = gpu_sample(dg, batch, targets, seed)
    d = oracle.dense_sample(dg.oracle, targets, fanouts, seed, direction)
    assert_dense_equal(view, d)

    table = feature_table(V, dims[0], feat_dtype, seed=2)
    w_self, w_nbr, bias = glorot_weights(dims, seed=3, bias_scale=bias_scale)
    in_dtype = dn.DN_F32 if feat_dtype == "f32" else dn.DN_BF16
    model = dn.Model(batch, dims, in_dtype)
    model.set_weights(to_dev(w_self), to_dev(w_nbr), to_dev(bias))
    if aggregation == "sum":
        model.set_aggregation(dn.DN_AGG_SUM)
    h0 = torch.empty((batch.node_capacity, dims[0]), dtype=table.dtype, device="cuda:0")
    table_dev = table.to("cuda:0")
    dn.dense_gather(batch, table_dev, h0)
    out = torch.empty((len(targets), dims[-1]), dtype=torch.float32, device="cuda:0")
    dn.sage_forward(model, batch, h0, out)
    if from_table:
        # layer 1 reads the table's rows itself: same values, same arithmetic, so the same bits; backward follows it
        out_gathered = out.clone()
        out.fill_(7.0)
        dn.sage_forward_table(model, batch, table_dev, out)
        assert torch.equal(out, out_gathered)

    params = oracle.SageParams(w_self, w_nbr, bias, aggregation=aggregation)
    h0_o = table.float().numpy()[d.node_ids]
    st = oracle.sage_forward(d, h0_o, params, mode="bf16")
    fwd_err = row_rel_err(out.cpu().numpy(), st.out)

    gout = oracle.mean_xent_grad(st.out, class_labels(len(targets), dims[-1]))
    grads = oracle.sage_backward(st, params, gout, mode="bf16")
    dws = [torch.full_like(t, 9.0) for t in to_dev(w_self)]
    dwn = [torch.full_like(t, 9.0) for t in to_dev(w_nbr)]
    dbs = [torch.full_like(t, 9.0) for t in to_dev(bias)]
    dh0 = torch.full((batch.node_capacity, dims[0]), 9.0, device="cuda:0") if want_dh0 else None
    dn.sage_backward(model, batch, torch.from_numpy(gout).to("cuda:0"), dws, dwn, dbs, dh0)
    torch.cuda.synchronize()
    fixups, overflow = model.status()
    assert overflow == 0, "the ReLU sign fix-up queue overflowed"
    errs = {"fwd": fwd_err}
    for i in range(len(fanouts)):
        errs["dws%d" % (i + 1)] = row_rel_err(dws[i].cpu().numpy(), grads.d_w_self[i])
        errs["dwn%d" % (i + 1)] = row_rel_err(dwn[i].cpu().numpy(), grads.d_w_nbr[i])
        errs["db%d" % (i + 1)] = row_rel_err(dbs[i].cpu().numpy(), grads.d_bias[i])
    if want_dh0:
        n = len(d.node_ids)
        errs["dh0"] = row_rel_err(dh0[:n].cpu().numpy(), grads.d_h0)
    if versus_exact:
        # distance from the fp64 oracle without any operand rounding, same upstream gradient
        st_e = oracle.sage_forward(d, h0_o, params, mode="exact")
        gr_e = oracle.sage_backward(st_e, params, gout, mode="exact")
        k = len(fanouts)
        got = {"fwd": out.cpu().numpy()}
        b16 = {"fwd": st.out}
        exa = {"fwd": st_e.out}
        for i in range(k):
            for key, dev_t, gb, ge in (("dws%d" % (i + 1), dws[i], grads.d_w_self[i], gr_e.d_w_self[i]),
                                       ("dwn%d" % (i + 1), dwn[i], grads.d_w_nbr[i], gr_e.d_w_nbr[i]),
                                       ("db%d" % (i + 1), dbs[i], grads.d_bias[i], gr_e.d_bias[i])):
                got[key], b16[key], exa[key] = dev_t.cpu().numpy(), gb, ge
        exact_distance_report("run_case%s" % (dims,), got, b16, exa, d_out=dims[-1], layers=k, tol=TOL)
    return errs, (model, batch, h0, out, st, d)


def check(errs):
    print("row-normalised errors:", {k: float("%.2e" % v) for k, v in errs.items()})
    bad = {k: v for k, v in errs.items() if not v <= TOL}
    assert not bad, "row-normalised errors above %.0e: %s (all: %s)" % (TOL, bad, errs)


def test_config0_forward_backward(g16k):
    cfg = CONFIGS[0]
    for bi in range(3):
        errs, _ = run_case(g16k, cfg.fanouts, cfg.dims, cfg.batch, seed=bi, batch_index=bi, bias_scale=0.0, versus_exact=True)
        check(errs)


def test_config1_forward_backward(g1m):
    cfg = CONFIGS[1]
    errs, _ = run_case(g1m, cfg.fanouts, cfg.dims, cfg.batch, seed=0, batch_index=0, bias_scale=0.0, versus_exact=True)
    check(errs)


@pytest.mark.parametrize("fanouts,dims", [([6], [100, 100]), ([5, 4], [32, 48, 10]), ([4, 3, 2], [64, 256, 128, 172]),
                                          ([3, 3], [7, 9, 5]), ([8], [256, 153]), ([2, 2, 2, 2], [16, 16, 16, 16, 16])])
def test_shapes_with_bias_and_input_gradient(g16k, fanouts, dims):
    """Ragged widths (padding paths of the GEMMs), scalar and vector aggregation paths, dH^0."""
    errs, _ = run_case(g16k, fanouts, dims, 200, seed=5, want_dh0=True)
    check(errs)


@pytest.mark.parametrize("n_targets", [1, 63, 64, 65, 127, 128, 129, 1087, 1088, 1089])
def test_weight_gradient_row_counts_around_the_reduction_tiles(g16k, n_targets):
    """The weight gradient reduces over a layer's rows in tiles of 64 that go from memory straight into LDS; a last
    tile with fewer rows takes another way (through registers, zeros past the end).  The last layer has exactly
    n_targets rows: none, one or several whole tiles, with and without a partial one, in one and in two splits."""
    errs, _ = run_case(g16k, [3], [40, 24], n_targets, seed=11)
    check(errs)


@pytest.mark.parametrize("fanouts,dims,n_targets", [([3], [512, 40], 200), ([2, 2], [640, 200, 24], 300), ([4], [768, 256], 1)])
def test_forward_gemm_with_a_long_reduction(g16k, fanouts, dims, n_targets):
    """Layers whose X has 1024 columns or more take the forward GEMM that loads 128 x 128 operand tiles from memory
    straight into LDS: output widths below and above one tile, row counts that end inside a tile, a single row."""
    errs, _ = run_case(g16k, fanouts, dims, n_targets, seed=13, want_dh0=True)
    check(errs)


@pytest.mark.parametrize("dims", [[32, 64, 48, 10], [20, 36, 33, 7]])
def test_rows_read_by_hundreds_of_slots(dims):
    """A star inside a ring: every node points at node 0 and at two ring neighbours, and the fanout takes all three.
    Node 0 is then read by every target's and every first-hop node's segment: in the backward aggregation of
    layers 2 and 3 its row has hundreds of transposed slots, far above the 64 that a lane group handles, and its
    gradient is the dZ row of the layer below (ReLU mask and bf16 terms applied by the workgroup that sums it).
    The second shape has widths that are no multiples of four and padding columns in every dZ."""
    V = 3000
    src = np.repeat(np.arange(V, dtype=np.int64), 3)
    dst = np.stack([np.zeros(V, dtype=np.int64), (np.arange(V) + 1) % V, (np.arange(V) + 7) % V], axis=1).reshape(-1)
    keep = src != dst                                      # node 0 does not point at itself
    src, dst = src[keep], dst[keep]
    order = np.lexsort((dst, src))
    src, dst = src[order], dst[order]
    rowptr = np.zeros(V + 1, dtype=np.int64)
    np.add.at(rowptr, src + 1, 1)
    rowptr = np.cumsum(rowptr)
    dg = DeviceGraph(rowptr, dst.astype(np.int32))
    targets = (np.arange(400, dtype=np.int32) * 5 + 11) % V           # 400 distinct nodes, none of them node 0
    errs, (_, _, _, _, _, d) = run_case(dg, [3, 3, 3], dims, len(targets), seed=4, targets=targets, want_dh0=True)
    pos0 = int(np.nonzero(np.asarray(d.node_ids) == 0)[0][0])
    readers = int(np.sum(np.asarray(d.repr_map) == pos0))
    assert readers > 500, readers                            # the hub row is what this test is about
    check(errs)


@pytest.mark.parametrize("fanouts,dims,want_dh0", [([10], [24, 20], True), ([10, 3], [24, 32, 12], False)])
def test_twenty_thousand_slots_on_a_hundred_rows(fanouts, dims, want_dh0):
    """Two thousand targets whose neighbours all lie among a hundred hub nodes: the 20,000 pairs of the transpose index
    fall into one workgroup's range of keys, so in the one-kernel form of the build every wave meets more of that
    workgroup's pairs than its list in LDS holds and places them by walking its steps instead; every hub row is read by
    about two hundred slots.  With one layer the index covers all slots (input gradient), with two only the targets'."""
    V, H = 6000, 100
    rng = np.random.default_rng(5)
    rows = []
    for u in range(V):
        if u < H:
            rows.append(np.array([(u + 1) % H, (u + 7) % H], dtype=np.int64))             # hubs: a small ring
        else:
            rows.append(np.sort(rng.choice(H, size=12, replace=False)).astype(np.int64))
    rowptr = np.zeros(V + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum([len(r) for r in rows])
    dg = DeviceGraph(rowptr, np.concatenate(rows).astype(np.int32))
    targets = (H + rng.permutation(V - H)[:2000]).astype(np.int32)
    errs, (_, _, _, _, _, d) = run_case(dg, fanouts, dims, len(targets), seed=9, targets=targets, want_dh0=want_dh0)
    first_hop = np.asarray(d.repr_map)[-2000 * fanouts[0]:]                              # the targets' slots come last
    assert len(np.unique(first_hop)) <= H and len(first_hop) == 20000
    check(errs)


def test_one_launch_layer_with_long_and_empty_segments(g16k):
    """Layers above the first with 64, 128, 192 or 256 input columns run aggregation and linear map in one launch.
    Fanout 48 over both edge directions (up to 96 slots a row) gives its rows segments beyond the 16 slots fetched at once and beyond one
    chunk of 64, next to rows without any slot; 192 input columns and 40 output columns leave lanes and waves idle."""
    errs, (_, _, _, _, _, d) = run_case(g16k, [48, 3], [24, 192, 40], 300, seed=21, direction=2, want_dh0=True)
    seg = np.diff(np.asarray(d.nbr_offsets))[-300:]                 # the targets' segments: layer 2's rows
    assert seg.max() > 64 and (seg > 16).sum() > 10 and (seg == 0).any(), (seg.max(), (seg > 16).sum(), (seg == 0).sum())
    check(errs)
    errs, _ = run_case(g16k, [40, 2], [16, 128, 256], 77, seed=22, direction=2, aggregation="sum")
    check(errs)


@pytest.mark.parametrize("feat_dtype", ["f32", "bf16"])
def test_forward_from_the_table_equals_gather_then_forward(g16k, feat_dtype):
    errs, _ = run_case(g16k, [7, 4], [36, 64, 12], 200, seed=11, feat_dtype=feat_dtype, want_dh0=True, from_table=True)
    check(errs)


def test_additive_aggregation_of_algorithm_3(g16k):
    errs, _ = run_case(g16k, [6, 5], [32, 48, 10], 150, seed=12, want_dh0=True, aggregation="sum")
    check(errs)
    errs, _ = run_case(g16k, [5], [24, 16], 90, seed=13, direction=2, want_dh0=True, aggregation="sum", from_table=True)
    check(errs)


def test_bf16_features(g16k):
    errs, _ = run_case(g16k, [5, 3], [768, 256, 153], 128, seed=6, feat_dtype="bf16", want_dh0=True)
    check(errs)


def test_link_prediction_shape_both_directions(g16k):
    """One layer, fanout 20 over in- and out-edges, learnable 100-dim inputs: dH^0 is the embedding gradient."""
    errs, _ = run_case(g16k, [20], [100, 100], 1500, seed=7, direction=2, want_dh0=True)
    check(errs)


def test_degenerate_batches(g16k):
    deg = np.diff(g16k.oracle.rowptr_out)
    iso = np.nonzero(deg == 0)[0][:9].astype(np.int32)
    errs, _ = run_case(g16k, [4, 2], [32, 16, 8], 0, seed=1, targets=iso, want_dh0=True)      # no neighbour anywhere
    check(errs)
    one = np.array([int(np.argmax(deg))], dtype=np.int32)
    errs, _ = run_case(g16k, [4, 2], [32, 16, 8], 0, seed=1, targets=one, want_dh0=True)      # a single target
    check(errs)


def test_results_are_deterministic_run_to_run(g16k):
    cfg = CONFIGS[0]
    errs, (model, batch, h0, out, st, d) = run_case(g16k, cfg.fanouts, cfg.dims, cfg.batch, seed=3, want_dh0=True)
    gout = torch.from_numpy(oracle.mean_xent_grad(st.out, class_labels(cfg.batch, cfg.dims[-1]))).to("cuda:0")
    ref = None
    for _ in range(100):
        o = torch.empty_like(out)
        dn.sage_forward(model, batch, h0, o)
        dws = [torch.empty((a, b), device="cuda:0") for a, b in zip(cfg.dims[:-1], cfg.dims[1:])]
        dwn = [torch.empty_like(t) for t in dws]
        dbs = [torch.empty(b, device="cuda:0") for b in cfg.dims[1:]]
        dh0 = torch.empty((batch.node_capacity, cfg.dims[0]), device="cuda:0")
        dn.sage_backward(model, batch, gout, dws, dwn, dbs, dh0)
        n = len(d.node_ids)
        cur = [o] + dws + dwn + dbs + [dh0[:n]]
        cur = [t.clone() for t in cur]
        if ref is None:
            ref = cur
        else:
            for a, b in zip(ref, cur):
                assert torch.equal(a, b)


def test_backward_before_forward_is_an_error(g16k):
    batch = dn.Batch(g16k.num_nodes, 8, [3])
    model = dn.Model(batch, [4, 4])
    w = [torch.zeros((4, 4), device="cuda:0")]
    b = [torch.zeros(4, device="cuda:0")]
    model.set_weights(w, w, b)
    gpu_sample(g16k, batch, target_batch(g16k.num_nodes, 8, 0), 0)
    with pytest.raises(dn.DenseError) as e:
        dn.sage_backward(model, batch, torch.zeros((8, 4), device="cuda:0"), w, w, b)
    assert e.value.code == -4


@pytest.mark.parametrize("direction,fanouts,dims", [(0, [6, 4], [24, 32, 8]), (2, [5], [100, 100])])
def test_backward_with_fused_sgd_update_equals_backward_then_embedding_sgd(g16k, direction, fanouts, dims):
    V = g16k.num_nodes
    targets = target_batch(V, 300, 4)
    batch = dn.Batch(V, len(targets), fanouts, direction)
    gpu_sample(g16k, batch, targets, seed=21)
    table = feature_table(V, dims[0], "f32", seed=2).to("cuda:0")
    w_self, w_nbr, bias = glorot_weights(dims, seed=3, bias_scale=0.1)
    model = dn.Model(batch, dims)
    model.set_weights(to_dev(w_self), to_dev(w_nbr), to_dev(bias))
    out = torch.empty((len(targets), dims[-1]), device="cuda:0")
    dn.sage_forward_table(model, batch, table, out)
    gout = torch.randn(out.shape, generator=torch.Generator().manual_seed(5)).to("cuda:0")
    grads_a = [[torch.empty_like(t) for t in to_dev(g)] for g in (w_self, w_nbr, bias)]
    grads_b = [[torch.empty_like(t) for t in to_dev(g)] for g in (w_self, w_nbr, bias)]
    dh0 = torch.empty((batch.node_capacity, dims[0]), device="cuda:0")
    # two-step form on a copy of the table
    dn.sage_backward(model, batch, gout, *grads_a, dh0)
    two_step = table.clone()
    dn.embedding_sgd(batch, two_step, dh0, 0.05)
    # fused form on another copy
    fused = table.clone()
    dn.sage_backward_sgd(model, batch, gout, *grads_b, fused, 0.05)
    torch.cuda.synchronize()
    assert torch.equal(two_step, fused)
    assert not torch.equal(fused, table)
    for ga, gb in zip(grads_a, grads_b):
        for a, b in zip(ga, gb):
            assert torch.equal(a, b)
