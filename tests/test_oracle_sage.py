"""Pins for the oracle's GraphSage forward/backward over DENSE (CPU only)."""
import numpy as np
import pytest
import torch

import oracle
from conftest import random_small_graph


def make_params(dims, rng, bias=True, aggregation="mean"):
    ws = [rng.uniform(-0.5, 0.5, (a, b)).astype(np.float32) for a, b in zip(dims[:-1], dims[1:])]
    wn = [rng.uniform(-0.5, 0.5, (a, b)).astype(np.float32) for a, b in zip(dims[:-1], dims[1:])]
    bs = [(rng.standard_normal(b) * (0.3 if bias else 0.0)).astype(np.float32) for b in dims[1:]]
    return oracle.SageParams(ws, wn, bs, aggregation=aggregation)


def small_case(seed, n=48, avg_deg=3.0, fan=(3, 2), dims=(5, 4, 3), n_targets=6):
    rng = np.random.default_rng(seed)
    rowptr, col = random_small_graph(rng, n, avg_deg)
    g = oracle.Graph(n, rowptr, col)
    targets = rng.choice(n, size=n_targets, replace=False).astype(np.int32)
    d = oracle.dense_sample(g, targets, list(fan), seed=seed)
    table = rng.standard_normal((n, dims[0]))
    params = make_params(dims, rng)
    return g, targets, d, table, params


def test_round_bf16_matches_an_independent_conversion():
    rng = np.random.default_rng(0)
    x = np.concatenate([
        rng.standard_normal(200000).astype(np.float32) * np.float32(10.0) ** rng.integers(-20, 20, 200000).astype(np.float32),
        rng.integers(0, 2**32, 200000, dtype=np.uint64).astype(np.uint32).view(np.float32),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, np.inf, -np.inf, 3.3895314e38, 1e-45], dtype=np.float32),
    ])
    x = x[~np.isnan(x)]
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    got = oracle.round_bf16(x)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # ties go to the even neighbour: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert oracle.round_bf16(np.float32(1.00390625)) == np.float32(1.0)
    assert oracle.round_bf16(np.float32(1.01171875)) == np.float32(1.015625)
    assert np.isnan(oracle.round_bf16(np.array([np.nan], dtype=np.float32)))[0]


def recursive_definition(d, table, params, targets):
    """h_v^i = AGG(h_v^{i-1}, {h_u^{i-1} : u in S(v)}) (Section 2), evaluated per node with
    memoisation, S(v) being the one sample DENSE stores for v."""
    k = len(params.w_self)
    owners = d.node_ids[d.node_id_offsets[1]:]
    sample = {int(v): d.nbrs[d.nbr_offsets[q]:d.nbr_offsets[q + 1]].tolist() for q, v in enumerate(owners)}
    memo = {}

    def h(i, v):
        if i == 0:
            return table[v].astype(np.float64)
        if (i, v) not in memo:
            nb = sample[v]
            agg = np.zeros(params.w_nbr[i - 1].shape[0])
            for u in nb:
                agg += h(i - 1, u)
            if nb and params.aggregation == "mean":
                agg /= len(nb)
            z = h(i - 1, v) @ params.w_self[i - 1].astype(np.float64) + agg @ params.w_nbr[i - 1].astype(np.float64) \
                + params.bias[i - 1].astype(np.float64)
            memo[(i, v)] = np.maximum(z, 0) if i < k else z
        return memo[(i, v)]

    return np.stack([h(k, int(t)) for t in targets])


@pytest.mark.parametrize("seed,fan,dims", [(1, (3, 2), (5, 4, 3)), (2, (2, 2, 2), (4, 6, 5, 2)), (3, (4,), (3, 7)),
                                           (4, (1, 1, 1, 1), (3, 3, 3, 3, 3))])
def test_forward_equals_recursive_definition(seed, fan, dims):
    g, targets, d, table, params = small_case(seed, fan=fan, dims=dims)
    h0 = oracle.dense_gather(np.ascontiguousarray(table), d.node_ids)
    st = oracle.sage_forward(d, h0, params, mode="exact")
    want = recursive_definition(d, table, params, targets)
    assert st.out.shape == want.shape
    np.testing.assert_allclose(st.out, want, rtol=0, atol=1e-12)


def test_exhaustive_fanout_equals_full_graph_graphsage():
    """Fanout >= max degree: the output at the targets is full-graph GraphSage-mean,
    H <- act(H W_s + D^-1 A H W_n + b), computed with dense matrices."""
    rng = np.random.default_rng(11)
    n, dims = 40, (6, 5, 4, 3)
    rowptr, col = random_small_graph(rng, n, 2.5)
    g = oracle.Graph(n, rowptr, col)
    A = np.zeros((n, n))
    for v in range(n):
        A[v, col[rowptr[v]:rowptr[v + 1]]] = 1.0
    deg = A.sum(1)
    P = A / np.maximum(deg, 1)[:, None]
    table = rng.standard_normal((n, dims[0]))
    params = make_params(dims, rng)
    H = table.copy()
    k = len(dims) - 1
    for i in range(k):
        Z = H @ params.w_self[i].astype(np.float64) + P @ H @ params.w_nbr[i].astype(np.float64) + params.bias[i]
        H = np.maximum(Z, 0) if i < k - 1 else Z
    targets = rng.choice(n, size=9, replace=False).astype(np.int32)
    d = oracle.dense_sample(g, targets, [n] * k, seed=0)
    st = oracle.sage_forward(d, oracle.dense_gather(table, d.node_ids), params, mode="exact")
    np.testing.assert_allclose(st.out, H[targets], rtol=0, atol=1e-12)


def test_zero_neighbour_weights_give_an_mlp_on_the_targets():
    g, targets, d, table, params = small_case(5, fan=(3, 3), dims=(5, 6, 4))
    params.w_nbr = [np.zeros_like(w) for w in params.w_nbr]
    st = oracle.sage_forward(d, oracle.dense_gather(table, d.node_ids), params, mode="exact")
    x = table[targets]
    x = np.maximum(x @ params.w_self[0].astype(np.float64) + params.bias[0], 0)
    x = x @ params.w_self[1].astype(np.float64) + params.bias[1]
    np.testing.assert_allclose(st.out, x, rtol=0, atol=1e-12)


def test_additive_aggregation_reproduces_algorithm_3():
    """Algorithm 3 as printed: H' = segment_sum(H[repr_map], nbr_offsets) + H[node_id_offsets[1]:]."""
    g, targets, d, table, _ = small_case(6, fan=(3,), dims=(4, 4))
    eye = np.eye(4, dtype=np.float32)
    params = oracle.SageParams([eye], [eye], [np.zeros(4, dtype=np.float32)], aggregation="sum")
    h0 = oracle.dense_gather(table, d.node_ids)
    st = oracle.sage_forward(d, h0, params, mode="exact")
    nbr_repr = h0[d.repr_map]
    want = np.zeros((len(targets), 4))
    for q in range(len(targets)):
        want[q] = nbr_repr[d.nbr_offsets[q]:d.nbr_offsets[q + 1]].sum(0) + h0[d.node_id_offsets[1] + q]
    np.testing.assert_allclose(st.out, want, rtol=0, atol=1e-13)


def test_layer_outputs_are_rows_after_first_delta():
    """Step 1: layer i's output rows are node_ids[node_id_offsets[1]:] of the current DENSE."""
    g, targets, d, table, params = small_case(7, fan=(3, 2, 2), dims=(4, 5, 6, 3))
    st = oracle.sage_forward(d, oracle.dense_gather(table, d.node_ids), params, mode="exact")
    off = d.node_id_offsets
    for i in range(1, 4):
        assert st.h[i].shape[0] == off[-1] - off[i]
        assert st.layers[i - 1].view.node_ids.tolist() == d.node_ids[off[i - 1]:].tolist()


def loss_of(d, h0, params, gout):
    return float((oracle.sage_forward(d, h0, params, mode="exact").out * gout).sum())


@pytest.mark.parametrize("seed,fan,dims", [(21, (3, 2), (4, 5, 3)), (22, (2, 2, 2), (3, 4, 4, 2))])
def test_backward_matches_central_finite_differences(seed, fan, dims):
    g, targets, d, table, params = small_case(seed, n=30, fan=fan, dims=dims, n_targets=4)
    # keep float64 copies so that a finite step is not lost to fp32 storage
    params.w_self = [w.astype(np.float64) for w in params.w_self]
    params.w_nbr = [w.astype(np.float64) for w in params.w_nbr]
    params.bias = [b.astype(np.float64) for b in params.bias]
    rng = np.random.default_rng(seed)
    h0 = oracle.dense_gather(table, d.node_ids)
    gout = rng.standard_normal((len(targets), dims[-1]))
    st = oracle.sage_forward(d, h0, params, mode="exact")
    grads = oracle.sage_backward(st, params, gout, mode="exact")
    eps = 1e-6

    def fd(arr, idx):
        old = arr[idx]
        arr[idx] = old + eps
        up = loss_of(d, h0, params, gout)
        arr[idx] = old - eps
        dn = loss_of(d, h0, params, gout)
        arr[idx] = old
        return (up - dn) / (2 * eps)

    for i in range(len(fan)):
        for arr, grad in ((params.w_self[i], grads.d_w_self[i]), (params.w_nbr[i], grads.d_w_nbr[i]),
                          (params.bias[i], grads.d_bias[i])):
            for _ in range(12):
                idx = tuple(rng.integers(0, s) for s in arr.shape)
                assert abs(fd(arr, idx) - grad[idx]) < 1e-6 * max(1.0, abs(grad[idx]))
    for _ in range(40):
        idx = (rng.integers(0, h0.shape[0]), rng.integers(0, h0.shape[1]))
        assert abs(fd(h0, idx) - grads.d_h0[idx]) < 1e-6 * max(1.0, abs(grads.d_h0[idx]))


def test_backward_is_the_adjoint_of_the_linearised_forward():
    """Without ReLU (one layer) the map H^0 -> H^1 is linear: <G, J d> == <J^T G, d>."""
    g, targets, d, table, params = small_case(31, fan=(4,), dims=(5, 3), n_targets=8)
    params.bias = [np.zeros(3, dtype=np.float32)]
    rng = np.random.default_rng(0)
    h0 = oracle.dense_gather(table, d.node_ids)
    delta = rng.standard_normal(h0.shape)
    gout = rng.standard_normal((len(targets), 3))
    st = oracle.sage_forward(d, h0, params, mode="exact")
    j_delta = oracle.sage_forward(d, delta, params, mode="exact").out
    jt_g = oracle.sage_backward(st, params, gout, mode="exact").d_h0
    assert abs((gout * j_delta).sum() - (jt_g * delta).sum()) < 1e-10


def test_bf16_mode_rounds_operands_only():
    """In bf16 mode, with inputs and weights already representable in bfloat16 and a single
    layer, the only rounding left is that of the neighbour mean."""
    g, targets, d, table, params = small_case(41, fan=(4,), dims=(8, 4), n_targets=10)
    table = oracle.round_bf16(table.astype(np.float32)).astype(np.float64)
    params.w_self = [oracle.round_bf16(w) for w in params.w_self]
    params.w_nbr = [oracle.round_bf16(w) for w in params.w_nbr]
    h0 = oracle.dense_gather(table, d.node_ids)
    st_b = oracle.sage_forward(d, h0.astype(np.float32), params, mode="bf16")
    # rebuild by hand: fp32 sequential mean, rounded, then exact products
    want = np.zeros((len(targets), 4))
    for q in range(len(targets)):
        seg = d.repr_map[d.nbr_offsets[q]:d.nbr_offsets[q + 1]]
        acc = np.zeros(8, dtype=np.float32)
        for r in seg:
            acc = acc + h0[r].astype(np.float32)
        if len(seg):
            acc = acc / np.float32(len(seg))
        want[q] = h0[d.node_id_offsets[1] + q] @ params.w_self[0].astype(np.float64) \
            + oracle.round_bf16(acc).astype(np.float64) @ params.w_nbr[0].astype(np.float64) + params.bias[0]
    np.testing.assert_allclose(st_b.out, want.astype(np.float32), rtol=0, atol=1e-6)
    st_e = oracle.sage_forward(d, h0, params, mode="exact")
    assert np.abs(st_b.out - st_e.out).max() < 0.05


def test_bf16_backward_close_to_exact():
    g, targets, d, table, params = small_case(51, n=60, fan=(4, 3), dims=(16, 12, 5), n_targets=12)
    rng = np.random.default_rng(3)
    h0 = oracle.dense_gather(table, d.node_ids)
    gout = rng.standard_normal((len(targets), 5))
    ge = oracle.sage_backward(oracle.sage_forward(d, h0, params, "exact"), params, gout, "exact")
    gb = oracle.sage_backward(oracle.sage_forward(d, h0.astype(np.float32), params, "bf16"), params, gout, "bf16")
    for a, b in zip(ge.d_w_self + ge.d_w_nbr + ge.d_bias + [ge.d_h0], gb.d_w_self + gb.d_w_nbr + gb.d_bias + [gb.d_h0]):
        scale = np.abs(a).max() + 1e-12
        assert np.abs(a - b).max() / scale < 0.05


def test_bf16_terms_error_bounds():
    """One term is the nearest bfloat16 (8 significand bits: off by up to 2^-9 of the binade, so up to 2^-8 of the value);
    two terms reproduce a bfloat16-representable value exactly and any other fp32 value to 2^-16 of it."""
    rng = np.random.default_rng(5)
    x = (rng.standard_normal(400000) * 10.0 ** rng.integers(-6, 6, 400000)).astype(np.float32)
    x = x[np.abs(x) > 1e-30]
    x64 = x.astype(np.float64)
    e1 = np.abs(oracle.bf16_terms(x, 1) - x64) / np.abs(x64)
    e2 = np.abs(oracle.bf16_terms(x, 2) - x64) / np.abs(x64)
    assert e1.max() <= 2.0 ** -8 and e1.max() > 2.0 ** -9.5          # a single rounding is this coarse ...
    assert e2.max() <= 2.0 ** -16 and e2.max() > 2.0 ** -18          # ... the second term buys eight more bits, not all 24
    assert np.array_equal(oracle.bf16_terms(x, 1), oracle.round_bf16(x).astype(np.float64))
    rep = oracle.round_bf16(x)                                         # representable: both forms are exact
    assert np.array_equal(oracle.bf16_terms(rep, 1), rep.astype(np.float64))
    assert np.array_equal(oracle.bf16_terms(rep, 2), rep.astype(np.float64))
    # worked values: 1 + 2^-8 + 2^-12 -> hi = 1 + 2^-7 (above the tie), lo = -(2^-8 - 2^-12) = -15 * 2^-12, exact in bfloat16
    v = np.array([1.0 + 2.0 ** -8 + 2.0 ** -12], dtype=np.float32)
    assert oracle.bf16_terms(v, 1)[0] == 1.0 + 2.0 ** -7
    assert oracle.bf16_terms(v, 2)[0] == float(v[0])
    # 1 + 2^-9 + 2^-20: hi = 1, lo = bf16(2^-9 + 2^-20) = 2^-9 (the 2^-20 lies below lo's eight bits)
    v = np.array([1.0 + 2.0 ** -9 + 2.0 ** -20], dtype=np.float32)
    assert oracle.bf16_terms(v, 2)[0] == 1.0 + 2.0 ** -9


def _rb1(x):
    """nearest bfloat16 of one fp32 scalar, by torch's conversion (independent of the oracle's bit arithmetic)"""
    return float(torch.tensor(float(np.float32(x)), dtype=torch.float32).to(torch.bfloat16).to(torch.float32))


def _terms(x, n):
    """scalar fp32 x as n bfloat16 terms, summed in fp64"""
    x = np.float32(x)
    hi = np.float32(_rb1(x))
    if n == 1:
        return float(hi)
    return float(hi) + _rb1(np.float32(x - hi))


def hand_two_layer_bf16(d, h0, params, gout, fwd_terms=(1, 2), dz_terms=(2, 1)):
    """The bf16-operand reading of a TWO-layer encoder written out with scalar loops, forward and backward.
    fwd_terms[i-1]: bfloat16 terms of layer i's [self | mean] operand; dz_terms[i-1]: terms of dZ^i in the gradient
    contractions.  The reading under test is (1, 2) / (2, 1): what derives from the caller's inputs is one term, what
    the device computed through an accumulation (H^1, its means, dZ^1) is two.  The neighbour mean is an fp32 sum in
    ascending slot order and an fp32 division; H^1, dL/dH^1 are stored as fp32; weights are one term; everything
    else is fp64."""
    off = [int(v) for v in d.node_id_offsets]
    N = off[-1]
    nbr_off = [int(v) for v in d.nbr_offsets]
    rmap = [int(v) for v in d.repr_map]
    d0, d1, d2 = h0.shape[1], params.w_self[0].shape[1], params.w_self[1].shape[1]
    W = [[np.vectorize(_rb1)(params.w_self[i]).astype(np.float64), np.vectorize(_rb1)(params.w_nbr[i]).astype(np.float64)]
         for i in range(2)]
    h0 = np.asarray(h0, dtype=np.float32)

    def layer_forward(h_in, base_in, layer, d_in, d_out, terms):
        """rows p >= off[layer]; h_in row r is node_ids position base_in + r"""
        rows = N - off[layer]
        a_self = np.zeros((rows, d_in)); a_mean = np.zeros((rows, d_in)); z = np.zeros((rows, d_out))
        cnt = np.zeros(rows, dtype=np.int64)
        for ro in range(rows):
            p = off[layer] + ro
            q = p - off[1]
            seg = range(nbr_off[q], nbr_off[q + 1])
            cnt[ro] = len(seg)
            for c in range(d_in):
                acc = np.float32(0.0)
                for j in seg:
                    acc = np.float32(acc + h_in[rmap[j] - base_in, c])
                if len(seg):
                    acc = np.float32(acc / np.float32(len(seg)))
                a_mean[ro, c] = _terms(acc, terms)
                a_self[ro, c] = _terms(h_in[p - base_in, c], terms)
            for n in range(d_out):
                s = float(params.bias[layer - 1][n])
                for c in range(d_in):
                    s += a_self[ro, c] * W[layer - 1][0][c, n] + a_mean[ro, c] * W[layer - 1][1][c, n]
                z[ro, n] = s
        return a_self, a_mean, z, cnt

    s1, m1, z1, c1 = layer_forward(h0, 0, 1, d0, d1, fwd_terms[0])
    h1 = np.maximum(z1, 0.0).astype(np.float32)
    s2, m2, z2, c2 = layer_forward(h1, off[1], 2, d1, d2, fwd_terms[1])
    out = z2.astype(np.float32)

    def layer_backward(dz, a_self, a_mean, cnt, layer, base_in, rows_in, terms):
        rows, d_out = dz.shape
        d_in = a_self.shape[1]
        dzb = np.array([[_terms(dz[r, n], terms) for n in range(d_out)] for r in range(rows)]).reshape(rows, d_out)
        dws = np.zeros((d_in, d_out)); dwn = np.zeros((d_in, d_out)); db = np.zeros(d_out)
        for r in range(rows):
            for n in range(d_out):
                db[n] += dz[r, n]                                  # the bias gradient sums the unrounded dZ
                for c in range(d_in):
                    dws[c, n] += a_self[r, c] * dzb[r, n]
                    dwn[c, n] += a_mean[r, c] * dzb[r, n]
        g_in = np.zeros((rows_in, d_in))
        for r in range(rows):
            p = off[layer] + r
            q = p - off[1]
            for c in range(d_in):
                ds = sum(dzb[r, n] * W[layer - 1][0][c, n] for n in range(d_out))
                dm = sum(dzb[r, n] * W[layer - 1][1][c, n] for n in range(d_out))
                g_in[p - base_in, c] += ds
                for j in range(nbr_off[q], nbr_off[q + 1]):
                    g_in[rmap[j] - base_in, c] += dm / cnt[r]
        return dws, dwn, db, g_in.astype(np.float32).astype(np.float64)

    g2 = np.asarray(gout, dtype=np.float32).astype(np.float64)
    dws2, dwn2, db2, g1 = layer_backward(g2, s2, m2, c2, 2, off[1], N - off[1], dz_terms[1])
    dz1 = g1 * (z1 > 0.0)
    dws1, dwn1, db1, g0 = layer_backward(dz1, s1, m1, c1, 1, 0, N, dz_terms[0])
    return dict(out=out, h1=h1, dws=[dws1, dws2], dwn=[dwn1, dwn2], db=[db1, db2], dh0=g0)


def test_two_layer_bf16_mode_equals_the_reading_written_out_with_loops():
    """Pins mode="bf16" for more than one layer: one-term layer 1, two-term layer 2, one-term dZ^2, two-term dZ^1.
    The same loops with the term counts swapped must NOT agree, so a swap in the oracle cannot pass."""
    g, targets, d, table, params = small_case(61, n=40, avg_deg=3.0, fan=(3, 2), dims=(6, 5, 4), n_targets=5)
    rng = np.random.default_rng(61)
    h0 = oracle.dense_gather(table, d.node_ids).astype(np.float32)
    gout = rng.standard_normal((len(targets), 4)).astype(np.float32)
    st = oracle.sage_forward(d, h0, params, mode="bf16")
    gr = oracle.sage_backward(st, params, gout, mode="bf16")
    assert len(d.nbrs) > 20 and d.node_id_offsets[1] > 0             # both layers aggregate something

    def distance(hand):
        pairs = [(hand["out"], st.out), (hand["h1"], st.h[1]), (hand["dh0"], gr.d_h0)]
        pairs += list(zip(hand["dws"], gr.d_w_self)) + list(zip(hand["dwn"], gr.d_w_nbr)) + list(zip(hand["db"], gr.d_bias))
        return [float(np.abs(np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64)).max()) for a, b in pairs]

    same = distance(hand_two_layer_bf16(d, h0, params, gout))
    assert max(same) < 1e-6, same
    # the loops have the power to tell the readings apart: any other assignment of term counts is off by far more
    for fwd_terms, dz_terms in (((2, 1), (2, 1)), ((1, 1), (2, 1)), ((1, 2), (1, 2)), ((1, 2), (1, 1)), ((2, 2), (2, 1)),
                                ((1, 2), (2, 2))):
        other = distance(hand_two_layer_bf16(d, h0, params, gout, fwd_terms, dz_terms))
        assert max(other) > 2e-5, (fwd_terms, dz_terms, other)
