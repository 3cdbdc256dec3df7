"""Pins of the DistMult decoder oracle (oracle/distmult.py) to things other than itself:
brute-force loops over the textbook definition, closed forms, symmetries, finite differences."""
import math

import numpy as np
import pytest

import oracle


def _case(rng, n=23, n_rel=5, d=7, B=11, chunk=4, Nn=6):
    H = rng.standard_normal((n, d)).astype(np.float32)
    R = rng.standard_normal((n_rel, d)).astype(np.float32)
    src = rng.integers(0, n, B)
    dst = rng.integers(0, n, B)
    rel = rng.integers(0, n_rel, B)
    C = (B + chunk - 1) // chunk
    neg = rng.integers(0, n, (C, Nn))
    return H, R, src, rel, dst, neg, chunk


def test_scores_match_brute_force_loops():
    rng = np.random.default_rng(1)
    H, R, src, rel, dst, neg, chunk = _case(rng)
    st = oracle.distmult_forward(H, R, src, rel, dst, neg, chunk)
    d = H.shape[1]
    for e in range(len(src)):
        q = e // chunk
        pos = sum(float(H[src[e], j]) * float(R[rel[e], j]) * float(H[dst[e], j]) for j in range(d))
        assert st.pos[e] == pytest.approx(pos, rel=1e-12, abs=1e-12)
        tot_d, tot_s = math.exp(pos), math.exp(pos)
        for n in range(neg.shape[1]):
            v = neg[q, n]
            sd = sum(float(H[src[e], j]) * float(R[rel[e], j]) * float(H[v, j]) for j in range(d))
            ss = sum(float(H[v, j]) * float(R[rel[e], j]) * float(H[dst[e], j]) for j in range(d))
            assert st.neg_dst[e, n] == pytest.approx(sd, rel=1e-12, abs=1e-12)
            assert st.neg_src[e, n] == pytest.approx(ss, rel=1e-12, abs=1e-12)
            tot_d += math.exp(sd)
            tot_s += math.exp(ss)
        loss = (math.log(tot_d) - pos) + (math.log(tot_s) - pos)
        assert st.loss[e] == pytest.approx(loss, rel=1e-11)


def test_one_negative_is_softplus():
    # one negative per side: -log softmax = log(1 + exp(neg - pos))
    rng = np.random.default_rng(2)
    H, R, src, rel, dst, neg, chunk = _case(rng, B=5, chunk=2, Nn=1)
    st = oracle.distmult_forward(H, R, src, rel, dst, neg, chunk)
    want = np.log1p(np.exp(st.neg_dst[:, 0] - st.pos)) + np.log1p(np.exp(st.neg_src[:, 0] - st.pos))
    np.testing.assert_allclose(st.loss, want, rtol=1e-12)


def test_negatives_equal_to_the_true_endpoint_give_log_count():
    # every negative of a chunk is the edge's own endpoint: all Nn + 1 scores are equal, loss = 2 log(Nn + 1)
    rng = np.random.default_rng(3)
    H = rng.standard_normal((9, 4)).astype(np.float32)
    R = rng.standard_normal((3, 4)).astype(np.float32)
    src, dst, rel = np.array([2, 2]), np.array([2, 2]), np.array([1, 0])
    neg = np.full((1, 5), 2)
    st = oracle.distmult_forward(H, R, src, rel, dst, neg, chunk=2)
    np.testing.assert_allclose(st.loss, 2 * math.log(6.0), rtol=1e-12)


def test_symmetry_of_the_score():
    # f(s, r, d) = f(d, r, s): swapping the endpoint arrays swaps the two corruption sides
    rng = np.random.default_rng(4)
    H, R, src, rel, dst, neg, chunk = _case(rng)
    a = oracle.distmult_forward(H, R, src, rel, dst, neg, chunk)
    b = oracle.distmult_forward(H, R, dst, rel, src, neg, chunk)
    np.testing.assert_allclose(a.pos, b.pos, rtol=1e-13)
    np.testing.assert_allclose(a.neg_dst, b.neg_src, rtol=1e-13)
    np.testing.assert_allclose(a.neg_src, b.neg_dst, rtol=1e-13)
    ga, gb = oracle.distmult_backward(a), oracle.distmult_backward(b)
    np.testing.assert_allclose(ga[0], gb[0], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(ga[1], gb[1], rtol=1e-10, atol=1e-12)


def test_chunks_are_independent():
    # a batch equals its chunks run one by one (own negatives each); gradients add up
    rng = np.random.default_rng(5)
    H, R, src, rel, dst, neg, chunk = _case(rng, B=10, chunk=4)
    whole = oracle.distmult_forward(H, R, src, rel, dst, neg, chunk)
    dH, dR = oracle.distmult_backward(whole)
    sum_dH, sum_dR = np.zeros_like(dH), np.zeros_like(dR)
    for q in range(neg.shape[0]):
        lo, hi = q * chunk, min(len(src), (q + 1) * chunk)
        part = oracle.distmult_forward(H, R, src[lo:hi], rel[lo:hi], dst[lo:hi], neg[q:q + 1], chunk)
        np.testing.assert_allclose(part.loss, whole.loss[lo:hi], rtol=1e-13)
        g = oracle.distmult_backward(part)
        sum_dH += g[0]
        sum_dR += g[1]
    np.testing.assert_allclose(dH, sum_dH, rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(dR, sum_dR, rtol=1e-10, atol=1e-13)
    # the negatives of one chunk do not reach another chunk's edges
    neg2 = neg.copy()
    neg2[1] = (neg2[1] + 1) % H.shape[0]
    other = oracle.distmult_forward(H, R, src, rel, dst, neg2, chunk)
    np.testing.assert_array_equal(other.loss[:chunk], whole.loss[:chunk])
    assert not np.allclose(other.loss[chunk:2 * chunk], whole.loss[chunk:2 * chunk])


def test_gradients_match_finite_differences():
    rng = np.random.default_rng(6)
    H, R, src, rel, dst, neg, chunk = _case(rng, n=9, n_rel=3, d=4, B=7, chunk=3, Nn=4)
    H = (0.5 * H).astype(np.float32)
    dH, dR = oracle.distmult_backward(oracle.distmult_forward(H, R, src, rel, dst, neg, chunk))

    def total(Hx, Rx):
        # the definition again, in fp64 without the oracle's float32 cast of its inputs
        tot = 0.0
        for e in range(len(src)):
            q = e // chunk
            r = Rx[rel[e]]
            pos = float((Hx[src[e]] * r * Hx[dst[e]]).sum())
            sd = np.array([(Hx[src[e]] * r * Hx[v]).sum() for v in neg[q]])
            ss = np.array([(Hx[v] * r * Hx[dst[e]]).sum() for v in neg[q]])
            tot += math.log(math.exp(pos) + np.exp(sd).sum()) - pos
            tot += math.log(math.exp(pos) + np.exp(ss).sum()) - pos
        return tot

    H64, R64 = H.astype(np.float64), R.astype(np.float64)
    eps = 1e-6
    for arr, grad, which in ((H64, dH, "H"), (R64, dR, "R")):
        for idx in np.ndindex(arr.shape):
            keep = arr[idx]
            arr[idx] = keep + eps
            up = total(H64, R64)
            arr[idx] = keep - eps
            down = total(H64, R64)
            arr[idx] = keep
            assert grad[idx] == pytest.approx((up - down) / (2 * eps), rel=2e-6, abs=2e-8), (which, idx)


def test_gradient_rows_of_untouched_nodes_and_relations_are_zero():
    rng = np.random.default_rng(7)
    H, R, src, rel, dst, neg, chunk = _case(rng, n=40, n_rel=9)
    dH, dR = oracle.distmult_backward(oracle.distmult_forward(H, R, src, rel, dst, neg, chunk))
    used = np.zeros(40, bool)
    used[src] = used[dst] = True
    used[neg.ravel()] = True
    assert np.all(dH[~used] == 0) and np.all(np.abs(dH[used]).sum(axis=1) > 0)
    used_r = np.zeros(9, bool)
    used_r[rel] = True
    assert np.all(dR[~used_r] == 0)


def test_bf16_mode_rounds_the_contraction_operands_only():
    rng = np.random.default_rng(8)
    H, R, src, rel, dst, neg, chunk = _case(rng, d=16)
    ex = oracle.distmult_forward(H, R, src, rel, dst, neg, chunk, mode="exact")
    bf = oracle.distmult_forward(H, R, src, rel, dst, neg, chunk, mode="bf16")
    np.testing.assert_array_equal(ex.pos, bf.pos)                    # the positive's score is not rounded
    # operands are bfloat16 values: 8 significant bits
    for op in (bf.q_dst, bf.q_src, bf.e_neg):
        as32 = op.astype(np.float32)
        assert np.all(as32.astype(np.float64) == op)
        assert np.all((as32.view(np.uint32) & 0xFFFF) == 0)
    # q is the rounding of the fp32 product
    np.testing.assert_array_equal(bf.q_dst, oracle.round_bf16(H[src] * R[rel]).astype(np.float64))
    # scores move by at most the operand roundings: 2 * 2^-9 relative per product
    bound = 2.0 ** -7 * (np.abs(ex.q_dst)[:, None, :] * np.abs(ex.e_neg[np.arange(len(src)) // chunk])).sum(axis=2)
    assert np.all(np.abs(bf.neg_dst - ex.neg_dst) <= bound)
    # values already representable in bfloat16 make both modes agree to fp64 rounding (two-term probabilities
    # are the only remaining difference in backward: 2^-16 relative)
    Hb, Rb = oracle.round_bf16(H), np.sign(R).astype(np.float32)
    ex = oracle.distmult_forward(Hb, Rb, src, rel, dst, neg, chunk, mode="exact")
    bf = oracle.distmult_forward(Hb, Rb, src, rel, dst, neg, chunk, mode="bf16")
    np.testing.assert_allclose(bf.neg_src, ex.neg_src, rtol=1e-13, atol=1e-13)
    ge, gb = oracle.distmult_backward(ex), oracle.distmult_backward(bf)
    np.testing.assert_allclose(gb[0], ge[0], rtol=0, atol=2.0 ** -15 * np.abs(ge[0]).max())
    np.testing.assert_allclose(gb[1], ge[1], rtol=0, atol=2.0 ** -15 * np.abs(ge[1]).max())


def test_ragged_last_chunk_and_empty_negative_list():
    rng = np.random.default_rng(9)
    H, R, src, rel, dst, neg, chunk = _case(rng, B=9, chunk=4, Nn=3)       # chunks of 4, 4, 1
    st = oracle.distmult_forward(H, R, src, rel, dst, neg, chunk)
    assert st.neg_dst.shape == (9, 3) and neg.shape[0] == 3
    # no negatives at all: softmax over the positive alone, loss 0, gradients 0
    none = oracle.distmult_forward(H, R, src, rel, dst, np.zeros((3, 0), np.int64), chunk)
    assert np.all(none.loss == 0)
    dH, dR = oracle.distmult_backward(none)
    assert np.all(dH == 0) and np.all(dR == 0)
