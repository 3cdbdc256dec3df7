"""Pins of oracle/heads.py: closed forms, invariants and finite differences for the softmax cross-entropy head,
hand-computed steps for Adagrad."""
import math

import numpy as np
import pytest

import oracle


def test_uniform_logits_give_log_of_class_count():
    loss, grad = oracle.softmax_xent(np.full((3, 7), 2.5), [0, 3, 6])
    np.testing.assert_allclose(loss, math.log(7.0), rtol=1e-14)
    want = np.full((3, 7), 1.0 / 7.0)
    want[[0, 1, 2], [0, 3, 6]] -= 1.0
    np.testing.assert_allclose(grad, want, rtol=1e-14)


def test_two_classes_is_the_logistic_loss():
    z = np.array([[0.3, -1.2], [4.0, 1.0]])
    loss, grad = oracle.softmax_xent(z, [0, 1])
    np.testing.assert_allclose(loss, [math.log1p(math.exp(-1.5)), math.log1p(math.exp(3.0))], rtol=1e-14)
    sig = 1.0 / (1.0 + math.exp(-3.0))                   # P(class 0) for the second row
    np.testing.assert_allclose(grad[1], [sig, -sig], rtol=1e-13)


def test_shift_invariance_large_logits_and_zero_sum_gradient():
    rng = np.random.default_rng(0)
    z = rng.standard_normal((9, 12)) * 5
    lab = rng.integers(0, 12, 9)
    a = oracle.softmax_xent(z, lab)
    b = oracle.softmax_xent(z + 1000.0, lab)              # no overflow, same result
    np.testing.assert_allclose(a[0], b[0], rtol=1e-10)
    np.testing.assert_allclose(a[1], b[1], rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(a[1].sum(axis=1), 0.0, atol=1e-14)


def test_gradient_matches_finite_differences_and_scale():
    rng = np.random.default_rng(1)
    z = rng.standard_normal((4, 5))
    lab = np.array([4, 0, 2, 2])
    _, grad = oracle.softmax_xent(z, lab, grad_scale=0.25)

    def total(zz):
        return 0.25 * sum(math.log(sum(math.exp(v) for v in row)) - row[l] for row, l in zip(zz, lab))
    eps = 1e-6
    for idx in np.ndindex(z.shape):
        up, dn = z.copy(), z.copy()
        up[idx] += eps
        dn[idx] -= eps
        assert grad[idx] == pytest.approx((total(up) - total(dn)) / (2 * eps), rel=1e-6, abs=1e-9)


def test_adagrad_hand_computed_steps():
    table = np.array([[1.0, 2.0], [3.0, 4.0], [5.0, 6.0]], dtype=np.float32)
    state = np.zeros_like(table)
    ids = np.array([2, 0])
    g = np.array([[3.0, 0.0], [-4.0, 0.5]], dtype=np.float32)
    t, s = oracle.embedding_adagrad(table, state, ids, g, lr=0.5, eps=0.0 + 1e-10)
    # first step from a zero accumulator: state = g^2, step = lr * g / |g| = lr * sign(g) (0 where g = 0)
    np.testing.assert_array_equal(s, np.array([[16.0, 0.25], [0.0, 0.0], [9.0, 0.0]], dtype=np.float32))
    np.testing.assert_allclose(t, [[1.5, 1.5], [3.0, 4.0], [4.5, 6.0]], rtol=1e-6)
    # second step with the same gradient: accumulator doubles, step shrinks by sqrt(2)
    t2, s2 = oracle.embedding_adagrad(t, s, ids, g, lr=0.5, eps=1e-10)
    np.testing.assert_array_equal(s2[2], np.float32([18.0, 0.0]))
    assert t2[2, 0] == pytest.approx(4.5 - 0.5 * 3.0 / math.sqrt(18.0), rel=1e-6)
    assert t2[1, 0] == 3.0 and s2[1, 1] == 0.0                                    # untouched row
    # inputs are not modified
    assert table[2, 0] == 5.0 and state[2, 0] == 0.0
