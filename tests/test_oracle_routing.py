"""Pins for the oracle's router, top-k gates and TAE (CPU only)."""
import numpy as np
import pytest
import scipy.special
import scipy.stats

import oracle


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


def test_logits_match_library_matmul():
    x, wr, b = _rand(1, 13, 40), _rand(2, 9, 40), _rand(3, 9)
    z = oracle.router_logits(x, wr, b)
    ref = x.astype(np.float64) @ wr.astype(np.float64).T + b.astype(np.float64)
    np.testing.assert_allclose(z, ref, rtol=1e-13, atol=1e-13)
    z0 = oracle.router_logits(x, wr, None)
    np.testing.assert_allclose(z0, ref - b, rtol=1e-13, atol=1e-13)


def test_logits_operand_orientation():
    # w_router is [E][d]: a one-hot row picks out one coordinate of x
    d, E = 5, 3
    wr = np.zeros((E, d), np.float32)
    wr[0, 4] = 1; wr[1, 2] = 2; wr[2, 0] = -1
    x = np.arange(10, dtype=np.float32).reshape(2, 5)
    z = oracle.router_logits(x, wr)
    np.testing.assert_array_equal(z, [[4, 4, 0], [9, 14, -5]])


@pytest.mark.parametrize("E,K", [(8, 2), (64, 6), (128, 8), (5, 5), (7, 1)])
def test_topk_is_library_argsort_and_softmax(E, K):
    z = np.random.default_rng(E * 31 + K).standard_normal((50, E)) * 2.0
    ids, w = oracle.topk_gates(z, K, renorm=True)
    order = np.argsort(-z.astype(np.float32), axis=1, kind="stable")[:, :K]
    np.testing.assert_array_equal(ids, order)
    p = scipy.special.softmax(z, axis=1)
    psel = np.take_along_axis(p, order, axis=1)
    np.testing.assert_allclose(w, psel / psel.sum(1, keepdims=True), rtol=1e-12)
    np.testing.assert_allclose(w.sum(1), 1.0, rtol=1e-12)
    assert (np.diff(w, axis=1) <= 0).all()          # slot 0 = largest
    ids2, w2 = oracle.topk_gates(z, K, renorm=False)
    np.testing.assert_array_equal(ids2, order)
    np.testing.assert_allclose(w2, psel, rtol=1e-12)


def test_topk_ties_go_to_lowest_index():
    z = np.array([[1.0, 3.0, 3.0, 0.0, 3.0], [2.0, 2.0, 2.0, 2.0, 2.0]])
    ids, w = oracle.topk_gates(z, 3)
    np.testing.assert_array_equal(ids, [[1, 2, 4], [0, 1, 2]])
    np.testing.assert_allclose(w, 1.0 / 3.0)


def test_topk_shift_invariance_and_large_logits():
    z = np.random.default_rng(5).standard_normal((20, 16))
    a = oracle.topk_gates(z, 4)
    b = oracle.topk_gates(z + 700.0, 4)             # exp(700+..) would overflow without the max shift
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_allclose(a[1], b[1], rtol=1e-9)
    assert np.isfinite(b[1]).all()


def test_topk_rejects_k_above_e():
    with pytest.raises(ValueError):
        oracle.topk_gates(np.zeros((1, 3)), 4)


def test_tae_closed_forms():
    # Eq. 1: uniform gates -> 1, one-hot -> 0, K=2 -> binary entropy in bits
    K = 6
    np.testing.assert_allclose(oracle.tae(np.full((1, K), 1.0 / K)), 1.0, rtol=1e-14)
    onehot = np.zeros((1, K)); onehot[0, 2] = 1.0
    np.testing.assert_allclose(oracle.tae(onehot), 0.0, atol=1e-15)
    p = np.array([0.1, 0.25, 0.5, 0.9])
    w = np.stack([p, 1 - p], axis=1)
    hb = -(p * np.log2(p) + (1 - p) * np.log2(1 - p))
    np.testing.assert_allclose(oracle.tae(w), hb, rtol=1e-13)
    w = np.random.default_rng(0).dirichlet(np.ones(8), size=30)
    np.testing.assert_allclose(oracle.tae(w), scipy.stats.entropy(w, base=8, axis=1), rtol=1e-12)
    t = oracle.tae(w)
    assert ((t >= 0) & (t <= 1)).all()
