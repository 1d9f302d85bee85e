"""Pins for the CPU oracle's backward: central finite differences of the oracle's
own forward (itself pinned in test_oracle_forward.py), the product-rule form of
the logit gradient derived directly from Eq. 1, and the row identity
sum_i G[i,j] = dO_j . o_j.
"""
import math

import numpy as np
import pytest


def rand4(T, d, seed, gain=1.0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((T, d)) * gain, rng.standard_normal((T, d)),
            rng.standard_normal((T, d)), rng.standard_normal((T, d)))


def loss(oracle, q, k, v, dout):
    o, _ = oracle.fwd(q, k, v)
    return float((o * dout).sum())


def finite_difference(oracle, q, k, v, dout, which, h=1e-6):
    arrs = {"q": q, "k": k, "v": v}
    base = arrs[which]
    g = np.zeros_like(base)
    for idx in np.ndindex(base.shape):
        p = base.copy(); p[idx] += h
        m = base.copy(); m[idx] -= h
        ap = dict(arrs); ap[which] = p
        am = dict(arrs); am[which] = m
        g[idx] = (loss(oracle, ap["q"], ap["k"], ap["v"], dout) -
                  loss(oracle, am["q"], am["k"], am["v"], dout)) / (2 * h)
    return g


@pytest.mark.parametrize("T,d,seed,gain", [(8, 4, 0, 1.0), (32, 8, 1, 1.0), (12, 3, 2, 4.0)])
def test_gradients_by_finite_differences(oracle, T, d, seed, gain):
    q, k, v, dout = rand4(T, d, seed, gain)
    dq, dk, dv = oracle.bwd(q, k, v, dout)
    for name, g in (("q", dq), ("k", dk), ("v", dv)):
        fd = finite_difference(oracle, q, k, v, dout, name)
        scale = np.abs(fd).max()
        assert np.abs(g - fd).max() <= 1e-6 * scale + 1e-9, name


def product_rule_grads(oracle, q, k, v, dout):
    """dZ[m,j] = (1-beta[m,j]) G[m,j] - beta[m,j] sum_{i<m} G[i,j]: the product
    rule applied to Eq. 1 (d A[i,j] / d z[m,j] is A(1-beta) for m = i, -A beta
    for i < m < j, 0 otherwise), then the chain rule through z = q.k/sqrt(d)."""
    T, d = q.shape
    A, beta, _ = oracle.weights(q, k)
    G = A * (dout @ v.T)                      # [j, i]
    excl = np.cumsum(G, axis=1) - G           # sum over i < m
    dZ = (1.0 - beta) * G - beta * excl
    dZ = np.tril(dZ, -1)
    s = 1.0 / math.sqrt(d)
    return s * dZ @ k, s * dZ.T @ q, A.T @ dout, G


@pytest.mark.parametrize("T,d,gain", [(64, 16, 1.0), (150, 8, 3.0)])
def test_product_rule_form(oracle, T, d, gain):
    q, k, v, dout = rand4(T, d, 17, gain)
    dq, dk, dv = oracle.bwd(q, k, v, dout)
    dq2, dk2, dv2, G = product_rule_grads(oracle, q, k, v, dout)
    np.testing.assert_allclose(dq, dq2, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(dk, dk2, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(dv, dv2, rtol=1e-9, atol=1e-12)
    # sum_i G[i,j] = dO_j . o_j
    o, _ = oracle.fwd(q, k, v)
    np.testing.assert_allclose(G.sum(axis=1), (dout * o).sum(axis=1), rtol=1e-9, atol=1e-12)


def test_backward_edge_rows(oracle):
    q, k, v, dout = rand4(20, 4, 5)
    dq, dk, dv = oracle.bwd(q, k, v, dout)
    assert np.array_equal(dq[0], np.zeros(4))       # first query sees no key
    assert np.array_equal(dk[-1], np.zeros(4))      # last key is seen by no query
    assert np.array_equal(dv[-1], np.zeros(4))
    dq1, dk1, dv1 = oracle.bwd(q[:1], k[:1], v[:1], dout[:1])
    assert not dq1.any() and not dk1.any() and not dv1.any()


def test_backward_batched_matches_per_head(oracle):
    rng = np.random.default_rng(6)
    B, H, T, d = 2, 2, 17, 4
    q, k, v, g = (rng.standard_normal((B, H, T, d)) for _ in range(4))
    dq, dk, dv = oracle.bwd(q, k, v, g)
    for b in range(B):
        for h in range(H):
            a, bb, c = oracle.bwd(q[b, h], k[b, h], v[b, h], g[b, h])
            assert np.array_equal(a, dq[b, h]) and np.array_equal(bb, dk[b, h]) and np.array_equal(c, dv[b, h])
