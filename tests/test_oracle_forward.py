"""Pins for the CPU oracle's forward: each test checks it against something the
paper or the mathematics fixes, written here independently of oracle/sb_oracle.c.

Index convention in these tests: arrays are [query j, key i], 0-based, key i is
valid for query j iff i < j.
"""
import math
import os

import numpy as np
import pytest


def rand_qkv(T, d, seed, gain=1.0):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((T, d)) * gain, rng.standard_normal((T, d)), rng.standard_normal((T, d))


# ---------------------------------------------------------------- brute force
def brute_force_weights(q, k):
    """Eq. 1 term by term in pure Python: an explicit product over i<k<j."""
    T, d = len(q), len(q[0])
    A = [[0.0] * T for _ in range(T)]
    for j in range(T):
        for i in range(j):
            z = sum(q[j][c] * k[i][c] for c in range(d)) / math.sqrt(d)
            w = 1.0 / (1.0 + math.exp(-z))
            for kk in range(i + 1, j):
                zk = sum(q[j][c] * k[kk][c] for c in range(d)) / math.sqrt(d)
                w *= 1.0 - 1.0 / (1.0 + math.exp(-zk))
            A[j][i] = w
    return np.array(A)


def test_brute_force_product(oracle):
    q, k, v = rand_qkv(9, 3, seed=11)
    A, beta, rem = oracle.weights(q, k)
    Ab = brute_force_weights(q.tolist(), k.tolist())
    np.testing.assert_allclose(A, Ab, rtol=1e-12, atol=1e-15)
    o, _ = oracle.fwd(q, k, v)
    np.testing.assert_allclose(o, Ab @ v, rtol=1e-12, atol=1e-14)


# ------------------------------------------------------- log-space form, Eq. 2
def log_space_weights(q, k):
    """A[i,j] = exp(z[i,j] - sum_{k=i}^{j-1} softplus(z[k,j]))   (Eq. 2)."""
    T, d = q.shape
    z = (q @ k.T) / math.sqrt(d)            # z[j, i]
    sp = np.logaddexp(0.0, z)
    A = np.zeros((T, T))
    for j in range(T):
        if j == 0:
            continue
        csum = np.cumsum(sp[j, :j][::-1])[::-1]   # sum over k = i .. j-1
        A[j, :j] = np.exp(z[j, :j] - csum)
    return A


@pytest.mark.parametrize("T,d,gain", [(40, 8, 1.0), (130, 16, 3.0)])
def test_log_space_form(oracle, T, d, gain):
    q, k, v = rand_qkv(T, d, seed=5, gain=gain)
    A, _, _ = oracle.weights(q, k)
    np.testing.assert_allclose(A, log_space_weights(q, k), rtol=1e-10, atol=1e-300)


# ------------------------------------------- gated recurrence view (section 3)
def recurrence_output(q, k, v):
    """o_j is the end state of h <- (1-beta[i,j]) h + beta[i,j] v_i, i = 1..j-1."""
    T, d = q.shape
    o = np.zeros((T, d))
    for j in range(T):
        h = np.zeros(d)
        for i in range(j):
            z = float(q[j] @ k[i]) / math.sqrt(d)
            b = 1.0 / (1.0 + math.exp(-z))
            h = (1.0 - b) * h + b * v[i]
        o[j] = h
    return o


def test_gated_recurrence(oracle):
    q, k, v = rand_qkv(50, 6, seed=3)
    o, _ = oracle.fwd(q, k, v)
    np.testing.assert_allclose(o, recurrence_output(q, k, v), rtol=1e-11, atol=1e-13)


# ------------------------------------------------------------------- row sums
def test_row_sums_and_remainder(oracle):
    q, k, v = rand_qkv(200, 8, seed=7)
    A, beta, rem = oracle.weights(q, k)
    s = A.sum(axis=1)
    assert np.all(s <= 1.0 + 1e-14) and np.all(s >= 0.0)
    # telescoping: sum_i A[i,j] = 1 - prod_{k<j} (1 - beta[k,j])
    prod = np.array([np.prod(1.0 - beta[j, :j]) for j in range(200)])
    np.testing.assert_allclose(s, 1.0 - prod, rtol=0, atol=1e-13)
    np.testing.assert_allclose(rem, prod, rtol=1e-12, atol=1e-300)
    # fwd() reports the same remainder
    _, rem2 = oracle.fwd(q, k, v)
    np.testing.assert_allclose(rem2, rem, rtol=1e-14)


def test_all_beta_tiny_attends_to_nothing(oracle):
    T, d = 16, 4
    q = np.zeros((T, d)); k = np.zeros((T, d)); v = np.ones((T, d))
    q[:, 0] = 1.0
    k[:, 0] = -200.0 * math.sqrt(d)          # z = -200 everywhere
    o, rem = oracle.fwd(q, k, v)
    assert np.abs(o).max() < 1e-80
    np.testing.assert_allclose(rem, 1.0, atol=1e-80)


# ---------------------------------------------------------------- closed forms
def test_geometric_fixture(oracle):
    path = os.path.join(os.path.dirname(__file__), "golden", "geometric_half.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    tab = np.array([[float(x) for x in r] for r in rows])
    T = tab.shape[0]
    rng = np.random.default_rng(0)
    q = np.zeros((T, 5)); k = rng.standard_normal((T, 5)); v = rng.standard_normal((T, 5))
    A, beta, rem = oracle.weights(q, k)
    assert np.array_equal(A[:, : T - 1], tab[:, 1:T])      # exact dyadic numbers
    assert np.array_equal(rem, tab[:, T])
    o, _ = oracle.fwd(q, k, v)
    np.testing.assert_allclose(o, tab[:, 1:T] @ v[: T - 1], rtol=1e-15, atol=1e-16)


@pytest.mark.parametrize("c", [-6.0, -1.0, 0.7, 4.0])
def test_constant_logit_closed_form(oracle, c):
    """A[i,j] = beta (1-beta)^(j-i-1) when every logit equals c."""
    T, d = 300, 16
    s = 0.37
    q = np.zeros((T, d)); k = np.zeros((T, d))
    q[:, 2] = s
    k[:, 2] = c * math.sqrt(d) / s
    A, _, rem = oracle.weights(q, k)
    b = 1.0 / (1.0 + math.exp(-c))
    j, i = np.meshgrid(np.arange(T), np.arange(T), indexing="ij")
    expect = np.where(i < j, b * (1.0 - b) ** np.clip(j - i - 1, 0, None), 0.0)
    np.testing.assert_allclose(A, expect, rtol=1e-10, atol=1e-300)
    np.testing.assert_allclose(rem, (1.0 - b) ** np.arange(T), rtol=1e-10, atol=1e-300)


def test_three_tokens_by_hand(oracle):
    q = np.array([[0.3, -1.2], [1.5, 0.4], [-0.7, 2.0]])
    k = np.array([[0.9, 0.1], [-0.4, 1.1], [2.0, -3.0]])
    v = np.array([[1.0, 2.0], [3.0, -1.0], [5.0, 5.0]])
    sig = lambda x: 1.0 / (1.0 + math.exp(-x))
    z = lambda j, i: float(q[j] @ k[i]) / math.sqrt(2.0)     # query j with key i
    A, _, _ = oracle.weights(q, k)
    assert np.all(A[0] == 0.0)
    assert A[1, 0] == pytest.approx(sig(z(1, 0)), rel=1e-14)
    assert A[2, 1] == pytest.approx(sig(z(2, 1)), rel=1e-14)
    assert A[2, 0] == pytest.approx(sig(z(2, 0)) * (1.0 - sig(z(2, 1))), rel=1e-14)
    assert np.all(A[np.triu_indices(3)] == 0.0)               # strictly causal
    o, _ = oracle.fwd(q, k, v)
    assert np.all(o[0] == 0.0)                                 # first token: empty sum
    np.testing.assert_allclose(o[1], sig(z(1, 0)) * v[0], rtol=1e-14)
    np.testing.assert_allclose(o[2], A[2, 0] * v[0] + A[2, 1] * v[1], rtol=1e-14)
    # the last key / value row can never matter (no later query)
    k2, v2 = k.copy(), v.copy(); k2[2] = 99.0; v2[2] = -99.0
    o2, _ = oracle.fwd(q, k2, v2)
    assert np.array_equal(o, o2)


def test_scale_is_one_over_sqrt_d(oracle):
    for d in (1, 4, 64, 128):
        q = np.full((2, d), 0.5); k = np.full((2, d), 0.25)
        A, _, _ = oracle.weights(q, k)
        z = d * 0.125 / math.sqrt(d)
        assert A[1, 0] == pytest.approx(1.0 / (1.0 + math.exp(-z)), rel=1e-14)


# ---------------------------------------------------------- saturation limits
def test_saturated_logits_pick_most_recent_positive(oracle):
    T, d = 64, 8
    q, k, v = rand_qkv(T, d, seed=21)
    o, rem = oracle.fwd(q * 1e7, k, v)
    z = q @ k.T
    for j in range(T):
        pos = [i for i in range(j) if z[j, i] > 0]
        expect = v[max(pos)] if pos else np.zeros(d)
        np.testing.assert_allclose(o[j], expect, atol=1e-9)
    assert np.all(np.isfinite(o)) and np.all(np.isfinite(rem))


def test_huge_negative_logits_give_zero(oracle):
    T, d = 32, 4
    q = np.ones((T, d)); k = -1e4 * np.ones((T, d)); v = np.ones((T, d))
    o, rem = oracle.fwd(q, k, v)
    assert np.array_equal(o, np.zeros((T, d)))
    assert np.array_equal(rem, np.ones(T))


# ------------------------------------------------------- structural properties
def test_recency_bias(oracle):
    """Equal logits: the nearer key never gets the smaller weight (section 2)."""
    T, d = 40, 4
    q = np.zeros((T, d)); k = np.zeros((T, d))
    q[:, 0] = 1.0; k[:, 0] = 0.8
    A, _, _ = oracle.weights(q, k)
    for j in range(1, T):
        row = A[j, :j]
        assert np.all(np.diff(row) >= 0.0)


def test_non_distraction(oracle):
    """A[i,j] depends only on the logits of keys i..j-1: changing earlier keys
    leaves it untouched (section 2)."""
    q, k, v = rand_qkv(60, 8, seed=2)
    A, _, _ = oracle.weights(q, k)
    k2 = k.copy(); k2[:20] = 50.0 * np.random.default_rng(1).standard_normal((20, 8))
    A2, _, _ = oracle.weights(q, k2)
    assert np.array_equal(A[:, 20:], A2[:, 20:])
    assert not np.allclose(A[21:, :20], A2[21:, :20])


def test_prefix_invariance_when_stick_is_used_up(oracle):
    """If the weights from key i on already sum to 1, earlier context is moot."""
    T, d = 30, 4
    q, k, v = rand_qkv(T, d, seed=9)
    q[:, 0] = 1.0; k[:, 0] = 0.0
    k[12, :] = 0.0; k[12, 0] = 1e4; q[:, 1:] *= 0.1          # key 12 takes everything left
    o, _ = oracle.fwd(q, k, v)
    k2, v2 = k.copy(), v.copy()
    k2[:12] = np.random.default_rng(4).standard_normal((12, d)); v2[:12] = 7.0
    o2, _ = oracle.fwd(q, k2, v2)
    np.testing.assert_allclose(o[13:], o2[13:], rtol=0, atol=1e-300)


# -------------------------------------------------------------- layout / API
def test_heads_are_independent_and_row_ranges(oracle):
    rng = np.random.default_rng(8)
    B, H, T, d = 2, 3, 33, 5
    q = rng.standard_normal((B, H, T, d)); k = rng.standard_normal((B, H, T, d)); v = rng.standard_normal((B, H, T, d))
    o, rem = oracle.fwd(q, k, v)
    assert o.shape == (B, H, T, d) and rem.shape == (B, H, T)
    for b in range(B):
        for h in range(H):
            o1, r1 = oracle.fwd(q[b, h], k[b, h], v[b, h])
            assert np.array_equal(o1, o[b, h]) and np.array_equal(r1, rem[b, h])
    o_tail, rem_tail = oracle.fwd(q, k, v, rows=(20, 33))
    assert np.array_equal(o_tail, o[:, :, 20:33]) and np.array_equal(rem_tail, rem[:, :, 20:33])


def test_single_token(oracle):
    o, rem = oracle.fwd(np.ones((1, 4)), np.ones((1, 4)), np.ones((1, 4)))
    assert np.array_equal(o, np.zeros((1, 4))) and np.array_equal(rem, np.ones(1))


def test_softplus_threshold_error_bound():
    """The paper's softplus cut at 15 (Eq. 3) changes a term by at most
    log(1+exp(-15)); a GPU path may use either form inside this bound."""
    x = np.linspace(15.0, 40.0, 1001)
    err = np.logaddexp(0.0, x) - x
    assert err.max() == pytest.approx(math.log1p(math.exp(-15.0)), rel=1e-12)
    assert err.max() < 3.1e-7
