"""Pins of the oracle's remainder-bias path (Appendix C: the unused part of the stick,
1 - sum_i A[i,j], goes to a per-head embedding r).  Closed forms, invariants and finite
differences; nothing here re-types the oracle's own loop."""
import numpy as np
import pytest


def rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_zero_embedding_is_the_plain_forward(oracle):
    q, k, v = (rand((2, 3, 17, 8), s) for s in (1, 2, 3))
    o0, rem0 = oracle.fwd(q, k, v)
    o1, rem1 = oracle.fwd(q, k, v, r=np.zeros((3, 8)))
    assert np.array_equal(o0, o1) and np.array_equal(rem0, rem1)


def test_partition_of_unity(oracle):
    """weights + remainder = 1: if every value and the embedding are the same vector c, o_j = c."""
    q, k = rand((1, 2, 40, 8), 4), rand((1, 2, 40, 8), 5)
    c = rand((8,), 6)
    v = np.broadcast_to(c, (1, 2, 40, 8)).copy()
    o, _ = oracle.fwd(q, k, v, r=np.broadcast_to(c, (2, 8)).copy())
    assert np.abs(o - c).max() < 1e-13


def test_first_row_and_nothing_to_attend_to(oracle):
    q, k, v = (rand((1, 2, 12, 4), s) for s in (7, 8, 9))
    r = rand((2, 4), 10)
    o, _ = oracle.fwd(q, k, v, r=r)
    assert np.allclose(o[0, :, 0], r, atol=0, rtol=0)           # no key before the first query
    # hugely negative logits: every beta = 0, the whole stick is left over
    qn = np.ones((1, 2, 12, 4)); kn = -1e6 * np.ones((1, 2, 12, 4))
    o, rem = oracle.fwd(qn, kn, v, r=r)
    assert np.array_equal(rem, np.ones_like(rem))
    assert np.allclose(o, np.broadcast_to(r[None, :, None, :], o.shape), atol=1e-300)


def test_adds_remainder_times_embedding(oracle):
    q, k, v = (rand((2, 2, 25, 8), s) for s in (11, 12, 13))
    r = rand((2, 8), 14)
    o0, rem = oracle.fwd(q, k, v)
    o1, _ = oracle.fwd(q, k, v, r=r)
    assert np.abs(o1 - (o0 + rem[..., None] * r[None, :, None, :])).max() < 1e-13


def test_constant_logit_closed_form(oracle):
    """Geometric case: A[i,j] = b (1-b)^(j-i-1), remainder (1-b)^j."""
    T, d, c = 30, 4, -1.3
    b = 1.0 / (1.0 + np.exp(-c))
    q = np.zeros((T, d)); k = np.zeros((T, d))
    q[:, 0] = 2.0; k[:, 0] = c * np.sqrt(d) / 2.0
    v = rand((T, d), 15); r = rand((d,), 16)
    o, rem = oracle.fwd(q, k, v, r=r)
    for j in range(T):
        ref = sum(b * (1 - b) ** (j - i - 1) * v[i] for i in range(j)) + (1 - b) ** j * r
        assert np.abs(o[j] - ref).max() < 1e-12
        assert abs(rem[j] - (1 - b) ** j) < 1e-13


@pytest.mark.parametrize("T,d", [(8, 4), (12, 8)])
def test_gradients_by_finite_differences(oracle, T, d):
    B, H = 2, 2
    q, k, v, g = (rand((B, H, T, d), s) for s in (20, 21, 22, 23))
    r = rand((H, d), 24)
    dq, dk, dv, dr = oracle.bwd(q, k, v, g, r=r)
    loss = lambda q_, k_, v_, r_: float((oracle.fwd(q_, k_, v_, r=r_)[0] * g).sum())
    h = 1e-6
    rng = np.random.default_rng(0)
    for name, x, grad in (("q", q, dq), ("k", k, dk), ("v", v, dv), ("r", r, dr)):
        idx = [tuple(rng.integers(0, n) for n in x.shape) for _ in range(25)]
        for ix in idx:
            xp, xm = x.copy(), x.copy()
            xp[ix] += h; xm[ix] -= h
            args_p = {"q": q, "k": k, "v": v, "r": r}; args_m = dict(args_p)
            args_p[name] = xp; args_m[name] = xm
            fd = (loss(args_p["q"], args_p["k"], args_p["v"], args_p["r"]) -
                  loss(args_m["q"], args_m["k"], args_m["v"], args_m["r"])) / (2 * h)
            assert abs(fd - grad[ix]) <= 1e-6 * max(1.0, abs(fd)), (name, ix, fd, grad[ix])


def test_dr_is_the_remainder_weighted_sum_of_dout(oracle):
    q, k, v, g = (rand((3, 2, 19, 4), s) for s in (30, 31, 32, 33))
    r = rand((2, 4), 34)
    _, rem = oracle.fwd(q, k, v)
    *_, dr = oracle.bwd(q, k, v, g, r=r)
    assert np.abs(dr - np.einsum("bhj,bhjc->hc", rem, g)).max() < 1e-12


def test_zero_embedding_gives_the_plain_gradients(oracle):
    q, k, v, g = (rand((1, 2, 15, 4), s) for s in (40, 41, 42, 43))
    a = oracle.bwd(q, k, v, g)
    b = oracle.bwd(q, k, v, g, r=np.zeros((2, 4)))
    for x, y in zip(a, b[:3]):
        assert np.array_equal(x, y)
