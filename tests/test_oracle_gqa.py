"""Pins of the oracle's grouped-kv-head wrappers (query heads in consecutive groups share
one kv head): they reduce to the plain oracle head by head, and the gradients of the shared
tensors match finite differences of the grouped forward."""
import numpy as np


def rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_group_of_one_is_the_plain_oracle(oracle):
    q, k, v, g = (rand((2, 3, 14, 4), s) for s in (1, 2, 3, 4))
    assert np.array_equal(oracle.fwd_gqa(q, k, v)[0], oracle.fwd(q, k, v)[0])
    for a, b in zip(oracle.bwd_gqa(q, k, v, g), oracle.bwd(q, k, v, g)):
        assert np.array_equal(a, b)


def test_each_query_head_sees_its_groups_kv_head(oracle):
    B, H, Hkv, T, d = 2, 6, 2, 11, 4
    q = rand((B, H, T, d), 5); k = rand((B, Hkv, T, d), 6); v = rand((B, Hkv, T, d), 7)
    o, rem = oracle.fwd_gqa(q, k, v)
    for h in range(H):
        oh, rh = oracle.fwd(q[:, h], k[:, h // 3], v[:, h // 3])
        assert np.array_equal(o[:, h], oh) and np.array_equal(rem[:, h], rh)


def test_shared_gradients_by_finite_differences(oracle):
    B, H, Hkv, T, d = 1, 4, 2, 9, 4
    q = rand((B, H, T, d), 8); k = rand((B, Hkv, T, d), 9); v = rand((B, Hkv, T, d), 10)
    g = rand((B, H, T, d), 11); r = rand((H, d), 12)
    dq, dk, dv, dr = oracle.bwd_gqa(q, k, v, g, r=r)
    assert dk.shape == k.shape and dv.shape == v.shape
    args = {"q": q, "k": k, "v": v, "r": r}
    loss = lambda a: float((oracle.fwd_gqa(a["q"], a["k"], a["v"], r=a["r"])[0] * g).sum())
    h = 1e-6
    rng = np.random.default_rng(0)
    for name, grad in (("q", dq), ("k", dk), ("v", dv), ("r", dr)):
        x = args[name]
        for _ in range(20):
            ix = tuple(rng.integers(0, n) for n in x.shape)
            ap, am = dict(args), dict(args)
            ap[name] = x.copy(); ap[name][ix] += h
            am[name] = x.copy(); am[name][ix] -= h
            fd = (loss(ap) - loss(am)) / (2 * h)
            assert abs(fd - grad[ix]) <= 1e-6 * max(1.0, abs(fd)), (name, ix, fd, grad[ix])
