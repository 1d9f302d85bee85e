"""Pins of the oracle's packed variable-length wrappers: sequences packed along T attend
only inside themselves."""
import numpy as np


def rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


CU = [0, 5, 5, 12, 13, 20]       # an empty and a one-token sequence included


def test_one_sequence_is_the_plain_oracle(oracle):
    q, k, v, g = (rand((3, 17, 4), s) for s in (1, 2, 3, 4))
    o, rem = oracle.fwd_varlen(q, k, v, [0, 17])
    o2, rem2 = oracle.fwd(q, k, v)
    assert np.array_equal(o, o2) and np.array_equal(rem, rem2)
    for a, b in zip(oracle.bwd_varlen(q, k, v, g, [0, 17]), oracle.bwd(q, k, v, g)):
        assert np.array_equal(a, b)


def test_sequences_do_not_see_each_other(oracle):
    q, k, v = (rand((2, 20, 4), s) for s in (5, 6, 7))
    o, rem = oracle.fwd_varlen(q, k, v, CU)
    # first token of every sequence has nothing to attend to
    for a in (0, 5, 12, 13):
        assert not o[:, a].any() and np.all(rem[:, a] == 1.0)
    # changing one sequence leaves the others untouched
    k2, v2 = k.copy(), v.copy()
    k2[:, 5:12] += 3.0; v2[:, 5:12] -= 2.0
    o2, _ = oracle.fwd_varlen(q, k2, v2, CU)
    keep = np.r_[0:5, 12:20]
    assert np.array_equal(o[:, keep], o2[:, keep])
    assert not np.array_equal(o[:, 6:12], o2[:, 6:12])


def test_equals_dense_attention_with_the_block_mask(oracle):
    """The same numbers from the dense weights of the whole packed row range with every
    cross-sequence logit forced to -inf (sigma = 0: takes nothing, passes the stick on)."""
    H, Ttot, d = 2, 20, 4
    q, k, v = (rand((H, Ttot, d), s) for s in (8, 9, 10))
    o, _ = oracle.fwd_varlen(q, k, v, CU)
    seq = np.zeros(Ttot, dtype=int)
    for s, (a, b) in enumerate(zip(CU, CU[1:])):
        seq[a:b] = s
    for h in range(H):
        z = q[h] @ k[h].T / np.sqrt(d)
        for j in range(Ttot):
            stick, acc = 1.0, np.zeros(d)
            for i in range(j - 1, -1, -1):
                beta = 1.0 / (1.0 + np.exp(-z[j, i])) if seq[i] == seq[j] else 0.0
                acc += beta * stick * v[h, i]
                stick *= 1.0 - beta
            assert np.abs(acc - o[h, j]).max() < 1e-12


def test_gradients_by_finite_differences(oracle):
    H, Hkv, Ttot, d = 4, 2, 20, 4
    q = rand((H, Ttot, d), 11); k = rand((Hkv, Ttot, d), 12); v = rand((Hkv, Ttot, d), 13)
    g = rand((H, Ttot, d), 14); r = rand((H, d), 15)
    dq, dk, dv, dr = oracle.bwd_varlen(q, k, v, g, CU, r=r)
    args = {"q": q, "k": k, "v": v, "r": r}
    loss = lambda a: float((oracle.fwd_varlen(a["q"], a["k"], a["v"], CU, r=a["r"])[0] * g).sum())
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
