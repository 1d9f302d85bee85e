"""Pins of the oracle's single-token decode: the output for a new query over a cache of T
keys/values is Eq. 1's last row."""
import math

import numpy as np


def rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_brute_force_product(oracle):
    B, H, Hkv, T, d = 2, 4, 2, 9, 4
    q = rand((B, H, d), 1); k = rand((B, Hkv, T, d), 2); v = rand((B, Hkv, T, d), 3); r = rand((H, d), 4)
    o, rem = oracle.decode(q, k, v, r=r)
    for b in range(B):
        for h in range(H):
            kv = h // (H // Hkv)
            beta = [1.0 / (1.0 + math.exp(-float(q[b, h] @ k[b, kv, i]) / math.sqrt(d))) for i in range(T)]
            acc = np.zeros(d)
            for i in range(T):
                w = beta[i]
                for kk in range(i + 1, T):
                    w *= 1.0 - beta[kk]
                acc += w * v[b, kv, i]
            left = 1.0
            for kk in range(T):
                left *= 1.0 - beta[kk]
            assert abs(left - rem[b, h]) < 1e-13
            assert np.abs(acc + left * r[h] - o[b, h]).max() < 1e-13


def test_is_the_next_row_of_the_full_forward(oracle):
    B, H, T, d = 1, 2, 12, 4
    q, k, v = (rand((B, H, T, d), s) for s in (5, 6, 7))
    o, rem = oracle.fwd(q, k, v)
    for j in (1, 5, 11):
        oj, rj = oracle.decode(q[:, :, j], k[:, :, :j], v[:, :, :j])
        assert np.array_equal(oj, o[:, :, j]) and np.array_equal(rj, rem[:, :, j])


def test_geometric_closed_form(oracle):
    T, d = 40, 4
    q = np.zeros((1, 1, d)); k = np.zeros((1, 1, T, d)); v = rand((1, 1, T, d), 8)
    o, rem = oracle.decode(q, k, v)          # all logits 0: A[i] = 2^-(T-i)
    ref = sum(2.0 ** -(T - i) * v[0, 0, i] for i in range(T))
    assert np.abs(o[0, 0] - ref).max() < 1e-15 and rem[0, 0] == 2.0 ** -T
