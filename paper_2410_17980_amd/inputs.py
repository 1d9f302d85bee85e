"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds no arithmetic of the attention method: it only draws random
tensors, scales or overwrites some coordinates, and rounds to the storage type.
Both the CPU oracle and the GPU library are fed from here, so they always see
bit-identical (already rounded) values.

Everything is generated on the CPU with a torch.Generator, so a given
(recipe, seed) is the same on every machine.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    direction: str      # "fwd" or "bwd"
    dtype: str          # "f32" or "bf16": storage type of q, k, v (and dout)
    B: int
    H: int
    T: int
    d: int
    seed: int
    sharp_half: bool = False   # heads h >= H/2 get k * 3 (near-saturated sigma)


# The five workloads, in order; the seed is the index.
WORKLOADS = (
    Workload("fwd_f32_B1_H1_T256_d64", "fwd", "f32", 1, 1, 256, 64, 0),
    Workload("fwd_bf16_B8_H16_T2048_d64", "fwd", "bf16", 8, 16, 2048, 64, 1),
    Workload("fwd_bf16_B8_H16_T4096_d128", "fwd", "bf16", 8, 16, 4096, 128, 2, sharp_half=True),
    Workload("bwd_bf16_B4_H16_T2048_d128", "bwd", "bf16", 4, 16, 2048, 128, 3),
    Workload("fwd_bf16_B1_H32_T16384_d128", "fwd", "bf16", 1, 32, 16384, 128, 4),
)


def _round(x: torch.Tensor, dtype: str) -> torch.Tensor:
    if dtype == "f32":
        return x.to(torch.float32)
    if dtype == "bf16":
        return x.to(torch.bfloat16)
    raise ValueError(dtype)


def gaussian(B: int, H: int, T: int, d: int, seed: int, dtype: str = "bf16",
             sharp_half: bool = False, with_dout: bool = False):
    """q, k, v (and dout) with i.i.d. N(0,1) entries, drawn in fp32 in the order
    q, k, v, dout.  With sharp_half the k vectors of heads h >= H/2 are
    multiplied by 3 in fp32 before rounding.  Returns tensors of the storage type."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    n = 4 if with_dout else 3
    ts = [torch.randn(B, H, T, d, generator=g, dtype=torch.float32) for _ in range(n)]
    if sharp_half:
        ts[1][:, H // 2:] *= 3.0
    return tuple(_round(t, dtype) for t in ts)


def workload_tensors(w: Workload):
    return gaussian(w.B, w.H, w.T, w.d, w.seed, w.dtype, w.sharp_half,
                    with_dout=(w.direction == "bwd"))


def slice_picks(w: Workload, n: int):
    """n distinct (b, h) pairs drawn with seed 1000 + workload seed; when the
    workload has sharp heads, half of the picks come from them."""
    g = torch.Generator(device="cpu")
    g.manual_seed(1000 + w.seed)
    picks = []
    while len(picks) < n:
        b = int(torch.randint(0, w.B, (1,), generator=g))
        h = int(torch.randint(0, w.H, (1,), generator=g))
        if w.sharp_half:
            want_sharp = (len(picks) % 2 == 1)
            if (h >= w.H // 2) != want_sharp:
                continue
        if (b, h) not in picks:
            picks.append((b, h))
    return picks


def constant_logit(B: int, H: int, T: int, d: int, seed: int, kval: float,
                   dtype: str = "bf16", with_dout: bool = False):
    """Every logit equal: q = e_1 for all rows, k = kval * e_1, so that
    z = kval / sqrt(d) for every pair.  v (and dout) are N(0,1).  With a
    negative kval the weights decay slowly and reach across many key tiles."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    q = torch.zeros(B, H, T, d)
    k = torch.zeros(B, H, T, d)
    q[..., 0] = 1.0
    k[..., 0] = kval
    v = torch.randn(B, H, T, d, generator=g)
    out = [q, k, v]
    if with_dout:
        out.append(torch.randn(B, H, T, d, generator=g))
    return tuple(_round(t, dtype) for t in out)


def biased_gaussian(B: int, H: int, T: int, d: int, seed: int, shift: float,
                    dtype: str = "bf16", with_dout: bool = False):
    """N(0,1) q, k, v with the last coordinate of q set to s and of k to -s,
    s = sqrt(|shift| * sqrt(d)), so the logits are about N(-|shift|, 1): small
    sigma everywhere, weights spread over hundreds of keys (long-range carry)."""
    q, k, v, *rest = gaussian(B, H, T, d, seed, "f32", with_dout=with_dout)
    s = math.sqrt(abs(shift) * math.sqrt(d))
    q[..., d - 1] = s
    k[..., d - 1] = -s
    out = [q, k, v] + rest
    return tuple(_round(t, dtype) for t in out)


def remainder_embedding(H: int, d: int, seed: int, dtype: str = "bf16"):
    """One N(0,1) embedding per head for the remainder bias, r [H, d]."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return _round(torch.randn(H, d, generator=g, dtype=torch.float32), dtype)


def scaled_gaussian(B: int, H: int, T: int, d: int, seed: int, gain: float,
                    dtype: str = "bf16", with_dout: bool = False):
    """N(0,1) tensors with k multiplied by gain (very sharp sigma for large gain)."""
    q, k, v, *rest = gaussian(B, H, T, d, seed, "f32", with_dout=with_dout)
    k = k * gain
    out = [q, k, v] + rest
    return tuple(_round(t, dtype) for t in out)
