"""GPU parity of the grouped-kv-head entry points (query heads in consecutive groups share
a kv head; Appendix C model table) against the CPU float64 oracle, through the C ABI.
Tolerances as for the plain path: forward 2e-2 max abs; gradients
max(2e-2, 2^-8 * max|ref|) per tensor (dk, dv are sums over the group, so the bound scales
with their own largest entry)."""
import numpy as np
import pytest
import torch

from helpers import check_grad, BF16_TOL, check_m, dev, max_abs, nan_bytes, to64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sb():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2410_17980_amd import binding
    binding.load(build_if_missing=False)
    return binding


@pytest.fixture(scope="module")
def gen():
    from paper_2410_17980_amd import inputs
    return inputs


def make(gen, B, H, Hkv, T, d, seed, kind="gaussian", **kw):
    f = getattr(gen, kind)
    q, _, _, g = f(B, H, T, d, seed=seed, with_dout=True, **kw)
    _, k, v, _ = f(B, Hkv, T, d, seed=seed + 1, with_dout=True, **kw)
    return q, k, v, g


def check(sb, oracle, q, k, v, g, r=None):
    qd, kd, vd, gd = dev(q, k, v, g)
    rd = r.cuda() if r is not None else None
    o, m = sb.sb_attn_fwd_gqa(qd, kd, vd, r=rd)
    grads = sb.sb_attn_bwd_gqa(qd, kd, vd, m, gd, r=rd, workspace=nan_bytes(sb.sb_attn_bwd_workspace_bytes(*q.shape)))
    torch.cuda.synchronize()
    r64 = to64(r) if r is not None else None
    ref, rem = oracle.fwd_gqa(to64(q), to64(k), to64(v), r=r64)
    err = max_abs(to64(o), ref)
    print(f"fwd err {err:.3e}")
    assert err <= BF16_TOL
    check_m(to64(m), rem)
    refs = oracle.bwd_gqa(to64(q), to64(k), to64(v), to64(g), r=r64)
    assert len(grads) == len(refs)
    for name, a, rf in zip(("dq", "dk", "dv", "dr"), grads, refs):
        a = to64(a)
        assert a.shape == rf.shape, name
        check_grad(name, a, rf)


@pytest.mark.parametrize("H,Hkv", [(4, 2), (6, 2), (12, 4), (3, 1), (2, 2)])
@pytest.mark.parametrize("T,d", [(100, 64), (300, 128), (200, 32)])
def test_groups(sb, oracle, gen, H, Hkv, T, d):
    check(sb, oracle, *make(gen, 2, H, Hkv, T, d, seed=H * 10 + Hkv))


@pytest.mark.parametrize("T", [1, 33, 65, 129])
def test_short_and_ragged(sb, oracle, gen, T):
    check(sb, oracle, *make(gen, 1, 4, 2, T, 128, seed=50 + T))


def test_long_range_carries_per_query_head(sb, oracle, gen):
    check(sb, oracle, *make(gen, 1, 4, 2, 600, 128, seed=60, kind="biased_gaussian", shift=-6.0))


def test_sharp_group_takes_the_redo(sb, oracle, gen):
    check(sb, oracle, *make(gen, 1, 4, 2, 260, 128, seed=61, kind="scaled_gaussian", gain=12.0))


def test_with_remainder_bias(sb, oracle, gen):
    q, k, v, g = make(gen, 2, 6, 3, 200, 64, seed=62, kind="biased_gaussian", shift=-4.0)
    check(sb, oracle, q, k, v, g, r=gen.remainder_embedding(6, 64, seed=63))


def test_equals_plain_call_on_repeated_heads(sb, gen):
    """A grouped call gives, bit for bit, the plain call's o and dq on explicitly repeated kv heads."""
    q, k, v, g = make(gen, 2, 4, 2, 333, 128, seed=64)
    qd, kd, vd, gd = dev(q, k, v, g)
    o, m = sb.sb_attn_fwd_gqa(qd, kd, vd)
    dq, dk, dv = sb.sb_attn_bwd_gqa(qd, kd, vd, m, gd)
    kr, vr = (t.repeat_interleave(2, dim=1).contiguous() for t in (kd, vd))
    o2, m2 = sb.sb_attn_fwd_train(qd, kr, vr)
    dq2, dk2, dv2 = sb.sb_attn_bwd(qd, kr, vr, m2, gd)
    torch.cuda.synchronize()
    assert torch.equal(o, o2) and torch.equal(m, m2) and torch.equal(dq, dq2)
    # dk, dv: the grouped kernel adds the heads in registers, the reference in fp32 afterwards
    assert torch.allclose(dk, dk2.view(2, 2, 2, 333, 128).sum(2), rtol=1e-5, atol=1e-5)
    assert torch.allclose(dv, dv2.view(2, 2, 2, 333, 128).sum(2), rtol=1e-5, atol=1e-5)


def test_argument_errors(sb, gen):
    q, k, v, g = make(gen, 1, 4, 3, 40, 64, seed=65)
    with pytest.raises(sb.SbAttnError):
        sb.sb_attn_fwd_gqa(*dev(q, k, v))
