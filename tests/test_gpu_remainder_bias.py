"""GPU parity of the remainder-bias entry points (Appendix C: the unused part of the
stick goes to a per-head embedding r) against the CPU float64 oracle, through the C ABI,
on the same seeded, already-rounded bf16 inputs.

Tolerances as for the plain path: forward max abs error 2e-2; gradients
max(2e-2, 2^-8 * max|ref|) (one bf16 rounding step of the largest entry).
"""
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


def check_fwd(sb, oracle, q, k, v, r):
    qd, kd, vd, rd = dev(q, k, v, r)
    o, m = sb.sb_attn_fwd_rb(qd, kd, vd, rd)
    o2 = sb.sb_attn_fwd_rb(qd, kd, vd, rd, want_m=False)
    torch.cuda.synchronize()
    ref, rem = oracle.fwd(to64(q), to64(k), to64(v), r=to64(r))
    err = max_abs(to64(o), ref)
    print(f"fwd err {err:.3e}")
    assert err <= BF16_TOL, err
    assert torch.equal(o, o2)
    check_m(to64(m), rem)
    return qd, kd, vd, rd, m


def check_bwd(sb, oracle, q, k, v, r, g):
    qd, kd, vd, rd, m = check_fwd(sb, oracle, q, k, v, r)
    gd, = dev(g)
    grads = sb.sb_attn_bwd_rb(qd, kd, vd, rd, m, gd, workspace=nan_bytes(sb.sb_attn_bwd_workspace_bytes(*q.shape)))
    torch.cuda.synchronize()
    refs = oracle.bwd(to64(q), to64(k), to64(v), to64(g), r=to64(r))
    for name, a, ref in zip(("dq", "dk", "dv", "dr"), grads, refs):
        a = to64(a)
        check_grad(name, a, ref)
    return grads


@pytest.mark.parametrize("T", [1, 2, 33, 64, 65, 129, 300])
@pytest.mark.parametrize("d", [32, 64, 128])
def test_shapes(sb, oracle, gen, T, d):
    q, k, v, g = gen.gaussian(2, 3, T, d, seed=100 + T + d, with_dout=True)
    check_bwd(sb, oracle, q, k, v, gen.remainder_embedding(3, d, seed=7), g)


@pytest.mark.parametrize("d", [32, 64, 128])
def test_large_remainder_across_tiles(sb, oracle, gen, d):
    """Logits around -6: most of the stick is left over for hundreds of keys, so the
    remainder term dominates o and the gradient of the logits."""
    q, k, v, g = gen.biased_gaussian(1, 2, 700, d, seed=5, shift=-6.0, with_dout=True)
    check_bwd(sb, oracle, q, k, v, gen.remainder_embedding(2, d, seed=8), g)


def test_constant_logits(sb, oracle, gen):
    q, k, v, g = gen.constant_logit(1, 2, 400, 128, seed=6, kval=-40.0, with_dout=True)
    check_bwd(sb, oracle, q, k, v, gen.remainder_embedding(2, 128, seed=9), g)


def test_sharp_heads_take_the_log_domain_redo(sb, oracle, gen):
    q, k, v, g = gen.scaled_gaussian(1, 2, 260, 128, seed=3, gain=12.0, with_dout=True)
    check_bwd(sb, oracle, q, k, v, gen.remainder_embedding(2, 128, seed=10), g)


def test_heads_use_their_own_embedding_and_dr_sums_the_batch(sb, oracle, gen):
    B, H, T, d = 3, 4, 150, 64
    q, k, v, g = gen.biased_gaussian(B, H, T, d, seed=12, shift=-4.0, with_dout=True)
    r = gen.remainder_embedding(H, d, seed=11)
    *_, dr = check_bwd(sb, oracle, q, k, v, r, g)
    # row 0 has nothing to attend to: the output is the head's embedding, bit for bit
    qd, kd, vd, rd = dev(q, k, v, r)
    o = sb.sb_attn_fwd_rb(qd, kd, vd, rd, want_m=False)
    torch.cuda.synchronize()
    assert torch.equal(o[:, :, 0].cpu(), r[None].expand(B, H, d))
    # dr is deterministic
    gd, = dev(g)
    _, m = sb.sb_attn_fwd_rb(qd, kd, vd, rd)
    dr2 = sb.sb_attn_bwd_rb(qd, kd, vd, rd, m, gd)[3]
    torch.cuda.synchronize()
    assert torch.equal(dr, dr2)


def test_zero_embedding_matches_the_plain_entry_points(sb, gen):
    q, k, v, g = gen.gaussian(2, 2, 333, 128, seed=21, with_dout=True)
    qd, kd, vd, gd = dev(q, k, v, g)
    rd = torch.zeros(2, 128, dtype=torch.bfloat16, device="cuda")
    o0, m0 = sb.sb_attn_fwd_train(qd, kd, vd)
    o1, m1 = sb.sb_attn_fwd_rb(qd, kd, vd, rd)
    assert torch.equal(o0, o1) and torch.equal(m0, m1)
    a = sb.sb_attn_bwd(qd, kd, vd, m0, gd)
    b = sb.sb_attn_bwd_rb(qd, kd, vd, rd, m0, gd)
    torch.cuda.synchronize()
    for x, y in zip(a, b[:3]):
        assert torch.equal(x, y)


def test_argument_errors(sb, gen):
    q, k, v = gen.gaussian(1, 2, 40, 64, seed=1)
    qd, kd, vd = dev(q, k, v)
    with pytest.raises(sb.SbAttnError):
        sb.sb_attn_fwd_rb(qd, kd, vd, torch.zeros(3, 64, dtype=torch.bfloat16, device="cuda"))
    with pytest.raises(sb.SbAttnError):
        sb.sb_attn_fwd_rb(qd, kd, vd, torch.zeros(2, 64, dtype=torch.float32, device="cuda"))
