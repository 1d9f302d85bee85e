"""GPU parity of the packed variable-length entry points (sequences packed along T attend
only inside themselves) against the CPU float64 oracle, through the C ABI.  Tolerances as
for the plain path: forward 2e-2 max abs; gradients max(2e-2, 2^-8 * max|ref|) per tensor."""
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


def packed(gen, H, Hkv, lens, d, seed, kind="gaussian", **kw):
    """q, k, v, dout packed [H, Ttot, d] and the int32 offsets."""
    Ttot = sum(lens)
    f = getattr(gen, kind)
    q, _, _, g = f(1, H, Ttot, d, seed=seed, with_dout=True, **kw)
    _, k, v, _ = f(1, Hkv, Ttot, d, seed=seed + 1, with_dout=True, **kw)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    return q[0], k[0], v[0], g[0], cu


def check(sb, oracle, q, k, v, g, cu, max_T=None, r=None):
    lens = np.diff(cu)
    max_T = int(lens.max()) if max_T is None else max_T
    qd, kd, vd, gd = dev(q, k, v, g)
    cud = torch.from_numpy(cu).cuda()
    rd = r.cuda() if r is not None else None
    o, m = sb.sb_attn_varlen_fwd(qd, kd, vd, cud, max_T, r=rd)
    ws = nan_bytes(sb.sb_attn_varlen_bwd_workspace_bytes(len(cu) - 1, q.shape[0], q.shape[1], max_T, q.shape[2]))
    grads = sb.sb_attn_varlen_bwd(qd, kd, vd, m, gd, cud, max_T, r=rd, workspace=ws)
    torch.cuda.synchronize()
    r64 = to64(r) if r is not None else None
    ref, rem = oracle.fwd_varlen(to64(q), to64(k), to64(v), cu, r=r64)
    err = max_abs(to64(o), ref)
    print(f"fwd err {err:.3e}")
    assert err <= BF16_TOL
    check_m(to64(m), rem)
    refs = oracle.bwd_varlen(to64(q), to64(k), to64(v), to64(g), cu, r=r64)
    assert len(grads) == len(refs)
    for name, a, rf in zip(("dq", "dk", "dv", "dr"), grads, refs):
        a = to64(a)
        assert a.shape == rf.shape, name
        check_grad(name, a, rf)
    return o, m, grads


@pytest.mark.parametrize("d", [32, 64, 128])
@pytest.mark.parametrize("lens", [[200], [1, 2, 3], [130, 0, 77, 1, 300], [64, 128, 256], [33, 500, 31], [65, 129, 1, 257]])
def test_length_mixes(sb, oracle, gen, lens, d):
    check(sb, oracle, *packed(gen, 3, 3, lens, d, seed=sum(lens) + d))


def test_grouped_heads_and_remainder_bias(sb, oracle, gen):
    q, k, v, g, cu = packed(gen, 6, 2, [150, 90, 260], 64, seed=7, kind="biased_gaussian", shift=-4.0)
    check(sb, oracle, q, k, v, g, cu, r=gen.remainder_embedding(6, 64, seed=8))


def test_long_range_inside_sequences(sb, oracle, gen):
    check(sb, oracle, *packed(gen, 2, 2, [700, 450], 128, seed=9, kind="biased_gaussian", shift=-6.0))


def test_sharp_sequences_take_the_redo(sb, oracle, gen):
    check(sb, oracle, *packed(gen, 2, 1, [260, 140], 128, seed=10, kind="scaled_gaussian", gain=12.0))


def test_loose_length_bound_gives_the_same_result(sb, oracle, gen):
    q, k, v, g, cu = packed(gen, 2, 2, [100, 40, 160], 128, seed=11)
    o1, m1, g1 = check(sb, oracle, q, k, v, g, cu)
    o2, m2, g2 = check(sb, oracle, q, k, v, g, cu, max_T=300)
    assert torch.equal(o1, o2) and torch.equal(m1, m2)
    for a, b in zip(g1, g2):
        assert torch.equal(a, b)


def test_equal_lengths_match_the_batched_call(sb, gen):
    """Packing B equal sequences gives, bit for bit, the batched entry points' results."""
    B, H, T, d = 3, 2, 200, 128
    q, k, v, g = gen.gaussian(B, H, T, d, seed=12, with_dout=True)
    qd, kd, vd, gd = dev(q, k, v, g)
    o, m = sb.sb_attn_fwd_train(qd, kd, vd)
    dq, dk, dv = sb.sb_attn_bwd(qd, kd, vd, m, gd)
    pack = lambda t: t.transpose(0, 1).reshape(H, B * T, d).contiguous()
    cu = torch.arange(0, (B + 1) * T, T, dtype=torch.int32, device="cuda")
    o2, m2 = sb.sb_attn_varlen_fwd(pack(qd), pack(kd), pack(vd), cu, T)
    dq2, dk2, dv2 = sb.sb_attn_varlen_bwd(pack(qd), pack(kd), pack(vd), m2, pack(gd), cu, T)
    torch.cuda.synchronize()
    assert torch.equal(o2, pack(o)) and torch.equal(m2, m.transpose(0, 1).reshape(H, B * T))
    assert torch.equal(dq2, pack(dq)) and torch.equal(dk2, pack(dk)) and torch.equal(dv2, pack(dv))


def test_argument_errors(sb, gen):
    q, k, v, g, cu = packed(gen, 2, 2, [40, 50], 64, seed=13)
    qd, kd, vd = dev(q, k, v)
    cud = torch.from_numpy(cu).cuda()
    with pytest.raises(sb.SbAttnError):
        sb.sb_attn_varlen_fwd(qd, kd, vd, cud, 0)
    with pytest.raises(sb.SbAttnError):
        sb.sb_attn_varlen_fwd(qd, kd, vd, cud, 91)
    with pytest.raises(sb.SbAttnError):
        sb.sb_attn_varlen_fwd(qd, kd, vd, cud.to(torch.int64), 50)
