"""GPU parity of single-token decode (one new query against a cache of T keys/values)
against the CPU float64 oracle, through the C ABI.  Tolerance 2e-2 max abs (bf16 inputs
and output, fp32 arithmetic), m to 2e-3."""
import numpy as np
import pytest
import torch

from helpers import BF16_TOL, dev, max_abs, nan_bytes, to64

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
    q, _, _ = f(B, H, 1, d, seed=seed, **kw)
    _, k, v = f(B, Hkv, T, d, seed=seed + 1, **kw)
    return q[:, :, 0].contiguous(), k, v


def check(sb, oracle, q, k, v, T=None, r=None):
    qd, kd, vd = dev(q, k, v)
    rd = r.cuda() if r is not None else None
    Tv_ = k.shape[2] if T is None else T
    ws = nan_bytes(sb.load().sb_attn_decode_workspace_bytes(q.shape[0], q.shape[1], Tv_, q.shape[2]))
    o, m = sb.sb_attn_decode(qd, kd, vd, T=T, r=rd, want_m=True, workspace=ws)
    torch.cuda.synchronize()
    Tv = k.shape[2] if T is None else T
    ref, rem = oracle.decode(to64(q), to64(k)[:, :, :Tv], to64(v)[:, :, :Tv], r=to64(r) if r is not None else None)
    err = max_abs(to64(o), ref)
    print(f"decode err {err:.3e}")
    assert err <= BF16_TOL
    ok = rem > 1e-290
    assert np.allclose(to64(m)[ok], np.log(rem[ok]), rtol=2e-3, atol=2e-3)
    return o


@pytest.mark.parametrize("d", [32, 64, 128])
@pytest.mark.parametrize("T", [1, 2, 63, 64, 65, 300, 1000, 5000])
def test_lengths(sb, oracle, gen, T, d):
    check(sb, oracle, *make(gen, 2, 3, 3, T, d, seed=T + d))


@pytest.mark.parametrize("H,Hkv", [(4, 2), (12, 4), (5, 1), (16, 2)])
def test_grouped_heads(sb, oracle, gen, H, Hkv):
    check(sb, oracle, *make(gen, 2, H, Hkv, 700, 128, seed=H + Hkv),
          r=gen.remainder_embedding(H, 128, seed=3))


@pytest.mark.parametrize("d", [64, 128])
def test_long_range_weights_reach_across_chunks(sb, oracle, gen, d):
    """Logits around -6: the weights spread over hundreds of keys, so the order-dependent
    combination of the chunks is exercised."""
    check(sb, oracle, *make(gen, 1, 2, 2, 3000, d, seed=5, kind="biased_gaussian", shift=-6.0),
          r=gen.remainder_embedding(2, d, seed=6))


def test_constant_logit_closed_form(sb, gen):
    T, d = 2500, 64
    q, k, v = gen.constant_logit(1, 1, T, d, seed=7, kval=-48.0)
    o = sb.sb_attn_decode(*dev(q[:, :, 0].contiguous(), k, v))
    torch.cuda.synchronize()
    b = 1.0 / (1.0 + np.exp(48.0 / np.sqrt(d)))
    w = b * (1.0 - b) ** np.arange(T - 1, -1, -1)
    assert max_abs(to64(o)[0, 0], w @ to64(v)[0, 0]) <= BF16_TOL


def test_sharp_logits(sb, oracle, gen):
    check(sb, oracle, *make(gen, 1, 4, 4, 900, 128, seed=8, kind="scaled_gaussian", gain=30.0))


def test_cache_longer_than_the_valid_prefix(sb, oracle, gen):
    q, k, v = make(gen, 2, 4, 2, 1024, 128, seed=9)
    o1 = check(sb, oracle, q, k, v, T=700)
    k2, v2 = k.clone(), v.clone()
    k2[:, :, 700:] = 50.0; v2[:, :, 700:] = -7.0       # rows beyond T must not matter
    o2 = check(sb, oracle, q, k2, v2, T=700)
    assert torch.equal(o1, o2)


def test_matches_the_full_forwards_last_row(sb, gen):
    B, H, T, d = 2, 4, 777, 128
    q, k, v = gen.gaussian(B, H, T, d, seed=10)
    qd, kd, vd = dev(q, k, v)
    o = sb.sb_attn_fwd(qd, kd, vd)
    od = sb.sb_attn_decode(qd[:, :, T - 1].contiguous(), kd[:, :, :T - 1].contiguous(), vd[:, :, :T - 1].contiguous())
    torch.cuda.synchronize()
    assert max_abs(to64(od), to64(o[:, :, T - 1])) <= BF16_TOL


def test_long_cache(sb, oracle, gen):
    check(sb, oracle, *make(gen, 1, 4, 2, 70000, 128, seed=11), r=gen.remainder_embedding(4, 128, seed=12))


def test_largest_cache_the_split_reaches(sb, oracle, gen):
    """T = 524288 = 256 chunks of 2048 keys, the most one call takes."""
    T, d = 524288, 64
    q, _, _ = gen.biased_gaussian(1, 1, 1, d, seed=21, shift=-8.0)
    _, k, v = gen.biased_gaussian(1, 1, T, d, seed=22, shift=-8.0)
    q = q[:, :, 0].contiguous()
    o, m = sb.sb_attn_decode(*dev(q, k, v), want_m=True)
    torch.cuda.synchronize()
    ref, rem = oracle.decode(to64(q), to64(k), to64(v))
    assert max_abs(to64(o), ref) <= BF16_TOL
    assert np.allclose(to64(m), np.log(rem), rtol=2e-3, atol=2e-3)
    with pytest.raises(sb.SbAttnError):
        sb.sb_attn_decode(*dev(q, k, v), T=T, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))


def test_argument_errors(sb, gen):
    q, k, v = make(gen, 1, 4, 3, 40, 64, seed=13)
    with pytest.raises(sb.SbAttnError):
        sb.sb_attn_decode(*dev(q, k, v))                       # 4 query heads, 3 kv heads
    q, k, v = make(gen, 1, 2, 2, 40, 64, seed=14)
    with pytest.raises(sb.SbAttnError):
        sb.sb_attn_decode(*dev(q, k, v), T=41)                 # more valid rows than the cache holds
