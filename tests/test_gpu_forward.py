"""GPU parity: the HIP forward (through the C ABI) against the CPU float64 oracle
on the same seeded, already-rounded inputs.

Tolerances (max abs error on o): 1e-5 for the fp32 path, 2e-2 for the bf16 path
(bf16 inputs, fp32 accumulation, weights rounded to bf16 as matrix operands).
"""
import math

import numpy as np
import pytest
import torch

from helpers import BF16_TOL, F32_TOL, check_m, dev, max_abs, to64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sb():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2410_17980_amd import binding
    binding.load(build_if_missing=False)      # the built library must be there
    return binding


@pytest.fixture(scope="module")
def gen():
    from paper_2410_17980_amd import inputs
    return inputs


def run_bf16(sb, oracle, q, k, v, tol=BF16_TOL, rows=None):
    qd, kd, vd = dev(q, k, v)
    o, m = sb.sb_attn_fwd_train(qd, kd, vd)
    o2 = sb.sb_attn_fwd(qd, kd, vd)
    torch.cuda.synchronize()
    assert torch.equal(o, o2), "fwd and fwd_train must give the same o"
    ref, rem = oracle.fwd(to64(q), to64(k), to64(v), rows=rows)
    og, mg = to64(o), to64(m)
    if rows is not None:
        og, mg = og[..., rows[0]:rows[1], :], mg[..., rows[0]:rows[1]]
    assert np.all(np.isfinite(og))
    err = max_abs(og, ref)
    assert err <= tol, f"max abs err {err}"
    check_m(mg, rem)
    return err


# ------------------------------------------------------------------ fp32 path
def test_f32_workload_1(sb, oracle, gen):
    w = gen.WORKLOADS[0]
    q, k, v = gen.workload_tensors(w)
    qd, kd, vd = dev(q, k, v)
    o, m = sb.sb_attn_fwd_f32(qd, kd, vd, want_m=True)
    torch.cuda.synchronize()
    ref, rem = oracle.fwd(to64(q), to64(k), to64(v))
    assert max_abs(to64(o), ref) <= F32_TOL
    check_m(to64(m), rem, rtol=1e-5, atol=1e-5)
    assert not to64(o)[0, 0, 0].any()


@pytest.mark.parametrize("T", [1, 2, 31, 64, 65, 200, 257])
@pytest.mark.parametrize("d", [32, 64, 128])
def test_f32_shapes(sb, oracle, gen, T, d):
    q, k, v = gen.gaussian(2, 3, T, d, seed=100 + T, dtype="f32")
    qd, kd, vd = dev(q, k, v)
    o = sb.sb_attn_fwd_f32(qd, kd, vd)
    torch.cuda.synchronize()
    ref, _ = oracle.fwd(to64(q), to64(k), to64(v))
    assert max_abs(to64(o), ref) <= F32_TOL


def test_f32_long_range_and_sharp(sb, oracle, gen):
    for q, k, v in (gen.constant_logit(1, 2, 700, 64, 5, kval=-48.0, dtype="f32"),
                    gen.biased_gaussian(1, 2, 600, 64, 6, shift=-6.0, dtype="f32"),
                    gen.scaled_gaussian(1, 2, 300, 128, 7, gain=30.0, dtype="f32")):
        qd, kd, vd = dev(q, k, v)
        o, m = sb.sb_attn_fwd_f32(qd, kd, vd, want_m=True)
        torch.cuda.synchronize()
        ref, rem = oracle.fwd(to64(q), to64(k), to64(v))
        # long sums of softplus in fp32: allow the carry's rounding, 2^-24 * |sum| per step
        assert max_abs(to64(o), ref) <= 5e-5
        check_m(to64(m), rem, rtol=1e-5, atol=1e-5)


# ------------------------------------------------------------------ bf16 path
@pytest.mark.parametrize("T", [1, 2, 31, 32, 33, 64, 100, 127, 128, 129, 300, 517])
@pytest.mark.parametrize("d", [32, 64, 128])
def test_bf16_shapes(sb, oracle, gen, T, d):
    q, k, v = gen.gaussian(2, 3, T, d, seed=200 + T + d, dtype="bf16")
    run_bf16(sb, oracle, q, k, v)


@pytest.mark.parametrize("d", [32, 64, 128])
def test_bf16_first_row_is_zero_and_deterministic(sb, gen, d):
    q, k, v = dev(*gen.gaussian(3, 5, 333, d, seed=9, dtype="bf16"))
    o1, m1 = sb.sb_attn_fwd_train(q, k, v)
    o2, m2 = sb.sb_attn_fwd_train(q, k, v)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2) and torch.equal(m1, m2)
    assert not o1[:, :, 0].any() and not m1[:, :, 0].any()


@pytest.mark.parametrize("d", [32, 64, 128])
def test_bf16_constant_logit_long_range(sb, oracle, gen, d):
    """Small equal sigma everywhere: weights reach across many key tiles, so a
    wrong cross-tile carry cannot hide.  Closed form: A = b (1-b)^(j-i-1)."""
    T = 1100
    kval = {32: -34.0, 64: -48.0, 128: -64.0}[d]          # logit about -6
    q, k, v = gen.constant_logit(1, 2, T, d, seed=3, kval=kval, dtype="bf16")
    run_bf16(sb, oracle, q, k, v)
    # and directly against the closed form, independent of the oracle
    o = to64(sb.sb_attn_fwd(*dev(q, k, v)))
    b = 1.0 / (1.0 + math.exp(-kval / math.sqrt(d)))
    j, i = np.meshgrid(np.arange(T), np.arange(T), indexing="ij")
    A = np.where(i < j, b * (1.0 - b) ** np.clip(j - i - 1, 0, None), 0.0)
    assert max_abs(o[0, 0], A @ to64(v)[0, 0]) <= BF16_TOL


@pytest.mark.parametrize("d", [32, 64, 128])
def test_bf16_biased_long_range(sb, oracle, gen, d):
    q, k, v = gen.biased_gaussian(1, 3, 900, d, seed=4, shift=-6.0, dtype="bf16")
    run_bf16(sb, oracle, q, k, v)


@pytest.mark.parametrize("gain", [3.0, 30.0, 1000.0])
def test_bf16_sharp_logits(sb, oracle, gen, gain):
    """Near-saturated sigma: the stability path (no overflow, no NaN)."""
    q, k, v = gen.scaled_gaussian(1, 2, 400, 128, seed=5, gain=gain, dtype="bf16")
    run_bf16(sb, oracle, q, k, v)


def test_bf16_hugely_negative_logits_attend_to_nothing(sb, gen):
    q, k, v = gen.constant_logit(1, 1, 200, 64, seed=1, kval=-4096.0, dtype="bf16")
    o, m = sb.sb_attn_fwd_train(*dev(q, k, v))
    torch.cuda.synchronize()
    assert not o.any() and not m.any()


# ------------------------------------------------ the paper-shaped workloads
def test_workload_2_sampled_heads(sb, oracle, gen):
    w = gen.WORKLOADS[1]
    q, k, v = gen.workload_tensors(w)
    qd, kd, vd = dev(q, k, v)
    o, m = sb.sb_attn_fwd_train(qd, kd, vd)
    torch.cuda.synchronize()
    for b, h in gen.slice_picks(w, 4):
        ref, rem = oracle.fwd(to64(q[b, h]), to64(k[b, h]), to64(v[b, h]))
        assert max_abs(to64(o[b, h]), ref) <= BF16_TOL
        check_m(to64(m[b, h]), rem)


def test_workload_3_headline_sampled_heads(sb, oracle, gen):
    w = gen.WORKLOADS[2]
    q, k, v = gen.workload_tensors(w)
    qd, kd, vd = dev(q, k, v)
    o, m = sb.sb_attn_fwd_train(qd, kd, vd)
    torch.cuda.synchronize()
    picks = gen.slice_picks(w, 4)
    assert sum(h >= w.H // 2 for _, h in picks) >= 2          # sharp heads are covered
    for b, h in picks:
        ref, rem = oracle.fwd(to64(q[b, h]), to64(k[b, h]), to64(v[b, h]))
        assert max_abs(to64(o[b, h]), ref) <= BF16_TOL
        check_m(to64(m[b, h]), rem)
    # properties that hold at any size
    of = o.float()
    assert torch.isfinite(of).all() and not of[:, :, 0].any()
    assert (m <= 0).all()


def test_workload_5_long_context_tail_rows(sb, oracle, gen):
    w = gen.WORKLOADS[4]
    q, k, v = gen.workload_tensors(w)
    qd, kd, vd = dev(q, k, v)
    o = sb.sb_attn_fwd(qd, kd, vd)
    torch.cuda.synchronize()
    r0, r1 = w.T - 512, w.T
    for b, h in gen.slice_picks(w, 2):
        ref, _ = oracle.fwd(to64(q[b, h]), to64(k[b, h]), to64(v[b, h]), rows=(r0, r1))
        assert max_abs(to64(o[b, h, r0:r1]), ref) <= BF16_TOL


# ---------------------------------------------------------------- early halt (inference forward)
def test_very_long_sequence_sampled_rows(sb, oracle, gen):
    """T = 65536 (1024 key tiles per row block, 64-bit row offsets in play): rows the oracle computes
    one by one, at the start, in the middle and at the end, on long-range inputs so that the carry
    matters across thousands of keys."""
    T, d = 65536, 64
    q, k, v = gen.biased_gaussian(1, 2, T, d, seed=31, shift=-6.0, dtype="bf16")
    o, m = sb.sb_attn_fwd_train(*dev(q, k, v))
    torch.cuda.synchronize()
    for r0 in (0, 32760, T - 64):
        ref, rem = oracle.fwd(to64(q), to64(k), to64(v), rows=(r0, r0 + 64))
        assert max_abs(to64(o[:, :, r0:r0 + 64]), ref) <= BF16_TOL
        check_m(to64(m[:, :, r0:r0 + 64]), rem)


def test_halt_matches_oracle_and_skips_tiles(sb, oracle, gen):
    """N(0,1) logits use up the stick within a few dozen keys: almost every tile beyond the
    diagonal band is skipped, and the output still matches the oracle."""
    q, k, v = gen.gaussian(1, 3, 2048, 128, seed=31, dtype="bf16")
    qd, kd, vd = dev(q, k, v)
    counts = torch.zeros(2, dtype=torch.int64, device="cuda")
    o = sb.sb_attn_fwd_halt(qd, kd, vd, 1e-9, tile_counts=counts)
    torch.cuda.synchronize()
    ref, _ = oracle.fwd(to64(q), to64(k), to64(v))
    assert max_abs(to64(o), ref) <= BF16_TOL
    swept, full = counts.cpu().tolist()
    print(f"tiles swept {swept} of {full}")
    assert 0 < swept < 0.35 * full


@pytest.mark.parametrize("d", [32, 64, 128])
def test_halt_never_triggers_on_slowly_decaying_weights(sb, gen, d):
    """Constant small logit: the stick is far from used up at T = 700, nothing may be skipped
    and the result is bit-identical to the plain forward."""
    kval = {32: -34.0, 64: -48.0, 128: -64.0}[d]          # logit about -6
    q, k, v = dev(*gen.constant_logit(1, 2, 700, d, seed=32, kval=kval, dtype="bf16"))
    counts = torch.zeros(2, dtype=torch.int64, device="cuda")
    o1 = sb.sb_attn_fwd(q, k, v)
    o2 = sb.sb_attn_fwd_halt(q, k, v, 1e-6, tile_counts=counts)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2)
    swept, full = counts.cpu().tolist()
    assert swept == full > 0


def test_halt_error_is_bounded_by_eps(sb, gen):
    """Logits around -3: weights spread over ~100 keys.  With a coarse eps the halted result
    differs from the full sweep by at most eps * max|v| (plus one bf16 rounding of o)."""
    q, k, v = dev(*gen.biased_gaussian(1, 2, 1500, 128, seed=33, shift=-3.0, dtype="bf16"))
    eps = 1e-2
    counts = torch.zeros(2, dtype=torch.int64, device="cuda")
    o_full = sb.sb_attn_fwd(q, k, v).float()
    o_halt = sb.sb_attn_fwd_halt(q, k, v, eps, tile_counts=counts).float()
    torch.cuda.synchronize()
    bound = eps * float(v.float().abs().max()) + 2.0 ** -7 * float(o_full.abs().max())
    diff = float((o_full - o_halt).abs().max())
    swept, full = counts.cpu().tolist()
    print(f"max diff {diff:.3e} bound {bound:.3e}, tiles swept {swept} of {full}")
    assert diff <= bound and swept < full


def test_halt_rejects_bad_eps(sb, gen):
    q, k, v = dev(*gen.gaussian(1, 1, 64, 64, seed=34, dtype="bf16"))
    for eps in (0.0, 1.0, -1.0, float("nan")):
        with pytest.raises(sb.SbAttnError):
            sb.sb_attn_fwd_halt(q, k, v, eps)


@pytest.mark.parametrize("kind", ["gaussian", "long_range", "sharp"])
def test_triangular_mfma_cumsum_variant(sb, oracle, gen, kind):
    """The measurement variant of the forward (in-tile cumulative sum as a product with a
    triangular matrix of ones on the matrix pipe, log form of Eq. 2) meets the same bound as the
    product path; T spans the diagonal band and many unmasked tiles."""
    if kind == "gaussian":
        q, k, v = gen.gaussian(2, 4, 1000, 128, seed=41, dtype="bf16", sharp_half=True)
    elif kind == "long_range":
        q, k, v = gen.biased_gaussian(1, 2, 1300, 128, seed=42, shift=-6.0)
    else:
        q, k, v = gen.scaled_gaussian(1, 2, 700, 128, seed=43, gain=30.0)
    qd, kd, vd = dev(q, k, v)
    o, m = sb.sb_diag_fwd_tri(qd, kd, vd)
    torch.cuda.synchronize()
    ref, rem = oracle.fwd(to64(q), to64(k), to64(v))
    err = max_abs(to64(o), ref)
    print(f"triangular-MFMA variant, {kind}: max abs err {err:.3e}")
    assert err <= BF16_TOL
    check_m(to64(m), rem)


def test_clock_sampling_forward_is_the_training_forward(sb, gen):
    """The forward that samples the shader clock (measurement aid) writes what
    sb_attn_fwd_train writes, bit for bit, and reports a plausible clock."""
    q, k, v = gen.gaussian(2, 4, 1100, 128, seed=44, dtype="bf16", sharp_half=True)
    qd, kd, vd = dev(q, k, v)
    o, m = sb.sb_attn_fwd_train(qd, kd, vd)
    o2, m2 = torch.full_like(o, 7.0), torch.full_like(m, 7.0)
    mhz = sb.sb_diag_fwd_clock(qd, kd, vd, o2, m2)
    torch.cuda.synchronize()
    assert torch.equal(o.view(torch.int16), o2.view(torch.int16))
    assert torch.equal(m.view(torch.int32), m2.view(torch.int32))
    assert 300.0 < mhz < 3000.0


def test_streaming_read_diagnostic_runs(sb):
    """The read-only streaming kernel (the decode path's practical ceiling) reports a rate
    between what a single HBM stack and the whole chip can deliver."""
    x = torch.randn(1 << 26, device="cuda")          # 256 MiB
    gbs = sb.sb_diag_stream_read(x, iters=5)
    print(f"streaming read: {gbs:.0f} GB/s")
    assert 500.0 < gbs < 8500.0
