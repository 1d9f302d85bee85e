"""GPU parity: the HIP backward (through the C ABI) against the CPU float64
oracle's analytic gradients (themselves pinned by finite differences) on the
same seeded, already-rounded bf16 inputs.

Tolerance on each of dq, dk, dv (helpers.check_grad): the flat 2e-2 max abs error of
the forward wherever the tensor's largest entry is at most 5.12; beyond that, max abs
error / max|ref| <= 2^-8, one bf16 rounding step of the largest entry (the weights A and
the logit gradients dZ enter the matrix cores rounded to bf16, so every gradient entry
carries a relative error of that order whatever its size).  The ratio is printed for
every tensor.
"""
import numpy as np
import pytest
import torch

from helpers import check_grad, dev, nan_bytes, to64

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


def gpu_grads(sb, q, k, v, g):
    qd, kd, vd, gd = dev(q, k, v, g)
    o, m = sb.sb_attn_fwd_train(qd, kd, vd)
    ws = nan_bytes(sb.sb_attn_bwd_workspace_bytes(*q.shape))
    dq, dk, dv = sb.sb_attn_bwd(qd, kd, vd, m, gd, workspace=ws)
    torch.cuda.synchronize()
    return to64(dq), to64(dk), to64(dv)


def check(sb, oracle, q, k, v, g):
    dq, dk, dv = gpu_grads(sb, q, k, v, g)
    rq, rk, rv = oracle.bwd(to64(q), to64(k), to64(v), to64(g))
    return {name: check_grad(name, a, r) for name, a, r in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv))}


@pytest.mark.parametrize("T", [1, 2, 32, 33, 64, 65, 100, 129, 257, 300])
@pytest.mark.parametrize("d", [32, 64, 128])
def test_bwd_shapes(sb, oracle, gen, T, d):
    q, k, v, g = gen.gaussian(2, 3, T, d, seed=300 + T + d, dtype="bf16", with_dout=True)
    check(sb, oracle, q, k, v, g)


@pytest.mark.parametrize("T", [319, 320, 321, 383, 384, 385, 447, 448, 449, 511, 512, 513, 577, 640, 705])
def test_bwd_steady_state_loop_boundaries(sb, oracle, gen, T):
    """d = 128: lengths around the points where a key block's sweep gains its first steady-state
    interval, where the last tile is complete, ragged by one row, or short by one row, and where
    the tile after the steady state is the ragged one (the key-stationary pass stages that tile
    from inside the steady-state loop only when it is complete)."""
    q, k, v, g = gen.gaussian(1, 2, T, 128, seed=900 + T, dtype="bf16", with_dout=True)
    check(sb, oracle, q, k, v, g)


@pytest.mark.parametrize("d", [32, 64, 128])
def test_bwd_finite_differences_T32(sb, oracle, gen, d):
    """Directional finite differences of the float64 forward at T = 32 against
    the GPU gradients (independent of the oracle's own backward)."""
    q, k, v, g = gen.gaussian(1, 1, 32, d, seed=77, dtype="bf16", with_dout=True)
    dq, dk, dv = gpu_grads(sb, q, k, v, g)
    q64, k64, v64, g64 = (to64(t)[0, 0] for t in (q, k, v, g))
    loss = lambda a, b, c: float((oracle.fwd(a, b, c)[0] * g64).sum())
    rng = np.random.default_rng(0)
    h = 1e-5
    for _ in range(6):
        uq, uk, uv = (rng.standard_normal(q64.shape) for _ in range(3))
        fd = (loss(q64 + h * uq, k64 + h * uk, v64 + h * uv) -
              loss(q64 - h * uq, k64 - h * uk, v64 - h * uv)) / (2 * h)
        an = float((dq[0, 0] * uq).sum() + (dk[0, 0] * uk).sum() + (dv[0, 0] * uv).sum())
        norm = np.sqrt((dq ** 2).sum() + (dk ** 2).sum() + (dv ** 2).sum()) * np.sqrt(3 * q64.size)
        assert abs(fd - an) <= 2e-3 * norm + 1e-3, (fd, an)


@pytest.mark.parametrize("d", [32, 64, 128])
def test_bwd_long_range(sb, oracle, gen, d):
    """Slowly decaying weights: the carries a and b cross many key tiles."""
    kval = {32: -34.0, 64: -48.0, 128: -64.0}[d]          # logit about -6
    q, k, v, g = gen.constant_logit(1, 2, 700, d, seed=13, kval=kval, dtype="bf16", with_dout=True)
    check(sb, oracle, q, k, v, g)
    q, k, v, g = gen.biased_gaussian(1, 2, 700, d, seed=14, shift=-6.0, dtype="bf16", with_dout=True)
    check(sb, oracle, q, k, v, g)


@pytest.mark.parametrize("gain", [3.0, 30.0])
def test_bwd_sharp_logits(sb, oracle, gen, gain):
    q, k, v, g = gen.scaled_gaussian(1, 2, 300, 128, seed=15, gain=gain, dtype="bf16", with_dout=True)
    check(sb, oracle, q, k, v, g)


def test_bwd_twice_agrees_and_overwrites(sb, gen):
    q, k, v, g = dev(*gen.gaussian(2, 4, 257, 128, seed=16, dtype="bf16", with_dout=True))
    o, m = sb.sb_attn_fwd_train(q, k, v)
    junk = lambda: torch.full(q.shape, 123.0, dtype=torch.float32, device="cuda")
    dq1, dk1, dv1 = sb.sb_attn_bwd(q, k, v, m, g, junk(), junk(), junk())
    dq2, dk2, dv2 = sb.sb_attn_bwd(q, k, v, m, g, junk(), junk(), junk())
    torch.cuda.synchronize()
    # no atomics anywhere: bit-reproducible
    assert torch.equal(dq1, dq2) and torch.equal(dk1, dk2) and torch.equal(dv1, dv2)
    assert not dk1[:, :, -1].any() and not dv1[:, :, -1].any()   # last key: no later query
    assert not dq1[:, :, 0].any()                                 # first query: no earlier key


@pytest.mark.parametrize("d", [64, 128])
def test_bwd_is_bit_reproducible_on_a_full_chip(sb, gen, d):
    """Enough workgroups to fill every CU several times over: a race in the LDS hand-over between
    the waves of a workgroup would show as run-to-run differences."""
    B, H, T = 4, 16, 2048
    q, k, v, g = dev(*gen.gaussian(B, H, T, d, seed=17, dtype="bf16", sharp_half=True, with_dout=True))
    o, m = sb.sb_attn_fwd_train(q, k, v)
    ws = nan_bytes(sb.sb_attn_bwd_workspace_bytes(B, H, T, d))
    ref = [t.clone() for t in sb.sb_attn_bwd(q, k, v, m, g, workspace=ws)]
    for rep in range(3):
        ws.fill_(0xFF)
        out = sb.sb_attn_bwd(q, k, v, m, g, workspace=ws)
        torch.cuda.synchronize()
        for name, a, b in zip(("dq", "dk", "dv"), out, ref):
            assert torch.equal(a, b), f"run {rep}: {name} differs"
    assert all(torch.isfinite(t).all() for t in ref)


def test_workload_4_sampled_heads(sb, oracle, gen):
    w = gen.WORKLOADS[3]
    q, k, v, g = gen.workload_tensors(w)
    qd, kd, vd, gd = dev(q, k, v, g)
    o, m = sb.sb_attn_fwd_train(qd, kd, vd)
    dq, dk, dv = sb.sb_attn_bwd(qd, kd, vd, m, gd)
    torch.cuda.synchronize()
    for b, h in gen.slice_picks(w, 4):
        rq, rk, rv = oracle.bwd(to64(q[b, h]), to64(k[b, h]), to64(v[b, h]), to64(g[b, h]))
        for name, a, r in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
            check_grad(f"{name}[{b},{h}]", to64(a[b, h]), r)
    assert torch.isfinite(dq).all() and torch.isfinite(dk).all() and torch.isfinite(dv).all()


def test_headline_shape_step_sampled_heads(sb, oracle, gen):
    """The benchmark's step (training forward + backward at B8 H16 T4096 d128, half the heads
    with k*3, same buffers and launch configuration) on heads the oracle computes one by one,
    two of them sharp; every gradient finite everywhere."""
    w = gen.WORKLOADS[2]
    q, k, v, g = gen.gaussian(w.B, w.H, w.T, w.d, w.seed, w.dtype, w.sharp_half, with_dout=True)
    qd, kd, vd, gd = dev(q, k, v, g)
    ws = torch.empty(sb.sb_attn_bwd_workspace_bytes(w.B, w.H, w.T, w.d), dtype=torch.uint8, device="cuda")
    o, m = sb.sb_attn_fwd_train(qd, kd, vd)
    dq, dk, dv = sb.sb_attn_bwd(qd, kd, vd, m, gd, workspace=ws)
    torch.cuda.synchronize()
    picks = gen.slice_picks(w, 4)
    assert sum(h >= w.H // 2 for _, h in picks) == 2
    for b, h in picks:
        rq, rk, rv = oracle.bwd(to64(q[b, h]), to64(k[b, h]), to64(v[b, h]), to64(g[b, h]))
        for name, a, r in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
            check_grad(f"{name}[{b},{h}]", to64(a[b, h]), r)
    assert torch.isfinite(dq).all() and torch.isfinite(dk).all() and torch.isfinite(dv).all()


def test_long_context_backward_one_head(sb, oracle, gen):
    """T = 8192: many tiles per block and 64 blocks per head; one (b, h) slice against the oracle
    (which needs 16 T^2 bytes = 1 GiB of host scratch for it)."""
    B, H, T, d = 1, 8, 8192, 128
    q, k, v, g = gen.gaussian(B, H, T, d, seed=23, dtype="bf16", sharp_half=True, with_dout=True)
    qd, kd, vd, gd = dev(q, k, v, g)
    o, m = sb.sb_attn_fwd_train(qd, kd, vd)
    dq, dk, dv = sb.sb_attn_bwd(qd, kd, vd, m, gd, workspace=nan_bytes(sb.sb_attn_bwd_workspace_bytes(B, H, T, d)))
    torch.cuda.synchronize()
    assert torch.isfinite(dq).all() and torch.isfinite(dk).all() and torch.isfinite(dv).all()
    for h in (1, 6):                                   # a plain and a sharp head
        rq, rk, rv = oracle.bwd(to64(q[0, h]), to64(k[0, h]), to64(v[0, h]), to64(g[0, h]))
        for name, a, r in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
            check_grad(f"{name}[0,{h}]", to64(a[0, h]), r)


@pytest.mark.parametrize("d", [64, 128])
def test_bwd_log_domain_redo_of_every_block(sb, oracle, gen, d):
    """Sharp logits in every head of a batch that fills the chip: the fast kernels flag (nearly)
    every block and the log-domain launches redo them all (384 block pairs per pass); heads at
    both ends of the grid against the oracle, everything finite."""
    B, H, T = 4, 16, 1536
    q, k, v, g = gen.scaled_gaussian(B, H, T, d, seed=31, gain=30.0, dtype="bf16", with_dout=True)
    qd, kd, vd, gd = dev(q, k, v, g)
    o, m = sb.sb_attn_fwd_train(qd, kd, vd)
    dq, dk, dv = sb.sb_attn_bwd(qd, kd, vd, m, gd, workspace=nan_bytes(sb.sb_attn_bwd_workspace_bytes(B, H, T, d)))
    torch.cuda.synchronize()
    assert torch.isfinite(dq).all() and torch.isfinite(dk).all() and torch.isfinite(dv).all()
    for b, h in ((0, 0), (2, 7), (3, 15)):
        rq, rk, rv = oracle.bwd(to64(q[b, h]), to64(k[b, h]), to64(v[b, h]), to64(g[b, h]))
        for name, a, r in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
            check_grad(f"{name}[{b},{h}]", to64(a[b, h]), r)


def test_bwd_split_passes_equal_the_whole(sb, gen):
    """sb_attn_bwd_dq followed by sb_attn_bwd_dkdv on one workspace is sb_attn_bwd, bit for bit."""
    q, k, v, g = dev(*gen.gaussian(2, 3, 333, 128, seed=21, dtype="bf16", with_dout=True))
    o, m = sb.sb_attn_fwd_train(q, k, v)
    dq, dk, dv = sb.sb_attn_bwd(q, k, v, m, g)
    dq2, ws = sb.sb_attn_bwd_dq(q, k, v, m, g)
    dk2, dv2 = sb.sb_attn_bwd_dkdv(q, k, v, g, ws)
    torch.cuda.synchronize()
    assert torch.equal(dq, dq2) and torch.equal(dk, dk2) and torch.equal(dv, dv2)


def test_bwd_sharp_blocks_are_redone_only_where_needed(sb, oracle, gen):
    """One head with logits far beyond the linear-domain range next to an ordinary one:
    the flagged blocks go through the log-domain variant, the rest do not, and both match."""
    q, k, v, g = gen.gaussian(1, 2, 400, 128, seed=22, dtype="bf16", with_dout=True)
    k[:, 1] = (k[:, 1].float() * 40.0).to(k.dtype)
    check(sb, oracle, q, k, v, g)


def test_mfma_rate_diagnostic_runs(sb):
    x = torch.randn(1 << 20, device="cuda").to(torch.bfloat16)
    tf, mhz = sb.sb_diag_mfma_rate(x, iters=200)
    assert 100.0 < tf < 2600.0 and 500.0 < mhz < 2600.0
