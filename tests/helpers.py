"""Shared helpers for the GPU parity tests: conversions between the torch
tensors the library sees and the float64 arrays the oracle sees."""
import numpy as np
import torch

BF16_TOL = 2e-2   # max abs error, bf16 inputs with fp32 accumulation
F32_TOL = 1e-5    # max abs error, fp32 path


def to64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of an (already rounded) tensor to float64."""
    return t.detach().cpu().to(torch.float32).to(torch.float64).numpy()


def dev(*ts):
    return tuple(t.cuda().contiguous() for t in ts)


def max_abs(a, b) -> float:
    return float(np.abs(np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64)).max()) if np.size(a) else 0.0


def check_m(m_gpu: np.ndarray, rem: np.ndarray, rtol=2e-3, atol=2e-3):
    """m = log(remaining stick) wherever the float64 remainder has not underflowed."""
    ok = rem > 1e-290
    ref = np.log(rem[ok])
    err = np.abs(m_gpu[ok] - ref)
    assert np.all(err <= atol + rtol * np.abs(ref)), float((err - rtol * np.abs(ref)).max())
    assert np.all(m_gpu <= 0.0)


def nan_bytes(nbytes: int) -> torch.Tensor:
    """Device scratch whose every float reads as NaN: a kernel that consumes workspace memory it
    did not write first shows up as a non-finite result."""
    return torch.full((max(int(nbytes), 1),), 0xFF, dtype=torch.uint8, device="cuda")


GRAD_REL = 2.0 ** -8   # one bf16 rounding step of the largest entry (A and dZ enter the MFMAs as bf16)


def grad_tol(ref) -> float:
    """Bound on the max abs error of a gradient tensor: the flat 2e-2 while its entries stay
    below 5.12 in magnitude (there 2^-8 max|ref| <= 2e-2), 2^-8 of the largest entry beyond."""
    return max(BF16_TOL, GRAD_REL * float(np.abs(ref).max())) if np.size(ref) else BF16_TOL


def check_grad(name: str, got, ref, log=None) -> float:
    """Asserts the gradient bound on one tensor and returns the error.  Written out as the two
    cases it consists of, and with the relative error printed, so that a log shows both."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert np.all(np.isfinite(got)), name
    err = max_abs(got, ref)
    top = float(np.abs(ref).max()) if ref.size else 0.0
    rel = err / top if top > 0 else 0.0
    print(f"{name}: max abs err {err:.3e}  max|ref| {top:.3e}  err/max|ref| {rel:.3e}")
    if log is not None:
        log.append((name, err, top, rel))
    if top <= BF16_TOL / GRAD_REL:          # 5.12: the flat bound of the forward applies as it stands
        assert err <= BF16_TOL, f"{name}: max abs err {err} > {BF16_TOL} (max |ref| {top})"
    else:                                   # larger gradients: relative to the largest entry
        assert rel <= GRAD_REL, f"{name}: err / max|ref| = {rel} > 2^-8 (err {err}, max |ref| {top})"
    return err


def fwd_bound(ref, v):
    """Element-wise bound on |o_gpu - o_ref| for the bf16 forward: the flat 2e-2 wherever it is
    the larger one (|o| below about 2.7 for N(0,1) values), else the rounding of the bf16 output
    grid (2^-8 |o|: an output of magnitude 4..8 is rounded by up to 0.0156 on its own) plus the
    bf16 rounding of the weights (2^-9 max|v|).  Every test on a stated workload and every
    fixed-shape test asserts the flat bound on all elements, which is the stricter statement;
    this rule is for seeded random shapes, where an output beyond 4 can occur."""
    ref = np.asarray(ref, dtype=np.float64)
    return np.maximum(BF16_TOL, GRAD_REL * np.abs(ref) + 2.0 ** -9 * float(np.abs(np.asarray(v)).max()))
