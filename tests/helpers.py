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
