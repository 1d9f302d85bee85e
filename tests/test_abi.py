"""The C-ABI library loads and exports every symbol the public header declares;
argument validation returns error codes without touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = []
    for header in ("sb_attn.h", "sb_diag.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b(sb_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


@pytest.fixture(scope="module")
def lib():
    from paper_2410_17980_amd import binding
    return binding.load()


def test_header_declares_the_expected_entry_points():
    names = declared_functions()
    for n in ("sb_attn_fwd", "sb_attn_fwd_train", "sb_attn_fwd_f32", "sb_attn_bwd",
              "sb_attn_bwd_workspace_bytes", "sb_status_string", "sb_version"):
        assert n in names


def test_every_declared_symbol_is_exported(lib):
    from paper_2410_17980_amd import binding
    for n in declared_functions():
        assert hasattr(lib, n), n
    assert set(binding.EXPORTS) == set(declared_functions())


def test_version_and_status_strings(lib):
    from paper_2410_17980_amd import binding
    assert binding.sb_version() >= 100
    assert binding.sb_status_string(0) == "ok"
    seen = {binding.sb_status_string(c) for c in range(-6, 1)}
    assert len(seen) == 7
    assert binding.sb_status_string(-99) == "unknown status"


def test_argument_validation_without_a_gpu(lib):
    p = ctypes.c_void_p(4096)          # never dereferenced: validation fails first
    odd = ctypes.c_void_p(4096 + 8)
    assert lib.sb_attn_fwd(None, p, p, p, 1, 1, 8, 64, None) == -1
    assert lib.sb_attn_fwd(p, p, p, None, 1, 1, 8, 64, None) == -1
    assert lib.sb_attn_fwd(p, p, p, p, 0, 1, 8, 64, None) == -2
    assert lib.sb_attn_fwd(p, p, p, p, 1, 1, 0, 64, None) == -2
    assert lib.sb_attn_fwd(p, p, p, p, 1, 1, 8, 96, None) == -3
    assert lib.sb_attn_fwd(p, odd, p, p, 1, 1, 8, 64, None) == -4
    assert lib.sb_attn_fwd(p, p, p, p, 1 << 20, 1 << 10, 1 << 12, 128, None) == -2
    assert lib.sb_attn_fwd_train(p, p, p, p, None, 1, 1, 8, 64, None) == -1
    assert lib.sb_attn_fwd_f32(p, p, None, p, None, 1, 1, 8, 64, None) == -1
    assert lib.sb_attn_fwd_f32(p, p, p, p, odd, 1, 1, 8, 64, None) == -4
    assert lib.sb_attn_bwd(p, p, p, None, p, p, p, p, None, 0, 1, 1, 8, 64, None) == -1
    assert lib.sb_attn_bwd(p, p, p, p, p, p, p, p, None, 0, 1, 1, 8, 48, None) == -3
    # remainder bias: r and dr are required
    assert lib.sb_attn_fwd_rb(p, p, p, None, p, None, 1, 1, 8, 64, None) == -1
    assert lib.sb_attn_fwd_rb(p, p, p, odd, p, None, 1, 1, 8, 64, None) == -4
    assert lib.sb_attn_bwd_rb(p, p, p, None, p, p, p, p, p, p, p, 1 << 20, 1, 1, 8, 64, None) == -1
    assert lib.sb_attn_bwd_rb(p, p, p, p, p, p, p, p, p, None, p, 1 << 20, 1, 1, 8, 64, None) == -1
    assert lib.sb_attn_bwd_rb(p, p, p, p, p, p, p, p, p, p, None, 0, 1, 1, 8, 64, None) == -6
    # grouped kv heads: H must be a multiple of Hkv
    assert lib.sb_attn_fwd_gqa(p, p, p, None, p, None, 1, 4, 3, 8, 64, None) == -2
    assert lib.sb_attn_fwd_gqa(p, p, p, None, p, None, 1, 4, 0, 8, 64, None) == -2
    assert lib.sb_attn_bwd_gqa(p, p, p, None, p, p, p, p, p, None, p, 1 << 20, 1, 4, 3, 8, 64, None) == -2
    assert lib.sb_attn_bwd_gqa(p, p, p, p, p, p, p, p, p, None, p, 1 << 20, 1, 4, 2, 8, 64, None) == -1
    # packed batches: offsets required, 1 <= max_T <= Ttot
    assert lib.sb_attn_varlen_fwd(p, p, p, None, p, None, None, 2, 2, 2, 100, 60, 64, None) == -1
    assert lib.sb_attn_varlen_fwd(p, p, p, None, p, None, p, 2, 2, 2, 100, 0, 64, None) == -2
    assert lib.sb_attn_varlen_fwd(p, p, p, None, p, None, p, 2, 2, 2, 100, 101, 64, None) == -2
    assert lib.sb_attn_varlen_fwd(p, p, p, None, p, None, p, 0, 2, 2, 100, 60, 64, None) == -2
    assert lib.sb_attn_varlen_fwd(p, p, p, None, p, None, p, 2, 3, 2, 100, 60, 64, None) == -2
    assert lib.sb_attn_varlen_fwd(p, p, p, None, p, None, p, 2, 2, 2, 100, 60, 80, None) == -3
    need_v = lib.sb_attn_varlen_bwd_workspace_bytes(3, 2, 100, 60, 64)
    assert need_v == 8 * 2 * 100 * 2 + 3 * 2 * (8 + 4 * 64) * 1
    assert lib.sb_attn_varlen_bwd_workspace_bytes(3, 2, 100, 101, 64) == 0
    assert lib.sb_attn_varlen_bwd(p, p, p, None, p, p, p, p, p, None, p, 3, 2, 2, 100, 60, 64, p, need_v - 1, None) == -6
    assert lib.sb_attn_varlen_bwd(p, p, p, None, None, p, p, p, p, None, p, 3, 2, 2, 100, 60, 64, p, need_v, None) == -1
    # decode: 1 <= T <= Tcap, T within the split's reach
    need_d = lib.sb_attn_decode_workspace_bytes(2, 4, 1000, 128)
    assert 0 < need_d <= 4 * 2 * 4 * 256 * 129
    assert lib.sb_attn_decode_workspace_bytes(2, 4, 0, 128) == 0
    assert lib.sb_attn_decode(p, p, p, None, p, None, p, need_d, 2, 4, 2, 1000, 999, 128, None) == -2
    assert lib.sb_attn_decode(p, p, p, None, p, None, p, need_d, 2, 4, 3, 1000, 1000, 128, None) == -2
    assert lib.sb_attn_decode(p, p, p, None, p, None, p, need_d, 2, 4, 2, 1 << 20, 1 << 20, 128, None) == -2
    assert lib.sb_attn_decode(p, p, p, None, p, None, None, 0, 2, 4, 2, 1000, 1000, 128, None) == -6
    assert lib.sb_attn_decode(p, p, p, None, p, None, p, need_d - 1, 2, 4, 2, 1000, 1000, 128, None) == -6
    assert lib.sb_attn_decode(None, p, p, None, p, None, p, need_d, 2, 4, 2, 1000, 1000, 128, None) == -1
    # workspace: size query, then missing / too small / misaligned workspace
    need = lib.sb_attn_bwd_workspace_bytes(2, 3, 100, 64)
    # two floats per (row, 32-key strip), one int per 128-row query block and key block,
    # d floats per 128-row block
    assert need == 2 * 3 * (8 * 100 * 4 + 4 * (1 + 1) + 4 * 64 * 1)
    assert lib.sb_attn_bwd_workspace_bytes(2, 3, 100, 65) == 0
    assert lib.sb_attn_bwd(p, p, p, p, p, p, p, p, None, 0, 2, 3, 100, 64, None) == -6
    assert lib.sb_attn_bwd(p, p, p, p, p, p, p, p, p, need - 1, 2, 3, 100, 64, None) == -6
    assert lib.sb_attn_bwd(p, p, p, p, p, p, p, p, odd, need, 2, 3, 100, 64, None) == -4


def test_binding_fails_loudly_on_cpu_tensors():
    import torch
    from paper_2410_17980_amd import binding
    x = torch.zeros(1, 1, 4, 64, dtype=torch.bfloat16)
    with pytest.raises(binding.SbAttnError):
        binding.sb_attn_fwd(x, x, x, x)
