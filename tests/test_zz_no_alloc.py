"""The decode entry point that allocates nothing (its chunk partials live in a static device
array of the library) against the workspace-taking entry point, through the C ABI: same
kernels, same chunking, so the outputs must be bit-identical.  Two calls in a row, the second
on a smaller input, so that what the first call left in the shared scratch would show."""
import ctypes

import pytest
import torch

from helpers import dev, nan_bytes

pytestmark = pytest.mark.gpu

STATIC_BYTES = 32 << 20


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


def case(gen, B, H, Hkv, T, d, seed):
    q, _, _ = gen.gaussian(B, H, 1, d, seed=seed)
    _, k, v = gen.gaussian(B, Hkv, T, d, seed=seed + 1)
    return dev(q[:, :, 0].contiguous(), k, v)


def both(sb, q, k, v, T=None, r=None):
    B, H, d = q.shape
    Tv = k.shape[2] if T is None else T
    ws = nan_bytes(sb.load().sb_attn_decode_workspace_bytes(B, H, Tv, d))
    o_ref, m_ref = sb.sb_attn_decode(q, k, v, T=T, r=r, want_m=True, workspace=ws)
    o = torch.full_like(q, float("nan"))
    m = torch.full((B, H), float("nan"), dtype=torch.float32, device="cuda")
    sb.sb_attn_decode_static(q, k, v, o, T=T, r=r, m=m)
    torch.cuda.synchronize()
    assert torch.equal(o.view(torch.int16), o_ref.view(torch.int16))
    assert torch.equal(m.view(torch.int32), m_ref.view(torch.int32))


def test_two_calls_in_a_row_second_smaller(sb, gen):
    r = gen.remainder_embedding(8, 128, seed=5).cuda()
    both(sb, *case(gen, 2, 8, 2, 5000, 128, seed=21), r=r)     # 79 chunks per head, grouped heads
    both(sb, *case(gen, 1, 3, 3, 300, 64, seed=22))            # 5 chunks per head: stale partials beyond
    both(sb, *case(gen, 2, 8, 2, 5000, 128, seed=23), T=1)     # one key, one chunk


def test_rejects_sizes_beyond_the_static_scratch(sb):
    lib = sb.load()
    p = ctypes.c_void_p(4096)                                  # never dereferenced: validation fails first
    B, H, T, d = 8, 64, 16384, 128
    assert lib.sb_attn_decode_workspace_bytes(B, H, T, d) > STATIC_BYTES
    assert lib.sb_attn_decode_static(p, p, p, None, p, None, B, H, H, T, T, d, None) == -6
    assert lib.sb_attn_decode_static(p, p, p, None, None, None, 1, 1, 1, 8, 8, 64, None) == -1
    assert lib.sb_attn_decode_static(p, p, p, None, p, None, 1, 1, 1, 8, 4, 64, None) == -2
