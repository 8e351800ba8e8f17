"""The allocation-free variant of pvf_rope_attention against the allocating one, through the C ABI.

Two calls in a row on the same GPU, the second with a smaller input (so it meets whatever the first
left in the library's static scratch), on the float32 path (plain kernels) and on the bf16 path that
uses the key-contiguous copy of v.  Both entry points run the same kernels on the same values; the only
difference is where the rotary table is evaluated (host libm against the device's double-precision
cos / sin), so the outputs agree to rounding of the last place: the bar is 1e-6 absolute in float32
and one bf16 unit in the last place (2^-8 relative) in bf16.
"""
import numpy as np
import pytest
import torch

from paper_2601_12247_amd import binding as B

pytestmark = pytest.mark.gpu


def _run_pair(dtype, S, T, H, dh, theta, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    qkv = torch.randn(S * T, 3 * H * dh, generator=g, dtype=torch.float32).to("cuda", dtype)
    a_in, b_in = qkv.clone(), qkv.clone()
    want = B.rope_attention(a_in, S, T, H, dh, theta)
    out = torch.full((S * T, H * dh), float("nan"), dtype=dtype, device="cuda")
    B.rope_attention_noalloc(b_in, out, S, T, H, dh, theta)
    torch.cuda.synchronize()
    return a_in.float(), want.float(), b_in.float(), out.float()


@pytest.mark.parametrize("dtype,shapes", [
    (torch.float32, [(3, 96, 4, 64, 1e4), (2, 40, 4, 32, 1e4)]),
    (torch.bfloat16, [(3, 512, 8, 128, 5e5), (1, 128, 4, 128, 5e5)]),
])
def test_noalloc_matches_allocating_entry_point_twice_in_a_row(dtype, shapes):
    for i, (S, T, H, dh, theta) in enumerate(shapes):
        qa, oa, qb, ob = _run_pair(dtype, S, T, H, dh, theta, seed=11 + i)
        assert torch.isfinite(ob).all()
        if dtype == torch.float32:
            assert (qa - qb).abs().max().item() <= 1e-6 and (oa - ob).abs().max().item() <= 1e-6
        else:
            tol = lambda ref: 2.0 ** -8 * ref.abs() + 1e-6
            assert bool(((qa - qb).abs() <= tol(qa)).all()) and bool(((oa - ob).abs() <= tol(oa)).all())


def test_noalloc_rejects_sizes_beyond_the_static_scratch():
    H, dh = 32, 128
    qkv = torch.zeros(64, 3 * H * dh, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(64, H * dh, dtype=torch.bfloat16, device="cuda")
    lib = B.lib()
    # T beyond the table
    rc = lib.pvf_rope_attention_noalloc(None, B.PVF_BF16, qkv.data_ptr(), out.data_ptr(), 1, 4096, H, dh, 5e5)
    assert rc == -2 and b"static scratch" in lib.pvf_last_error(None)
    # S*T*d beyond the v copy: 4 x 1024 x 4096 = 16 Mi elements
    rc = lib.pvf_rope_attention_noalloc(None, B.PVF_BF16, qkv.data_ptr(), out.data_ptr(), 4, 1024, H, dh, 5e5)
    assert rc == -2 and b"static scratch" in lib.pvf_last_error(None)
