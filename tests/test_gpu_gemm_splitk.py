"""The split-K GEMMs a context launches for few rows (window forward of a K/V-cached round: 64 rows per live
canvas; full forward of one short canvas), through pvf_ctx_gemm / pvf_ctx_gemm_swiglu, against float64
products of the same bf16 inputs: every output element, every epilogue, at the layer shapes of the 8B model
and at ragged row counts; launches repeated back to back and compared bit for bit (the partial tiles are
added in split order)."""
import numpy as np
import pytest
import torch

from paper_2601_12247_amd import binding as B
from synth import inputs as S
from tests.gpu_util import make_context, to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    shape = S.ModelShape(n_layers=1, d_model=256, n_heads=2, d_ff=512, vocab=512, mask_id=511)
    w = S.make_weights(shape, seed=3, round_to_bf16=True)
    return make_context(shape, to_device(w, torch.bfloat16), max_seqs=1, max_T=64, max_rows=64)


def reference(A, W, kind, Rz, N):
    a64, w64 = A.double().cpu().numpy(), W.double().cpu().numpy()
    if kind == "swiglu":
        g, u = a64 @ w64[:N].T, a64 @ w64[N:].T
        return g / (1 + np.exp(-g)) * u
    want = a64 @ w64.T
    return want + Rz.double().cpu().numpy() if Rz is not None else want


@pytest.mark.parametrize("M", [64, 33, 1, 128, 320, 512])
@pytest.mark.parametrize("name,N,K,kind", [("qkv", 12288, 4096, "store"), ("o", 4096, 4096, "residual"),
                                           ("gate_up", 12288, 4096, "swiglu"), ("down", 4096, 12288, "residual"),
                                           ("wide", 9216, 512, "store"), ("wide_swiglu", 6144, 1024, "swiglu"),
                                           ("narrow", 2048, 2048, "residual")])
def test_context_gemm_every_element(ctx, M, name, N, K, kind):
    g = torch.Generator(device="cuda").manual_seed(M * 7 + N + K)
    A = torch.randn(M, K, device="cuda", generator=g).to(torch.bfloat16)
    W = (torch.randn(N * (2 if kind == "swiglu" else 1), K, device="cuda", generator=g) * 0.02).to(torch.bfloat16)
    Rz = torch.randn(M, N, device="cuda", generator=g).to(torch.bfloat16) if kind == "residual" else None
    run = (lambda: ctx.gemm_swiglu(A, W)) if kind == "swiglu" else (lambda: ctx.gemm(A, W, residual=Rz))
    outs = [run() for _ in range(3)]
    torch.cuda.synchronize()
    want = reference(A, W, kind, Rz, N)
    got = outs[0].float().cpu().numpy()
    tol = 2.0 ** -8 * np.abs(want) + 2e-4
    assert (np.abs(got - want) <= tol).all(), (name, M, float((np.abs(got - want) / tol).max()))
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


def test_context_gemm_in_place_residual_and_other_paths_agree(ctx):
    """h = h + a W^T in place (how the forward calls it), and the same product through the LDS-tiled kernels
    (pvf_gemm without a context) within one bf16 rounding of a different float32 summation order."""
    g = torch.Generator(device="cuda").manual_seed(77)
    A = torch.randn(64, 4096, device="cuda", generator=g).to(torch.bfloat16)
    W = (torch.randn(4096, 4096, device="cuda", generator=g) * 0.02).to(torch.bfloat16)
    h = torch.randn(64, 4096, device="cuda", generator=g).to(torch.bfloat16)
    want = ctx.gemm(A, W, residual=h)
    tiled = B.gemm(A, W, residual=h)
    h2 = h.clone()
    ctx.gemm(A, W, residual=h2, out=h2)
    torch.cuda.synchronize()
    assert torch.equal(h2, want)
    d = (want.float() - tiled.float()).abs()
    assert bool((d <= 2.0 ** -7 * tiled.float().abs() + 1e-3).all())
