"""GPU parity of the denoiser forward and its building blocks against the oracle (float64
arithmetic on the same float32 / bf16-rounded inputs), through the C ABI.

Tolerances: float32 path, logits scaled by the model's confidence temperature: max-abs 1e-4.
bf16 path, unscaled logits: max-abs 5e-2.  Building blocks carry tolerances derived from
their accumulation length and the output rounding (bf16: half an ulp = 2^-9 relative).
"""
import numpy as np
import pytest
import torch

from oracle import pvf_oracle as O
from paper_2601_12247_amd import binding as B
from synth import inputs as S
from tests.gpu_util import make_context, oracle_model_cfg, to_device

pytestmark = pytest.mark.gpu


def dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda", dtype)


def rnd(rng, shape, dtype, scale=1.0):
    x = (rng.standard_normal(shape) * scale).astype(np.float32)
    return S.bf16_round(x) if dtype == torch.bfloat16 else x


def tol(dtype, K, mag):
    """abs tolerance for a length-K dot product of O(1)xO(mag/sqrt(K)) terms."""
    if dtype == torch.float32:
        return 2e-6 * mag * max(1.0, np.sqrt(K) / 8)
    return mag * (2.0 ** -8)        # output rounding to bf16 dominates (fp32 accumulation)


GEMM_SHAPES = [(64, 64, 32), (100, 200, 72), (1, 8, 8), (257, 129, 520), (384, 768, 256),
               (384, 4096, 256), (130, 256, 704), (256, 256, 64), (300, 512, 1024), (1153, 256, 192)]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_and_residual(M, N, K, dtype):
    rng = np.random.default_rng(M * 7 + N)
    A, W, Rz = rnd(rng, (M, K), dtype), rnd(rng, (N, K), dtype, 1 / np.sqrt(K)), rnd(rng, (M, N), dtype)
    want = A.astype(np.float64) @ W.astype(np.float64).T
    got = B.gemm(dev(A, dtype), dev(W, dtype)).float().cpu().numpy()
    np.testing.assert_allclose(got, want, atol=tol(dtype, K, 4.0), rtol=2 ** -8 if dtype == torch.bfloat16 else 1e-5)
    r = dev(Rz, dtype)
    got = B.gemm(dev(A, dtype), dev(W, dtype), residual=r, out=r).float().cpu().numpy()   # in place on the residual
    np.testing.assert_allclose(got, want + Rz, atol=tol(dtype, K, 6.0), rtol=2 ** -8 if dtype == torch.bfloat16 else 1e-5)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("M,ff,K", [(64, 64, 32), (100, 88, 72), (384, 704, 256), (130, 256, 128), (520, 384, 512)])
def test_gemm_swiglu(M, ff, K, dtype):
    rng = np.random.default_rng(M + ff)
    A, W = rnd(rng, (M, K), dtype), rnd(rng, (2 * ff, K), dtype, 1 / np.sqrt(K))
    gu = A.astype(np.float64) @ W.astype(np.float64).T
    want = O.silu(gu[:, :ff]) * gu[:, ff:]
    got = B.gemm_swiglu(dev(A, dtype), dev(W, dtype)).float().cpu().numpy()
    np.testing.assert_allclose(got, want, atol=tol(dtype, K, 4.0), rtol=2 ** -7 if dtype == torch.bfloat16 else 1e-5)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("M,d", [(5, 256), (33, 4096), (7, 40)])
def test_rmsnorm(M, d, dtype):
    rng = np.random.default_rng(d)
    x, g = rnd(rng, (M, d), dtype, 3.0), rnd(rng, (d,), dtype)
    want = O.rmsnorm(x.astype(np.float64), g.astype(np.float64), 1e-5)
    got = B.rmsnorm(dev(x, dtype), dev(g, dtype), 1e-5).float().cpu().numpy()
    np.testing.assert_allclose(got, want, atol=1e-6 if dtype == torch.float32 else 0.0,
                               rtol=2e-6 if dtype == torch.float32 else 2 ** -8)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("S_,T,H,dh,theta", [(2, 128, 4, 64, 1e4), (1, 37, 2, 32, 1e4), (2, 200, 2, 128, 5e5),
                                             (1, 512, 2, 128, 5e5), (3, 1, 1, 16, 1e4),
                                             (2, 64, 1, 128, 5e5), (1, 192, 3, 128, 1e4),
                                             (1, 1280, 1, 128, 5e5)])
def test_rope_attention(S_, T, H, dh, theta, dtype):
    rng = np.random.default_rng(T + dh)
    d = H * dh
    qkv = rnd(rng, (S_ * T, 3 * d), dtype)
    want = np.empty((S_ * T, d))
    for s in range(S_):
        blk = qkv[s * T:(s + 1) * T].astype(np.float64)
        q, k, v = (blk[:, i * d:(i + 1) * d].reshape(T, H, dh) for i in range(3))
        want[s * T:(s + 1) * T] = O.attention(O.rope(q, theta), O.rope(k, theta), v).reshape(T, d)
    got = B.rope_attention(dev(qkv, dtype), S_, T, H, dh, theta).float().cpu().numpy()
    np.testing.assert_allclose(got, want, atol=3e-5 if dtype == torch.float32 else 2e-2, rtol=0)


@pytest.mark.parametrize("S_,T,H", [(5, 512, 32), (9, 1280, 32), (3, 512, 32), (1, 64, 2), (3, 96, 2), (2, 320, 4),
                                    (1, 1280, 6), (7, 160, 8), (1, 512, 32), (2, 512, 32), (4, 512, 32), (1, 128, 4)])
def test_qkv_attention_fused_epilogue_equals_separate_passes(S_, T, H):
    """The projection whose epilogue rotates q, k and writes the key-contiguous v, followed by the
    attention kernel, against pvf_gemm + pvf_rope_attention (rotation as a pass of its own)."""
    dh, d = 128, H * 128
    K = d                                                  # the projection maps d_model to 3 * d_model
    g = torch.Generator(device="cuda").manual_seed(S_ * T + H)
    x = torch.randn(S_ * T, K, device="cuda", generator=g).to(torch.bfloat16)
    w = (torch.randn(3 * d, K, device="cuda", generator=g) * (1.6 / K ** 0.5)).to(torch.bfloat16)   # scores of std ~2.5
    qkv, out = B.qkv_attention(x, w, S_, T, H, dh, 5e5)
    ref_qkv = B.gemm(x, w)
    v_plain = ref_qkv[:, 2 * d:].clone()
    ref_out = B.rope_attention(ref_qkv, S_, T, H, dh, 5e5)  # rotates ref_qkv in place
    torch.cuda.synchronize()
    assert torch.equal(qkv[:, 2 * d:], v_plain)             # v is stored unchanged
    a, b = qkv[:, : 2 * d].float(), ref_qkv[:, : 2 * d].float()
    # the same fp32 formula on both sides, up to the contraction of one multiply-add before the bf16 rounding
    assert (a - b).abs().max().item() <= 2 ** -7 * b.abs().max().item()
    assert (a != b).float().mean().item() < 0.02
    scale = ref_out.float().abs().max().item()
    assert scale > 0.3                                      # sharp enough that misplaced keys would show
    assert (out.float() - ref_out.float()).abs().max().item() <= 2e-2 * scale


@pytest.mark.parametrize("dtype,S_,T,H,dh", [(torch.float32, 2, 48, 2, 64), (torch.bfloat16, 1, 100, 2, 128),
                                             (torch.bfloat16, 2, 64, 3, 32)])
def test_qkv_attention_without_the_fused_epilogue(dtype, S_, T, H, dh):
    """Shapes the fused rotary epilogue does not cover (float32, head sizes other than 128, canvas
    lengths that are no multiple of 64): pvf_qkv_attention is pvf_gemm + pvf_rope_attention."""
    d = H * dh
    g = torch.Generator(device="cuda").manual_seed(S_ * T + dh)
    x = torch.randn(S_ * T, d, device="cuda", generator=g).to(dtype)
    w = (torch.randn(3 * d, d, device="cuda", generator=g) * (1.2 / d ** 0.5)).to(dtype)
    qkv, out = B.qkv_attention(x, w, S_, T, H, dh, 1e4)
    ref_qkv = B.gemm(x, w)
    ref_out = B.rope_attention(ref_qkv, S_, T, H, dh, 1e4)
    torch.cuda.synchronize()
    assert torch.equal(qkv, ref_qkv) and torch.equal(out, ref_out)


def test_forward_tiny_fp32_logits_within_1e4():
    shape = S.TINY
    w = S.make_weights(shape, seed=0)
    ctx = make_context(shape, to_device(w), max_seqs=3, max_T=128, max_rows=128)
    mc = oracle_model_cfg(shape)
    toks = np.stack([S.make_prompt(s, 128, shape.vocab, shape.mask_id) for s in range(3)])
    toks[:, 64:] = shape.mask_id
    toks[1, 70] = 5; toks[2, 64:80] = S.make_prompt(9, 16, shape.vocab, shape.mask_id)
    rows = np.stack([np.arange(64, 128), np.arange(0, 64), np.r_[np.arange(100, 128), -np.ones(36)]]).astype(np.int32)
    got = ctx.forward(dev(toks, torch.int32), dev(rows, torch.int32)).cpu().numpy()
    for s in range(3):
        ok = rows[s] >= 0
        want = O.forward(toks[s], w, mc, rows=rows[s][ok])
        err = np.abs(shape.logit_scale * (got[s][ok] - want)).max()
        assert err <= 1e-4, f"canvas {s}: scaled-logit error {err}"
        assert np.all(got[s][~ok] == 0)


def test_forward_is_batch_invariant_and_deterministic():
    shape = S.TINY
    w = to_device(S.make_weights(shape, seed=0))
    ctx = make_context(shape, w, max_seqs=4, max_T=96, max_rows=32)
    toks = np.stack([S.make_prompt(s, 96, shape.vocab, shape.mask_id) for s in range(4)])
    rows = np.tile(np.arange(64, 96, dtype=np.int32), (4, 1))
    a = ctx.forward(dev(toks, torch.int32), dev(rows, torch.int32))
    b = ctx.forward(dev(toks, torch.int32), dev(rows, torch.int32))
    assert torch.equal(a, b)
    one = ctx.forward(dev(toks[2:3], torch.int32), dev(rows[2:3], torch.int32))
    assert torch.equal(one[0], a[2])       # a canvas's logits do not depend on its batch mates


def test_forward_bf16_mfma_is_batch_invariant_above_640_rows():
    """On the MFMA path every GEMM tile shape accumulates k in the same order, attention works per
    canvas: with more than 640 token rows per launch (up to there GEMMs may split K, which changes the
    rounding order with the launch size) a canvas's bf16 logits are bit-identical whatever rides along.
    (The output head has 64 rows per canvas: its K = 256 is too short to be split.)"""
    shape = S.ModelShape(n_layers=2, d_model=256, n_heads=2, d_ff=512, vocab=2048, mask_id=2047, rope_theta=5e5)
    w = to_device(S.make_weights(shape, seed=4, round_to_bf16=True), torch.bfloat16)
    ctx = make_context(shape, w, max_seqs=4, max_T=704, max_rows=64)
    toks = np.stack([S.make_prompt(20 + s, 704, shape.vocab, shape.mask_id) for s in range(4)])
    rows = np.tile(np.arange(640, 704, dtype=np.int32), (4, 1))
    four = ctx.forward(dev(toks, torch.int32), dev(rows, torch.int32))
    again = ctx.forward(dev(toks, torch.int32), dev(rows, torch.int32))
    assert torch.equal(four, again)
    for sub in ([1], [0, 3], [2, 1, 0]):
        part = ctx.forward(dev(toks[sub], torch.int32), dev(rows[sub], torch.int32))
        for i, sq in enumerate(sub):
            assert torch.equal(part[i], four[sq]), f"canvas {sq} in a batch of {len(sub)}"


def test_forward_bf16_two_layer_small_within_5e2():
    """bf16 storage path on a reduced-width model (plain kernels or MFMA, whichever the
    dispatcher picks for these shapes)."""
    shape = S.ModelShape(n_layers=2, d_model=256, n_heads=2, d_ff=512, vocab=2048, mask_id=2047,
                         rope_theta=5e5)
    w = S.make_weights(shape, seed=3, round_to_bf16=True)
    ctx = make_context(shape, to_device(w, torch.bfloat16), max_seqs=2, max_T=160, max_rows=64)
    toks = np.stack([S.make_prompt(s, 160, shape.vocab, shape.mask_id) for s in range(2)])
    toks[:, 96:] = shape.mask_id
    rows = np.tile(np.arange(96, 160, dtype=np.int32), (2, 1))
    got = ctx.forward(dev(toks, torch.int32), dev(rows, torch.int32)).float().cpu().numpy()
    for s in range(2):
        want = O.forward(toks[s], w, oracle_model_cfg(shape), rows=rows[s])
        assert np.abs(got[s] - want).max() <= 5e-2


@pytest.mark.parametrize("S_,T", [(1, 256), (2, 160), (1, 64), (3, 128), (2, 96), (1, 512), (1, 640), (2, 320)])
def test_forward_bf16_few_rows_split_k_within_5e2(S_, T):
    """Forwards of at most 384 token rows take the split-K GEMMs (tall tiles, K divided over several
    workgroups, float32 partial sums added by a second kernel) for the O, gate/up and down projections;
    from there to 640 rows the O and down projections still do (128x128 tiles that would leave CUs idle)."""
    shape = S.ModelShape(n_layers=2, d_model=1024, n_heads=8, d_ff=2048, vocab=2048, mask_id=2047, rope_theta=5e5)
    w = S.make_weights(shape, seed=5, round_to_bf16=True)
    ctx = make_context(shape, to_device(w, torch.bfloat16), max_seqs=S_, max_T=T, max_rows=64)
    toks = np.stack([S.make_prompt(10 + s, T, shape.vocab, shape.mask_id) for s in range(S_)])
    toks[:, T - 40:] = shape.mask_id
    rows = np.tile(np.arange(T - 64, T, dtype=np.int32), (S_, 1))
    got = ctx.forward(dev(toks, torch.int32), dev(rows, torch.int32)).float().cpu().numpy()
    again = ctx.forward(dev(toks, torch.int32), dev(rows, torch.int32)).float().cpu().numpy()
    assert np.array_equal(got, again)                       # partial sums are added in a fixed order
    for s in range(S_):
        want = O.forward(toks[s], w, oracle_model_cfg(shape), rows=rows[s])
        assert np.abs(got[s] - want).max() <= 5e-2


def test_forward_shape_errors():
    shape = S.TINY
    ctx = make_context(shape, to_device(S.make_weights(shape, seed=0)), max_seqs=1, max_T=32, max_rows=8)
    t = torch.zeros(2, 32, dtype=torch.int32, device="cuda")
    r = torch.zeros(2, 8, dtype=torch.int32, device="cuda")
    with pytest.raises(B.PvfError) as e:
        ctx.forward(t, r)
    assert e.value.status == -2
