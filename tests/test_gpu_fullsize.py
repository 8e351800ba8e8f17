"""Parity at the benchmark's full sizes and launch configurations.

The oracle cannot run a 32-layer, 8B-parameter forward in seconds, so at full size each kernel is
checked on its own at the exact shapes the bench launches (same tile-shape selection, same
grid), on outputs the oracle can compute one by one:
  * the four per-layer GEMMs and the output head at M = 2560 (5 canvases x 512 tokens) and
    M = 512: sampled output elements against float64 dot products of the same bf16 inputs;
  * RoPE + attention at 32 heads, T = 512 and 1280: sampled (canvas, head, query) rows;
  * stage 1 on bf16 logits [8 x 256, 126464]: every row against the oracle;
  * a 2-layer model at the full widths (d 4096, ff 12288, vocab 126464), bf16, 2 canvases of 256 tokens
    (the few-row tile shapes and split-K): logits of the window rows within rms 1.5e-2 / max 8e-2 of the
    oracle's, the bound that replaces 5e-2 max-abs at this width (derived in test_gpu_bench_shapes.py,
    which also covers the launch shapes of the benchmark rounds);
  * a complete PVF decode of the benchmark workload: structural properties that hold for any
    weights (no mask left, prompt untouched, every token committed once, K = 0 commits by the
    threshold only, determinism).
"""
import numpy as np
import pytest
import torch

from oracle import pvf_oracle as O
from paper_2601_12247_amd import binding as B
from paper_2601_12247_amd import workloads as W
from synth import inputs as S
from tests.gpu_util import make_context, oracle_model_cfg, to_device

pytestmark = pytest.mark.gpu
D, FF, V = 4096, 12288, 126464


def randn_bf16(shape, seed, std):
    t = torch.empty(*shape, dtype=torch.bfloat16, device="cuda")
    B.fill_normal(t, seed, 0.0, std)
    return t


def f64(t):
    return t.float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("M", [2560, 512])
@pytest.mark.parametrize("name,N,K,kind", [("qkv", 3 * D, D, "store"), ("o", D, D, "residual"),
                                           ("gate_up", FF, D, "swiglu"), ("down", D, FF, "residual")])
def test_layer_gemms_at_bench_shapes(M, name, N, K, kind):
    rng = np.random.default_rng(M + N)
    A = randn_bf16((M, K), 1, 1.0)
    Wt = randn_bf16((N * (2 if kind == "swiglu" else 1), K), 2, 0.02)
    Rz = randn_bf16((M, N), 3, 1.0) if kind == "residual" else None
    if kind == "swiglu":
        out = B.gemm_swiglu(A, Wt)
    else:
        out = B.gemm(A, Wt, residual=Rz)
    ms = np.r_[0, M - 1, rng.integers(0, M, 30)]
    ns = np.r_[0, N - 1, rng.integers(0, N, 30)]
    a = f64(A[torch.as_tensor(ms, device="cuda")])
    for j, n in enumerate(ns):
        if kind == "swiglu":
            g = a[j] @ f64(Wt[int(n)])
            u = a[j] @ f64(Wt[N + int(n)])
            want = g / (1 + np.exp(-g)) * u
        else:
            want = a[j] @ f64(Wt[int(n)])
            if Rz is not None:
                want += float(Rz[int(ms[j]), int(n)])
        got = float(out[int(ms[j]), int(n)])
        assert abs(got - want) <= 2 ** -8 * abs(want) + 1e-2, (name, M, int(ms[j]), int(n), got, want)


def test_output_head_at_bench_shape():
    rows = 5 * 64
    A = randn_bf16((rows, D), 4, 1.0)
    Wt = randn_bf16((V, D), 5, 0.02)
    out = B.gemm(A, Wt)
    rng = np.random.default_rng(0)
    for m, n in zip(np.r_[0, rows - 1, rng.integers(0, rows, 40)], np.r_[0, V - 1, rng.integers(0, V, 40)]):
        want = f64(A[int(m)]) @ f64(Wt[int(n)])
        assert abs(float(out[int(m), int(n)]) - want) <= 2 ** -8 * abs(want) + 1e-2


@pytest.mark.parametrize("S_,T", [(5, 512), (2, 1280)])
def test_attention_at_bench_shapes(S_, T):
    H, dh, theta = 32, 128, 5e5
    qkv = randn_bf16((S_ * T, 3 * D), 6, 1.0)
    ref = qkv.clone()
    out = B.rope_attention(qkv, S_, T, H, dh, theta)
    rng = np.random.default_rng(T)
    for s, h in [(0, 0), (S_ - 1, H - 1)] + [(int(rng.integers(S_)), int(rng.integers(H))) for _ in range(3)]:
        blk = f64(ref[s * T:(s + 1) * T])
        q, k, v = (blk[:, i * D + h * dh: i * D + (h + 1) * dh].reshape(T, 1, dh) for i in range(3))
        want = O.attention(O.rope(q, theta), O.rope(k, theta), v)[:, 0, :]
        got = f64(out[s * T:(s + 1) * T, h * dh:(h + 1) * dh])
        rows = np.r_[0, T - 1, rng.integers(0, T, 30)]
        assert np.abs(got[rows] - want[rows]).max() <= 2e-2


def test_stage1_full_epilogue_workload_every_row():
    rows, mask_id = 8 * 256, 126336
    l = S.make_boosted_logits(3, rows, V, boost_hi=12.0, mask_id=mask_id)
    conf, tok = B.stage1(torch.from_numpy(l).to("cuda", torch.bfloat16), mask_id, 1.0)
    p, t = O.stage1(l, 1.0, mask_id)
    assert np.array_equal(tok.cpu().numpy(), t)
    np.testing.assert_allclose(conf.cpu().numpy(), p, rtol=5e-6)


def test_two_layer_full_width_bf16_forward_rms_1p5e2_max_8e2():
    shape = S.ModelShape(n_layers=2, d_model=D, n_heads=32, d_ff=FF, vocab=V, mask_id=126336, rope_theta=5e5)
    w = S.make_weights(shape, seed=21, round_to_bf16=True)
    ctx = make_context(shape, to_device(w, torch.bfloat16), max_seqs=2, max_T=256, max_rows=64)
    toks = np.stack([S.make_prompt(s, 256, V, shape.mask_id) for s in range(2)])
    toks[:, 128:] = shape.mask_id
    toks[1, 128:140] = S.make_prompt(7, 12, V, shape.mask_id)
    rows = np.tile(np.arange(128, 192, dtype=np.int32), (2, 1))
    got = ctx.forward(torch.from_numpy(toks).cuda(), torch.from_numpy(rows).cuda()).float().cpu().numpy()
    for s in range(2):
        want = O.forward(toks[s], w, oracle_model_cfg(shape), rows=rows[s])
        err = np.abs(got[s] - want).max()
        rms = float((got[s] - want).std())
        print(f"canvas {s}: logit error rms = {rms:.4f}, max = {err:.4f} over {want.size} logits "
              f"(logit std {want.std():.3f})")
        # At the full widths the 5e-2 max-abs bar (met by the reduced-width model in test_gpu_forward.py)
        # is a statistical extreme of bf16 storage itself: tests/bf16_emulation.py, the float64 forward
        # with only the round-to-bf16 of each stored activation, sits at rms ~1.3e-2 / max ~6e-2 from
        # the oracle (asserted in test_gpu_bench_shapes.py).  So the rms, which a wrong kernel would
        # blow up, and the maximum at ~6 rms are bounded instead.
        assert rms <= 1.5e-2
        assert err <= 8e-2
        # the decisions stage 1 takes on these logits agree wherever the oracle's top-2 gap exceeds the error
        p, t = O.stage1(want, 1.0, shape.mask_id)
        pg, tg = O.stage1(got[s], 1.0, shape.mask_id)
        top2 = np.sort(np.delete(want, shape.mask_id, axis=1), axis=1)[:, -2:]
        clear = (top2[:, 1] - top2[:, 0]) > 2 * err
        assert np.array_equal(t[clear], tg[clear])


def test_bench_workload_decode_properties():
    dims = dict(W.LLADA_8B)
    K, bl, P, Gn = 4, 32, 256, 256
    weights = W.random_model(dims, seed=0)
    ctx = W.make_context(dims, weights, max_seqs=1 + K, max_T=P + Gn, max_rows=2 * bl)
    prompt = W.random_prompts(1, P, dims["vocab"], dims["mask_id"], seed=1)
    bitmap = W.random_plan_bitmap(512, dims["vocab"], dims["mask_id"], seed=2)
    cfg = B.DecodeCfg(block_len=bl, prompt_len=P, gen_len=Gn, K=K, tau_high=0.9, logit_scale=12.0)
    out, st = ctx.decode(B.State(1, cfg), prompt, bitmap)
    out2, st2 = ctx.decode(B.State(1, cfg), prompt, bitmap)
    assert torch.equal(out, out2) and st.rounds == st2.rounds                    # deterministic
    assert int((out == dims["mask_id"]).sum()) == 0                              # nothing left masked
    assert torch.equal(out[:, :P], prompt)                                       # prompt untouched
    assert st.n_base + st.n_plan + st.n_ar == Gn                                 # every token committed once
    assert Gn // bl <= st.rounds <= Gn and st.rounds <= st.seq_forwards <= st.rounds * (1 + K)
    cfg0 = B.DecodeCfg(block_len=bl, prompt_len=P, gen_len=Gn, K=0, tau_high=0.9, logit_scale=12.0)
    out0, s0 = ctx.decode(B.State(1, cfg0), prompt, bitmap)
    assert s0.n_base == Gn and s0.n_plan == 0 and s0.n_ar == 0 and s0.seq_forwards == s0.rounds
    assert int((out0 == dims["mask_id"]).sum()) == 0
    # tau_high = 0 commits a whole block per round
    cfgz = B.DecodeCfg(block_len=bl, prompt_len=P, gen_len=Gn, K=0, tau_high=0.0, tau_plan_lo=0.0,
                       tau_plan_hi=0.0, logit_scale=12.0)
    _, sz = ctx.decode(B.State(1, cfgz), prompt, bitmap)
    assert sz.rounds == Gn // bl
