"""Parity against the oracle in the launch configurations the benchmark rounds take.

A round of the bench workload forwards 1-5 canvases of 512 tokens at the full model widths.  The
kernels such a launch selects (256 x 256 tiles with the rotary / key-contiguous-v epilogue for the QKV
projection, 320 x 128 or 192 x 128 tiles for the O and down projections, the 256 x 256 SwiGLU tile,
the MFMA attention) differ from those a 512-row launch selects, so they are checked here at M = 2560
(5 canvases) and M = 1536 (3 canvases):
  * a 2-layer model at the full widths, window logits of every canvas against oracle.forward;
  * the fused QKV epilogue against float64 directly: whole rows of rotated q | rotated k | v, and the
    whole key-contiguous copy of v;
  * every layer GEMM on whole rows and whole columns that cross every tile of every grid;
  * the bf16-storage emulation (tests/bf16_emulation.py) as the derivation of the full-width bound;
  * the same 2-layer model forwarded as 9 x 1280 and 80 x 1024 canvases (the larger full-batch forwards the
    benchmark times), a few canvases of each against oracle.forward.
"""
import numpy as np
import pytest
import torch

from oracle import pvf_oracle as O
from paper_2601_12247_amd import binding as B
from synth import inputs as S
from tests.bf16_emulation import forward_bf16_storage
from tests.gpu_util import make_context, oracle_model_cfg, to_device

pytestmark = pytest.mark.gpu
D, FF, V, H, DH, THETA = 4096, 12288, 126464, 32, 128, 5e5
T, P, R = 512, 256, 64
SHAPE = S.ModelShape(n_layers=2, d_model=D, n_heads=H, d_ff=FF, vocab=V, mask_id=126336, rope_theta=THETA)

# Bound that replaces the 5e-2 max-abs bar on bf16 logits at the full width (see the emulation test):
# rms of the logit error and its maximum over the ~8 million window logits of a canvas.
RMS_BOUND, MAX_BOUND = 1.5e-2, 8e-2


@pytest.fixture(scope="module")
def weights():
    w = S.make_weights(SHAPE, seed=21, round_to_bf16=True)
    return w, to_device(w, torch.bfloat16)


@pytest.fixture(scope="module")
def model(weights):
    w, w_dev = weights
    return w, make_context(SHAPE, w_dev, max_seqs=5, max_T=T, max_rows=R)


def canvases(n):
    """Backbone: prompt + masks with the first block partly committed; drafts: the backbone plus 1..4 fills."""
    base = np.full(T, SHAPE.mask_id, dtype=np.int32)
    base[:P] = S.make_prompt(31, P, V, SHAPE.mask_id)
    base[P:P + 9] = S.make_prompt(32, 9, V, SHAPE.mask_id)
    fills = S.make_prompt(33, 8, V, SHAPE.mask_id)
    out = [base]
    for j in range(1, n):
        c = base.copy()
        c[P + 9 + 2 * np.arange(j)] = fills[:j]
        out.append(c)
    return np.stack(out)


_oracle_cache = {}


def oracle_logits(w, canvas, rows):
    key = canvas.tobytes()
    if key not in _oracle_cache:
        _oracle_cache[key] = O.forward(canvas, w, oracle_model_cfg(SHAPE), rows=rows)
    return _oracle_cache[key]


@pytest.mark.parametrize("n_seq", [5, 3])
def test_two_layer_full_width_forward_at_bench_launch_shapes(model, n_seq):
    """M = 2560 and M = 1536: every canvas' window logits against the oracle, within the full-width bound."""
    w, ctx = model
    toks = canvases(n_seq)
    rows = np.tile(np.arange(P, P + R, dtype=np.int32), (n_seq, 1))
    got = ctx.forward(torch.from_numpy(toks).cuda(), torch.from_numpy(rows).cuda()).float().cpu().numpy()
    for s in range(n_seq):
        want = oracle_logits(w, toks[s], rows[s])
        diff = got[s] - want
        rms, err = float(np.sqrt(np.mean(diff ** 2))), float(np.abs(diff).max())
        print(f"S={n_seq} canvas {s}: rms {rms:.4f} max {err:.4f} (logit std {want.std():.3f})", flush=True)
        assert abs(float(diff.mean())) <= 1e-3                       # no bias
        assert rms <= RMS_BOUND and err <= MAX_BOUND
        _, t = O.stage1(want, 1.0, SHAPE.mask_id)
        _, tg = O.stage1(got[s], 1.0, SHAPE.mask_id)
        top2 = np.sort(np.delete(want, SHAPE.mask_id, axis=1), axis=1)[:, -2:]
        clear = (top2[:, 1] - top2[:, 0]) > 2 * err
        assert clear.sum() >= 8 and np.array_equal(t[clear], tg[clear])


def test_bf16_storage_emulation_derives_the_full_width_bound(model):
    """Why 5e-2 max-abs cannot hold at d = 4096 in bf16.  (a) The float64 forward with nothing but a
    round-to-bf16 at each stored activation already sits at rms ~1.2e-2 / max ~6e-2 from the oracle: the
    bound asserted above is this figure plus margin, not a property of the kernels.  (b) The kernels
    are no further from the oracle than that emulation is: they add nothing to the cost of bf16
    storage.  (The distance between kernels and emulation is printed only: the two round at different
    places -- the library folds each norm into the projections around it -- and the first rounding that
    falls differently changes which way later ones fall, so they are about as far from each other as
    two independent bf16 pipelines.)"""
    w, ctx = model
    toks = canvases(2)
    rows = np.tile(np.arange(P, P + R, dtype=np.int32), (2, 1))
    got = ctx.forward(torch.from_numpy(toks).cuda(), torch.from_numpy(rows).cuda()).float().cpu().numpy()
    for s in range(2):
        want = oracle_logits(w, toks[s], rows[s])
        emu = forward_bf16_storage(toks[s], w, 2, D, H, FF, SHAPE.rms_eps, THETA, rows=rows[s])
        e_rms, e_max = float(np.sqrt(np.mean((emu - want) ** 2))), float(np.abs(emu - want).max())
        g_rms, g_max = float(np.sqrt(np.mean((got[s] - emu) ** 2))), float(np.abs(got[s] - emu).max())
        o_rms = float(np.sqrt(np.mean((got[s] - want) ** 2)))
        print(f"canvas {s}: emulation vs oracle rms {e_rms:.4f} max {e_max:.4f}; GPU vs emulation rms {g_rms:.4f} "
              f"max {g_max:.4f}; GPU vs oracle rms {o_rms:.4f}", flush=True)
        assert 0.8e-2 <= e_rms <= RMS_BOUND and 4e-2 <= e_max <= MAX_BOUND    # bf16 storage alone costs this much
        assert o_rms <= 1.1 * e_rms                                           # the kernels add nothing to it


def big_canvases(n, T_, P_, seed):
    """n canvases of T_ tokens: one prompt + masks with a few committed tokens, the others differing in 1..3 fills."""
    base = np.full(T_, SHAPE.mask_id, dtype=np.int32)
    base[:P_] = S.make_prompt(seed, P_, V, SHAPE.mask_id)
    base[P_:P_ + 5] = S.make_prompt(seed + 1, 5, V, SHAPE.mask_id)
    fills = S.make_prompt(seed + 2, 3 * n, V, SHAPE.mask_id)
    out = np.tile(base, (n, 1))
    for j in range(1, n):
        k = 1 + j % 3
        out[j, P_ + 7 + 3 * np.arange(k)] = fills[3 * j:3 * j + k]
    return out


@pytest.mark.parametrize("n_seq,T_,P_,R_,check", [(9, 1280, 256, 128, (0, 8)), (80, 1024, 512, 64, (37, 79))])
def test_two_layer_full_width_forward_at_the_larger_configurations(weights, n_seq, T_, P_, R_, check):
    """9 x 1280 (M = 11 520) and 80 x 1024 (M = 81 920), the two larger full-batch forwards the benchmark times:
    every projection runs 256 x 256 tiles over many rounds there (O and down too, with 16 slots of folded-norm
    sums), attention has 10 / 8 query tiles per head.  Window logits of two canvases of each against the oracle,
    same bound as at 5 x 512."""
    w, w_dev = weights
    ctx = make_context(SHAPE, w_dev, max_seqs=n_seq, max_T=T_, max_rows=R_)
    toks = big_canvases(n_seq, T_, P_, seed=41)
    rows = np.tile(np.arange(P_, P_ + R_, dtype=np.int32), (n_seq, 1))
    got = ctx.forward(torch.from_numpy(toks).cuda(), torch.from_numpy(rows).cuda()).float().cpu().numpy()
    del ctx
    torch.cuda.empty_cache()
    for s in check:
        want = O.forward(toks[s], w, oracle_model_cfg(SHAPE), rows=rows[s])
        diff = got[s] - want
        rms, err = float(np.sqrt(np.mean(diff ** 2))), float(np.abs(diff).max())
        print(f"{n_seq} x {T_} canvas {s}: rms {rms:.4f} max {err:.4f} (logit std {want.std():.3f})", flush=True)
        assert abs(float(diff.mean())) <= 1e-3
        assert rms <= RMS_BOUND and err <= MAX_BOUND
        _, t = O.stage1(want, 1.0, SHAPE.mask_id)
        _, tg = O.stage1(got[s], 1.0, SHAPE.mask_id)
        top2 = np.sort(np.delete(want, SHAPE.mask_id, axis=1), axis=1)[:, -2:]
        clear = (top2[:, 1] - top2[:, 0]) > 2 * err
        assert clear.sum() >= 8 and np.array_equal(t[clear], tg[clear])


def spread_rows(M, n):
    """n rows, one per stretch of M / n, at varying offsets inside a 32-row group."""
    step = M // n
    return np.array([i * step + (7 * i) % min(step, 32) for i in range(n)])


def test_fused_qkv_epilogue_against_float64_at_m2560():
    """QKV projection of 5 x 512 rows with the rotary embedding and the key-contiguous copy of v in its
    epilogue: 80 whole rows (all 12288 columns, one row in every 32-row stretch, so every tile of the
    10 x 48 grid and every XCD band is crossed) against O.rope of the float64 product, and the whole vt."""
    S_, M = 5, 5 * T
    g = torch.Generator(device="cuda").manual_seed(5)
    x = torch.randn(M, D, device="cuda", generator=g).to(torch.bfloat16)
    w = (torch.randn(3 * D, D, device="cuda", generator=g) * 0.02).to(torch.bfloat16)
    vt = torch.zeros(S_, H, DH, T, dtype=torch.bfloat16, device="cuda")
    qkv, _ = B.qkv_attention(x, w, S_, T, H, DH, THETA, vt=vt)
    torch.cuda.synchronize()
    rows = spread_rows(M, 80)
    xs = x[torch.as_tensor(rows, device="cuda")].double().cpu().numpy()
    prod = xs @ w.double().cpu().numpy().T                                  # [80, 3d] float64
    got = qkv[torch.as_tensor(rows, device="cuda")].float().cpu().numpy()
    pos = (rows % T).astype(np.float64)
    for third in range(2):
        pre = prod[:, third * D:(third + 1) * D].reshape(len(rows), H, DH)
        want = O.rope(pre, THETA, pos)
        mag = np.abs(pre[..., :DH // 2]) + np.abs(pre[..., DH // 2:])       # |a| + |b| of each rotated pair
        # a and b are rounded to bf16 before the rotation (relative 2^-8 each, |cos|, |sin| <= 1), the result once more
        tol = 2.0 ** -8 * (np.concatenate([mag, mag], axis=-1) + np.abs(want)) + 1e-4
        err = np.abs(got[:, third * D:(third + 1) * D].reshape(len(rows), H, DH) - want)
        assert (err <= tol).all(), (third, float((err / tol).max()))
    v_want = prod[:, 2 * D:]
    v_got = got[:, 2 * D:]
    assert (np.abs(v_got - v_want) <= 2.0 ** -8 * np.abs(v_want) + 1e-4).all()
    # the key-contiguous copy: every element of v, keys of each 16 stored as 0-3, 8-11, 4-7, 12-15
    t = torch.arange(T, device="cuda")
    tp = (t & ~12) | ((t & 4) << 1) | ((t & 8) >> 1)
    v = qkv[:, 2 * D:].view(S_, T, H, DH).permute(0, 2, 3, 1)               # [S, H, DH, T]
    assert torch.equal(vt[..., tp], v)


@pytest.mark.parametrize("M", [2560, 1536])
@pytest.mark.parametrize("name,N,K,kind", [("qkv", 3 * D, D, "store"), ("o", D, D, "residual"),
                                           ("gate_up", FF, D, "swiglu"), ("down", D, FF, "residual")])
def test_layer_gemms_whole_rows_and_columns(M, name, N, K, kind):
    """One whole output row in every 32-row stretch and one whole column in every 64-column stretch:
    together they cross every tile of every tile shape the launch can take, in every XCD band."""
    g = torch.Generator(device="cuda").manual_seed(M + N)
    A = torch.randn(M, K, device="cuda", generator=g).to(torch.bfloat16)
    Wt = (torch.randn(N * (2 if kind == "swiglu" else 1), K, device="cuda", generator=g) * 0.02).to(torch.bfloat16)
    Rz = torch.randn(M, N, device="cuda", generator=g).to(torch.bfloat16) if kind == "residual" else None
    out = (B.gemm_swiglu(A, Wt) if kind == "swiglu" else B.gemm(A, Wt, residual=Rz)).float().cpu().numpy()
    a64, w64 = A.double().cpu().numpy(), Wt.double().cpu().numpy()
    res = Rz.double().cpu().numpy() if Rz is not None else None

    def reference(ms, ns):
        if kind == "swiglu":
            gate, up = a64[ms] @ w64[ns].T, a64[ms] @ w64[N + ns].T
            return gate / (1 + np.exp(-gate)) * up
        want = a64[ms] @ w64[ns].T
        return want + res[np.ix_(ms, ns)] if res is not None else want

    ms, ns = spread_rows(M, M // 32), spread_rows(N, N // 64)
    for rr, cc in ((ms, np.arange(N)), (np.arange(M), ns)):
        want = reference(rr, cc)
        err = np.abs(out[np.ix_(rr, cc)] - want)
        tol = 2.0 ** -8 * np.abs(want) + 2e-4
        assert (err <= tol).all(), (name, M, float((err / tol).max()))


def test_output_head_whole_rows_and_columns():
    rows = 5 * R
    g = torch.Generator(device="cuda").manual_seed(9)
    A = torch.randn(rows, D, device="cuda", generator=g).to(torch.bfloat16)
    Wt = (torch.randn(V, D, device="cuda", generator=g) * 0.02).to(torch.bfloat16)
    out = B.gemm(A, Wt).float().cpu().numpy()
    a64, w64 = A.double().cpu().numpy(), Wt.double().cpu().numpy()
    ms, ns = spread_rows(rows, 10), spread_rows(V, V // 64)
    for rr, cc in ((ms, np.arange(V)), (np.arange(rows), ns)):
        want = a64[rr] @ w64[cc].T
        assert (np.abs(out[np.ix_(rr, cc)] - want) <= 2.0 ** -8 * np.abs(want) + 2e-4).all()
