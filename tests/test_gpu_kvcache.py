"""GPU parity of decoding with the block-level K/V cache (decode_cfg.kv_cache = 1) against
oracle/pvf_kvcache.py, through pvf_round / pvf_decode.

Protocol as in test_gpu_decode.py: float32 tiny model, seeds walked to the first case whose
oracle decision margin is >= MARGIN; every round's confidences are compared within CONF_RTOL and
every decision (tokens, accept bits, winner, commits, next drafts) bit for bit."""
import numpy as np
import pytest
import torch

from oracle import pvf_kvcache as KV
from oracle import pvf_oracle as O
from paper_2601_12247_amd import binding as B
from synth import inputs as S
from tests.gpu_util import assert_state_equals, make_context, oracle_decode_cfg, oracle_model_cfg, to_device

pytestmark = pytest.mark.gpu

MARGIN = 2e-5
CONF_RTOL = 1e-4


def dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda", dtype)


@pytest.fixture(scope="module")
def tiny():
    shape = S.TINY
    w = S.make_weights(shape, seed=0)
    ctx = make_context(shape, to_device(w), max_seqs=12, max_T=128, max_rows=64)
    return shape, ctx, w, oracle_model_cfg(shape)


def oracle_rounds(shape, w, mcfg, cfg, prompts, plan):
    """Per group: list of (conf, tok, refreshed, new state, info) for every round, plus the margin."""
    ocfg = oracle_decode_cfg(cfg)
    out, margin = [], np.inf
    for p in prompts:
        st, cache, rounds = O.initial_state(p, ocfg, shape.mask_id), None, []
        while not st.done:
            conf, tok, cache, refreshed = KV.cached_summaries(st, cache, w, mcfg, ocfg, cfg.logit_scale, shape.mask_id)
            new, info = O.decide(st, conf, tok, ocfg, shape.mask_id, plan)
            rounds.append((conf, tok, refreshed, st, new, info))
            margin = min(margin, info.margin)
            st = new
        out.append(rounds)
    return out, margin


def find_case(shape, w, mcfg, cfg, G, first_seed, plan_n=400):
    for seed in range(first_seed, first_seed + 30):
        prompts = [S.make_prompt(1000 * seed + g, cfg.prompt_len, shape.vocab, shape.mask_id) for g in range(G)]
        plan = S.make_plan_vocab(seed + 7, plan_n, shape.vocab, shape.mask_id)
        rounds, margin = oracle_rounds(shape, w, mcfg, cfg, prompts, plan)
        if margin >= MARGIN:
            return prompts, plan, rounds
    pytest.fail(f"no seed with decision margin >= {MARGIN}")


def step_and_compare(shape, ctx, cfg, prompts, plan, rounds):
    G = len(prompts)
    bitmap = dev(S.plan_bitmap(plan, shape.vocab).view(np.int32), torch.int32)
    st = B.State(G, cfg)
    ctx.state_init(st, dev(np.stack(prompts), torch.int32))
    n_rounds = max(len(r) for r in rounds)
    seen = {"refresh": 0, "cached": 0, "cached_with_drafts": 0, "accepted_in_cached": 0}
    for t in range(n_rounds):
        ctx.round(st, bitmap, 0)
        torch.cuda.synchronize()
        for g in range(G):
            if t >= len(rounds[g]):
                assert bool(st.done[g])
                continue
            conf, tok, refreshed, old, new, info = rounds[g][t]
            n = old.drafts.n
            gc, gt = st.conf[g].cpu().numpy()[: 1 + n], st.tok[g].cpu().numpy()[: 1 + n]
            assert np.array_equal(gt, tok), f"round {t} group {g}: top-1 tokens (refreshed={refreshed})"
            np.testing.assert_allclose(gc, conf, rtol=CONF_RTOL, atol=1e-7)
            assert_state_equals(st, g, new, info, cfg, where=f"round {t} group {g}")
            seen["refresh" if refreshed else "cached"] += 1
            if not refreshed and n:
                seen["cached_with_drafts"] += 1
                seen["accepted_in_cached"] += sum(info.accept)
    return st, seen


def test_cached_decode_every_round_matches_oracle(tiny):
    shape, ctx, w, mcfg = tiny
    cfg = B.DecodeCfg(block_len=16, prompt_len=32, gen_len=48, K=3, tau_high=0.9, tau_ar_lo=0.3,
                      logit_scale=shape.logit_scale, kv_cache=1)
    prompts, plan, rounds = find_case(shape, w, mcfg, cfg, 3, first_seed=300)
    st, seen = step_and_compare(shape, ctx, cfg, prompts, plan, rounds)
    assert seen["cached"] > seen["refresh"] >= 3 and seen["cached_with_drafts"] > 0, seen
    for g in range(3):
        assert np.array_equal(st.canvas[g, 0].cpu().numpy(), rounds[g][-1][4].y)
    # the same through pvf_decode
    bitmap = dev(S.plan_bitmap(plan, shape.vocab).view(np.int32), torch.int32)
    out, stats = ctx.decode(B.State(3, cfg), dev(np.stack(prompts), torch.int32), bitmap)
    for g in range(3):
        assert np.array_equal(out[g].cpu().numpy(), rounds[g][-1][4].y)
    assert stats.rounds == max(len(r) for r in rounds)
    assert stats.n_base + stats.n_plan + stats.n_ar == 3 * cfg.gen_len


@pytest.mark.parametrize("kw", [dict(K=0), dict(K=2, n_sparse=4), dict(K=4, routes=2, block_len=32, gen_len=64)])
def test_cached_decode_variants(tiny, kw):
    """Threshold decoding, early cross-block revelation (4-block window) and a window cut by the
    end of the canvas (last block: half of the window rows do not exist)."""
    shape, ctx, w, mcfg = tiny
    base = dict(block_len=16, prompt_len=32, gen_len=32, tau_high=0.9, tau_ar_lo=0.3, logit_scale=shape.logit_scale,
                kv_cache=1)
    base.update(kw)
    cfg = B.DecodeCfg(**base)
    prompts, plan, rounds = find_case(shape, w, mcfg, cfg, 2, first_seed=340)
    st, seen = step_and_compare(shape, ctx, cfg, prompts, plan, rounds)
    assert seen["cached"] > 0
    for g in range(2):
        assert np.array_equal(st.canvas[g, 0].cpu().numpy(), rounds[g][-1][4].y)


def test_cache_is_an_approximation_and_first_round_is_exact(tiny):
    shape, ctx, w, mcfg = tiny
    kw = dict(block_len=16, prompt_len=32, gen_len=32, K=2, tau_high=0.9, logit_scale=shape.logit_scale)
    prompts = np.stack([S.make_prompt(77, 32, shape.vocab, shape.mask_id)])
    bitmap = torch.zeros((shape.vocab + 31) // 32, dtype=torch.int32, device="cuda")
    confs = {}
    for kv in (0, 1):
        cfg = B.DecodeCfg(kv_cache=kv, **kw)
        st = B.State(1, cfg)
        ctx.state_init(st, dev(prompts, torch.int32))
        ctx.round(st, bitmap, 0)
        first = st.conf[0, 0].cpu().numpy().copy()
        ctx.round(st, bitmap, 0)
        confs[kv] = (first, st.conf[0, 0].cpu().numpy().copy(), int(st.k_active[0]))
    assert np.array_equal(confs[0][0], confs[1][0])                       # refresh round = the full forward itself
    if confs[1][2] == 0:                                                  # still in block 0: the second round was cached
        assert not np.array_equal(confs[0][1], confs[1][1])
        np.testing.assert_allclose(confs[0][1], confs[1][1], atol=0.2)    # ... and close to the exact one


def test_bf16_cached_decode_completes_and_agrees_on_refresh_rounds():
    """bf16 weights of a small wide model (MFMA GEMMs with few rows): the cached decode finishes,
    commits gen_len tokens, and its first round equals the uncached first round bit for bit (both forward the
    two backbone canvases only: the kernels a forward takes, hence its rounding order, depend on its row count)."""
    shape = S.ModelShape(n_layers=2, d_model=256, n_heads=2, d_ff=512, vocab=4096, mask_id=4095, logit_scale=20.0)
    w = S.make_weights(shape, seed=3)
    ctx = make_context(shape, to_device(w, torch.bfloat16), max_seqs=10, max_T=192, max_rows=64)
    prompts = np.stack([S.make_prompt(5 + g, 64, shape.vocab, shape.mask_id) for g in range(2)])
    bitmap = dev(S.plan_bitmap(S.make_plan_vocab(1, 400, shape.vocab, shape.mask_id), shape.vocab).view(np.int32), torch.int32)
    kw = dict(block_len=32, prompt_len=64, gen_len=128, K=4, tau_high=0.9, logit_scale=shape.logit_scale)
    first = {}
    for kv in (0, 1):
        cfg = B.DecodeCfg(kv_cache=kv, **kw)
        st = B.State(2, cfg)
        ctx.state_init(st, dev(prompts, torch.int32))
        ctx.round(st, bitmap, 2)
        first[kv] = (st.conf.cpu().numpy().copy(), st.canvas.cpu().numpy().copy())
        out, stats = ctx.decode(B.State(2, cfg), dev(prompts, torch.int32), bitmap)
        assert not (out == shape.mask_id).any() and stats.n_base + stats.n_plan + stats.n_ar == 2 * cfg.gen_len
        assert torch.equal(out[:, :64].cpu(), torch.from_numpy(prompts))
    assert np.array_equal(first[0][0], first[1][0]) and np.array_equal(first[0][1], first[1][1])


@pytest.mark.parametrize("bl,pl,gl", [(32, 64, 128), (24, 48, 144)], ids=["mfma-window", "row-major-v-cache"])
def test_bf16_window_attention_on_matrix_cores_matches_oracle(bl, pl, gl):
    """d_head = 128, bf16, 64-row window: the cached round takes the MFMA window-attention path.
    With blocks of 24 the window kernel does not apply: the cache keeps V row-major, which the fused
    QKV projection of the refresh round then has to write (it otherwise writes only the key-contiguous copy).
    Round 1 (refresh) and round 2 (cached) are run on the GPU; the oracle repeats round 2 from the
    GPU's own state after round 1, on the bf16-rounded weights.  bf16 activations move a
    confidence by a few 1e-3 at this temperature, so confidences are compared within 2e-2 absolute
    / 4e-3 on average, and top-1 tokens wherever the oracle's confidence is not tiny."""
    from tests.gpu_util import oracle_state
    shape = S.ModelShape(n_layers=2, d_model=256, n_heads=2, d_ff=512, vocab=4096, mask_id=4095, logit_scale=6.0)
    w = S.make_weights(shape, seed=5)
    wb = {k: (S.bf16_round(v) if k != "layers" else [{kk: S.bf16_round(vv) for kk, vv in lw.items()} for lw in v])
          for k, v in w.items()}
    mcfg = oracle_model_cfg(shape)
    ctx = make_context(shape, to_device(wb, torch.bfloat16), max_seqs=10, max_T=192, max_rows=64)
    cfg = B.DecodeCfg(block_len=bl, prompt_len=pl, gen_len=gl, K=4, tau_high=0.9, tau_plan_lo=0.05, tau_plan_hi=0.6,
                      tau_ar_lo=0.05, logit_scale=shape.logit_scale, kv_cache=1)
    ocfg = oracle_decode_cfg(cfg)
    G = 2
    prompts = np.stack([S.make_prompt(15 + g, pl, shape.vocab, shape.mask_id) for g in range(G)])
    plan = S.make_plan_vocab(1, 2000, shape.vocab, shape.mask_id)
    bitmap = dev(S.plan_bitmap(plan, shape.vocab).view(np.int32), torch.int32)
    st = B.State(G, cfg)
    ctx.state_init(st, dev(prompts, torch.int32))
    ctx.round(st, bitmap, 0)                                  # refresh: full forward, cache filled
    torch.cuda.synchronize()
    ost = [oracle_state(st, g) for g in range(G)]
    assert all(not o.done and o.k_active == 0 for o in ost) and sum(o.drafts.n for o in ost) > 0
    ctx.round(st, bitmap, 0)                                  # cached: window rows only
    torch.cuda.synchronize()
    worst, total, n, tok_ok, tok_n = 0.0, 0.0, 0, 0, 0
    for g in range(G):
        y0 = np.array(list(prompts[g]) + [shape.mask_id] * cfg.gen_len, dtype=np.int32)
        _, cache = KV.forward_full(y0, wb, mcfg)              # what the refresh round cached: the initial canvas
        cache.block = 0
        conf, tok, _, refreshed = KV.cached_summaries(ost[g], cache, wb, mcfg, ocfg, cfg.logit_scale, shape.mask_id)
        assert not refreshed
        k = 1 + ost[g].drafts.n
        gc, gt = st.conf[g].cpu().numpy()[:k], st.tok[g].cpu().numpy()[:k]
        diff = np.abs(gc - conf)
        worst, total, n = max(worst, float(diff.max())), total + float(diff.sum()), n + diff.size
        sure = conf > 0.05
        tok_ok += int((gt[sure] == tok[sure]).sum()); tok_n += int(sure.sum())
    print(f"window MFMA attention: max |dconf| {worst:.2e}, mean {total / n:.2e}, tokens {tok_ok}/{tok_n}")
    assert worst <= 2e-2 and total / n <= 4e-3 and tok_ok >= 0.98 * tok_n and tok_n > 20
