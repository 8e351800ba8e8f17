"""End-to-end parity of pvf_round / pvf_decode with the oracle on the small float32 model.

Every round's decisions (accept bits, winner, commits, proposals, next canvases) and the final
committed sequence must be identical.  A scaled-logit error e moves a top-1 probability p by
at most 2 e p (1 - p), i.e. by 2e relative.  The float32 path is held to e <= 1e-5 here
(test_scaled_logit_error_bound; the acceptance bar on logits is 1e-4), so a case is meaningful
when no oracle comparison sits closer than 2e-5 (relative) to flipping; each case walks seeds
from its first one to the first that qualifies.
"""
import numpy as np
import pytest
import torch

from oracle import pvf_oracle as O
from paper_2601_12247_amd import binding as B
from synth import inputs as S
from tests.gpu_util import (assert_state_equals, make_context, oracle_decode_cfg, oracle_model_cfg,
                            to_device)

pytestmark = pytest.mark.gpu
MARGIN = 2e-5
LOGIT_ERR = 1e-5


def dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda", dtype)


@pytest.fixture(scope="module")
def tiny():
    shape = S.TINY
    w = S.make_weights(shape, seed=0)
    ctx = make_context(shape, to_device(w), max_seqs=12, max_T=128, max_rows=64)
    cache = {}

    def fwd(canvas):
        key = bytes(np.asarray(canvas, np.int32))
        if key not in cache:
            cache[key] = O.forward(canvas, w, oracle_model_cfg(shape))
        return cache[key]

    return shape, ctx, fwd


def oracle_runs(shape, fwd, cfg, prompts, plan):
    ocfg = oracle_decode_cfg(cfg)
    return [O.decode(p, fwd, ocfg, cfg.logit_scale, shape.mask_id, plan) for p in prompts]


def find_case(shape, fwd, cfg, G, first_seed, plan_n=64):
    for seed in range(first_seed, first_seed + 30):
        prompts = [S.make_prompt(1000 * seed + g, cfg.prompt_len, shape.vocab, shape.mask_id) for g in range(G)]
        plan = S.make_plan_vocab(seed + 7, plan_n, shape.vocab, shape.mask_id)
        res = oracle_runs(shape, fwd, cfg, prompts, plan)
        if min(r.margin for r in res) >= MARGIN:
            return seed, prompts, plan, res
    pytest.fail(f"no seed with decision margin >= {MARGIN}")


def step_and_compare(shape, ctx, fwd, cfg, prompts, plan, compact, ws_trace=None):
    """Drive pvf_round from Python and compare the state with the oracle after every round."""
    G = len(prompts)
    ocfg = oracle_decode_cfg(cfg)
    bitmap = dev(S.plan_bitmap(plan, shape.vocab).view(np.int32), torch.int32)
    st = B.State(G, cfg)
    ctx.state_init(st, dev(np.stack(prompts), torch.int32))
    ost = [O.initial_state(p, ocfg, shape.mask_id) for p in prompts]
    rounds = 0
    while not all(o.done for o in ost):
        n_seq = sum(0 if o.done else 1 + o.drafts.n for o in ost)
        if compact:
            assert st.live_seqs() == n_seq
        ctx.round(st, bitmap, n_seq if compact else 0)
        torch.cuda.synchronize()
        rounds += 1
        for g in range(G):
            if ost[g].done:
                assert bool(st.done[g])
                continue
            new, info = O.pvf_round(ost[g], fwd, ocfg, cfg.logit_scale, shape.mask_id, plan)
            assert_state_equals(st, g, new, info, cfg, where=f"round {rounds} group {g}")
            if ws_trace is not None:
                ws_trace.append((new.ws, ost[g].ws, sum(info.accept)))
            ost[g] = new
        assert rounds <= cfg.gen_len + 1
    return st, rounds


def test_scaled_logit_error_bound(tiny):
    """The margin protocol above rests on this bound."""
    shape, ctx, fwd = tiny
    worst = 0.0
    for s in range(4):
        canvas = S.make_prompt(50 + s, 128, shape.vocab, shape.mask_id)
        canvas[64 + 8 * s:] = shape.mask_id
        rows = np.arange(64, 128, dtype=np.int32)
        got = ctx.forward(dev(canvas[None], torch.int32), dev(rows[None], torch.int32))[0].cpu().numpy()
        worst = max(worst, float(np.abs(shape.logit_scale * (got - fwd(canvas)[rows])).max()))
    print(f"max scaled-logit error: {worst:.3e}")
    assert worst <= LOGIT_ERR


def test_c1_committed_sequence_and_every_round_match(tiny):
    """64 prompt + 64 masked, block 32, tau 0.9, K = 2, planning vocabulary of 64 ids."""
    shape, ctx, fwd = tiny
    cfg = B.DecodeCfg(block_len=32, prompt_len=64, gen_len=64, K=2, tau_high=0.9, logit_scale=shape.logit_scale)
    seed, prompts, plan, res = find_case(shape, fwd, cfg, 1, first_seed=1)
    st, rounds = step_and_compare(shape, ctx, fwd, cfg, prompts, plan, compact=True)
    assert rounds == res[0].nfe
    assert np.array_equal(st.canvas[0, 0].cpu().numpy(), res[0].tokens)
    # the same through pvf_decode
    bitmap = dev(S.plan_bitmap(plan, shape.vocab).view(np.int32), torch.int32)
    out, stats = ctx.decode(B.State(1, cfg), dev(np.stack(prompts), torch.int32), bitmap)
    assert np.array_equal(out[0].cpu().numpy(), res[0].tokens)
    assert stats.rounds == res[0].nfe
    assert (stats.n_base, stats.n_plan, stats.n_ar) == (res[0].n_base, res[0].n_plan, res[0].n_ar)
    assert stats.n_base + stats.n_plan + stats.n_ar == cfg.gen_len
    assert not (out == shape.mask_id).any()


@pytest.mark.parametrize("compact", [True, False])
def test_batch_of_groups_with_ragged_draft_counts(tiny, compact):
    shape, ctx, fwd = tiny
    cfg = B.DecodeCfg(block_len=16, prompt_len=32, gen_len=48, K=3, tau_high=0.9, tau_ar_lo=0.3,
                      logit_scale=shape.logit_scale)
    seed, prompts, plan, res = find_case(shape, fwd, cfg, 3, first_seed=40, plan_n=400)
    st, rounds = step_and_compare(shape, ctx, fwd, cfg, prompts, plan, compact)
    assert rounds == max(r.nfe for r in res)
    for g in range(3):
        assert np.array_equal(st.canvas[g, 0].cpu().numpy(), res[g].tokens)


@pytest.mark.parametrize("kw", [dict(K=0), dict(K=2, routes=0), dict(K=2, routes=1), dict(K=4, routes=2)])
def test_threshold_mode_and_single_routes(tiny, kw):
    shape, ctx, fwd = tiny
    cfg = B.DecodeCfg(block_len=16, prompt_len=16, gen_len=32, tau_high=0.9, logit_scale=shape.logit_scale, **kw)
    seed, prompts, plan, res = find_case(shape, fwd, cfg, 2, first_seed=80, plan_n=400)
    bitmap = dev(S.plan_bitmap(plan, shape.vocab).view(np.int32), torch.int32)
    out, stats = ctx.decode(B.State(2, cfg), dev(np.stack(prompts), torch.int32), bitmap)
    for g in range(2):
        assert np.array_equal(out[g].cpu().numpy(), res[g].tokens)
    assert stats.rounds == max(r.nfe for r in res)
    assert stats.n_plan == sum(r.n_plan for r in res) and stats.n_ar == sum(r.n_ar for r in res)
    if kw.get("K") == 0 or kw.get("routes") == 0:
        assert stats.n_plan == 0 and stats.n_ar == 0 and stats.seq_forwards == sum(r.nfe for r in res)


@pytest.mark.parametrize("n_sparse", [4, 16])
def test_early_cross_block_revelation_end_to_end(tiny, n_sparse):
    """N_s > 0 (App. A.4.1): every round and the committed sequence match the oracle."""
    shape, ctx, fwd = tiny
    cfg = B.DecodeCfg(block_len=16, prompt_len=32, gen_len=64, K=3, tau_high=0.9, tau_ar_lo=0.3,
                      logit_scale=shape.logit_scale, n_sparse=n_sparse)
    assert cfg.R == 64
    seed, prompts, plan, res = find_case(shape, fwd, cfg, 2, first_seed=120, plan_n=400)
    trace = []
    st, rounds = step_and_compare(shape, ctx, fwd, cfg, prompts, plan, compact=True, ws_trace=trace)
    assert rounds == max(r.nfe for r in res)
    assert any(w == 2 for w, _, _ in trace)            # the working set did widen
    for g in range(2):
        assert np.array_equal(st.canvas[g, 0].cpu().numpy(), res[g].tokens)
    bitmap = dev(S.plan_bitmap(plan, shape.vocab).view(np.int32), torch.int32)
    out, stats = ctx.decode(B.State(2, cfg), dev(np.stack(prompts), torch.int32), bitmap)
    for g in range(2):
        assert np.array_equal(out[g].cpu().numpy(), res[g].tokens)
    assert stats.rounds == max(r.nfe for r in res)
    assert (stats.n_base, stats.n_plan, stats.n_ar) == tuple(sum(getattr(r, k) for r in res)
                                                             for k in ("n_base", "n_plan", "n_ar"))


def test_static_decoding_and_full_expansion_round_counts(tiny):
    """tau_high above 1 never fires, so the progress rule commits one token per forward
    (static one-token-per-step decoding); tau_high = 0 with N_s = block length commits two
    blocks per forward."""
    shape, ctx, fwd = tiny
    prompts = [S.make_prompt(5, 16, shape.vocab, shape.mask_id)]
    bitmap = torch.zeros((shape.vocab + 31) // 32, dtype=torch.int32, device="cuda")
    cfg = B.DecodeCfg(block_len=16, prompt_len=16, gen_len=32, K=0, tau_high=1.5, tau_plan_lo=0.0,
                      tau_plan_hi=0.0, logit_scale=shape.logit_scale)
    out, stats = ctx.decode(B.State(1, cfg), dev(np.stack(prompts), torch.int32), bitmap)
    assert stats.rounds == 32 and stats.n_base == 32 and not (out == shape.mask_id).any()
    cfg = B.DecodeCfg(block_len=16, prompt_len=16, gen_len=64, K=2, tau_high=0.0, tau_plan_lo=0.0,
                      tau_plan_hi=0.0, logit_scale=shape.logit_scale, n_sparse=16)
    out, stats = ctx.decode(B.State(1, cfg), dev(np.stack(prompts), torch.int32), bitmap)
    assert stats.rounds == 2 and stats.n_base == 64 and not (out == shape.mask_id).any()


def test_tau_high_zero_needs_one_round_per_block(tiny):
    shape, ctx, fwd = tiny
    cfg = B.DecodeCfg(block_len=16, prompt_len=16, gen_len=64, K=2, tau_high=0.0, tau_plan_lo=0.0,
                      tau_plan_hi=0.0, logit_scale=shape.logit_scale)
    prompts = [S.make_prompt(5, 16, shape.vocab, shape.mask_id)]
    bitmap = torch.zeros((shape.vocab + 31) // 32, dtype=torch.int32, device="cuda")
    out, stats = ctx.decode(B.State(1, cfg), dev(np.stack(prompts), torch.int32), bitmap)
    assert stats.rounds == 4 and stats.n_base == 64
    assert not (out == shape.mask_id).any()


def test_round_rejects_shapes_beyond_the_context(tiny):
    shape, ctx, fwd = tiny
    cfg = B.DecodeCfg(block_len=32, prompt_len=64, gen_len=128, K=2, logit_scale=20.0)   # T = 192 > 128
    st = B.State(1, cfg)
    bitmap = torch.zeros((shape.vocab + 31) // 32, dtype=torch.int32, device="cuda")
    with pytest.raises(B.PvfError) as e:
        ctx.round(st, bitmap)
    assert e.value.status == -2


def test_round_sync_status_words_equal_the_state(tiny):
    """pvf_round_sync = pvf_round + the packed per-group status read back with one copy."""
    shape, ctx, fwd = tiny
    cfg = B.DecodeCfg(block_len=16, prompt_len=32, gen_len=32, K=2, logit_scale=shape.logit_scale)
    G = 3
    prompts = np.stack([S.make_prompt(70 + g, 32, shape.vocab, shape.mask_id) for g in range(G)])
    plan = S.make_plan_vocab(5, 400, shape.vocab, shape.mask_id)
    bitmap = dev(S.plan_bitmap(plan, shape.vocab).view(np.int32), torch.int32)
    st, ref = B.State(G, cfg), B.State(G, cfg)
    ctx.state_init(st, dev(prompts, torch.int32))
    ctx.state_init(ref, dev(prompts, torch.int32))
    n_seq, rounds = G, 0
    while n_seq > 0:
        words = ctx.round_sync(st, bitmap, n_seq)
        ctx.round(ref, bitmap, n_seq)
        torch.cuda.synchronize()
        rounds += 1
        assert torch.equal(st.canvas, ref.canvas)
        for g in range(G):
            assert words[g] == (int(ref.done[g]), int(ref.n_drafts[g]), *ref.n_commit[g].cpu().tolist())
        n_seq = sum(0 if w[0] else 1 + w[1] for w in words)
        assert rounds <= 40
    assert int(ref.done.sum()) == G


def test_forward_driven_decode_accepts_planning_and_ar_drafts():
    """A model with self-consistent predictions (S.make_consistent_weights): through real forwards a planning
    draft passes Eq. (at) and wins Filter 2, and AR drafts pass the acceptance set of Sec. 4.3; every round of
    the decode, accepted drafts included, equals the oracle's."""
    shape = S.TINY
    w = S.make_consistent_weights(shape, seed=0, mix=20.0)
    ctx = make_context(shape, to_device(w), max_seqs=4, max_T=96, max_rows=64)
    cache = {}

    def fwd(canvas):
        key = bytes(np.asarray(canvas, np.int32))
        if key not in cache:
            cache[key] = O.forward(canvas, w, oracle_model_cfg(shape))
        return cache[key]

    cfg = B.DecodeCfg(block_len=32, prompt_len=32, gen_len=64, K=3, tau_high=0.5, tau_plan_lo=0.05, tau_plan_hi=0.4,
                      tau_ar_lo=0.01, logit_scale=24.0)
    plan = S.prior_plan_vocab(w, 256, shape.mask_id)
    ocfg = oracle_decode_cfg(cfg)
    for seed in range(1, 20):
        prompt = S.make_prompt(seed, cfg.prompt_len, shape.vocab, shape.mask_id)
        ref = O.decode(prompt, fwd, ocfg, cfg.logit_scale, shape.mask_id, plan)
        acc = {1: 0, 2: 0}
        for r in ref.rounds:
            if r.accept:
                acc[r.route] += sum(r.accept)
        if ref.margin >= MARGIN and acc[1] > 0 and acc[2] > 0 and ref.n_plan > 0 and ref.n_ar > 0:
            break
    else:
        pytest.fail("no prompt on which both a planning draft and an AR draft are accepted")
    st, rounds = step_and_compare(shape, ctx, fwd, cfg, [prompt], plan, compact=True)
    assert rounds == ref.nfe and np.array_equal(st.canvas[0, 0].cpu().numpy(), ref.tokens)
    bitmap = dev(S.plan_bitmap(plan, shape.vocab).view(np.int32), torch.int32)
    out, stats = ctx.decode(B.State(1, cfg), dev(prompt[None], torch.int32), bitmap)
    assert np.array_equal(out[0].cpu().numpy(), ref.tokens)
    assert (stats.n_base, stats.n_plan, stats.n_ar) == (ref.n_base, ref.n_plan, ref.n_ar)
    assert stats.n_plan > 0 and stats.n_ar > 0 and stats.drafts_accepted > 0
