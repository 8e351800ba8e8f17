"""GPU parity of the decision epilogue against the oracle, through the C ABI.

Bar: token ids, accept bits, winners, committed canvases, proposals -> bit-exact;
confidences -> relative 5e-6 (float32 sum order and exp2 differ from the oracle's float64).
Because a confidence within a few ulps of a threshold could flip a decision, each decision
case walks seeds from its first one to the first whose oracle decision margin is >= 1e-5.
"""
import numpy as np
import pytest
import torch

from oracle import pvf_oracle as O
from paper_2601_12247_amd import binding as B
from synth import inputs as S
from tests.gpu_util import assert_state_equals, oracle_decode_cfg, oracle_state

pytestmark = pytest.mark.gpu
CONF_RTOL = 5e-6


def dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda", dtype)


def check_stage1(l_np, dtype, mask_id, scale):
    conf, tok = B.stage1(dev(l_np, dtype), mask_id, scale)
    p, t = O.stage1(l_np, scale, mask_id)
    assert np.array_equal(tok.cpu().numpy(), t)
    np.testing.assert_allclose(conf.cpu().numpy(), p, rtol=CONF_RTOL, atol=0)


@pytest.mark.parametrize("rows,V,dtype,scale", [
    (37, 126464, torch.bfloat16, 1.0),     # full vocabulary width, 16-byte path, ragged last stride
    (16, 126464, torch.bfloat16, 7.5),
    (64, 4096, torch.float32, 20.0),       # small parity model's shape
    (64, 4096, torch.bfloat16, 1.0),
    (9, 8200, torch.float32, 3.0),         # 16-byte path with a short tail
    (5, 1001, torch.bfloat16, 2.0),        # odd width -> element-wise path
    (5, 77, torch.float32, 1.0),
    (3, 2, torch.float32, 1.0),            # a single live column
])
def test_stage1_matches_oracle(rows, V, dtype, scale):
    mask_id = V - 1 if V < 100000 else 126336
    l = S.make_boosted_logits(11, rows, V, boost_hi=14.0, mask_id=mask_id)
    if dtype == torch.float32:             # use values that are not bf16-representable too
        l = (l + np.random.default_rng(1).standard_normal(l.shape).astype(np.float32) * 1e-3).astype(np.float32)
    check_stage1(l, dtype, mask_id, scale)


def test_stage1_ties_mask_column_and_extremes():
    V, mask_id = 16384, 5000
    rng = np.random.default_rng(3)
    l = S.bf16_round(rng.standard_normal((8, V)).astype(np.float32))
    l[0, [9000, 300, 12000]] = 6.0          # three-way tie -> lowest id
    l[1, mask_id] = 50.0                    # the mask column must be ignored
    l[2, :] = 1.5                           # all equal -> p = 1/(V-1), id 0
    l[3, V - 1] = 30.0                      # winner in the very last element
    l[4, 0] = 30.0                          # ... and in the very first
    l[5, mask_id - 1] = 9.0; l[5, mask_id + 1] = 9.0   # tie around the mask column
    l[6, :] = -40.0; l[6, 77] = -39.0       # all-negative row
    for dtype in (torch.bfloat16, torch.float32):
        check_stage1(l, dtype, mask_id, 1.0)
    conf, tok = B.stage1(dev(l, torch.bfloat16), mask_id, 1.0)
    t = tok.cpu().numpy()
    assert (t[0], t[2], t[3], t[4], t[5], t[6]) == (300, 0, V - 1, 0, mask_id - 1, 77)
    assert t[1] != mask_id


def test_stage1_is_deterministic():
    l = dev(S.make_boosted_logits(5, 64, 126464, mask_id=126336), torch.bfloat16)
    a = B.stage1(l, 126336, 1.0)
    b = B.stage1(l, 126336, 1.0)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_stage1_rejects_bad_arguments():
    l = torch.zeros(2, 64, device="cuda")
    with pytest.raises(B.PvfError):
        B.stage1(l, 64, 1.0)                # mask id out of range
    with pytest.raises(B.PvfError):
        B.stage1(l, 3, 0.0)                 # non-positive scale
    conf, tok = B.stage1(torch.zeros(0, 64, device="cuda"), 3, 1.0)   # empty input is fine
    assert conf.numel() == 0


# ------------------------------------------------------------------------------------------
# full epilogue: two chained rounds per group so that the second one has drafts to verify
# ------------------------------------------------------------------------------------------
def draft_consistent_logits(rng, G, K, R, V, mask_id, boost_hi, jitter):
    """[G, 1+K, R, V]: slot 0 rows are boosted-noise rows, draft slots are slot 0 plus small
    noise so that most (not all) top-1 tokens survive."""
    base = S.make_boosted_logits(int(rng.integers(1 << 30)), G * R, V, boost_hi, mask_id).reshape(G, 1, R, V)
    out = np.repeat(base, 1 + K, axis=1)
    out[:, 1:] += rng.standard_normal((G, K, R, V)).astype(np.float32) * jitter
    return S.bf16_round(out)


def run_two_rounds(seed, G, K, bl, gen_len, V, dtype, routes=3, tau_high=0.9, boost_hi=18.0,
                   plan_n=None, jitter=0.4, prompt_len=4, band=(0.2, 0.65), n_sparse=0, rounds=3,
                   persistent=False, round_jitter=0.15, tau_ar=0.1):
    """persistent: every round scores the SAME boosted table plus fresh small noise (a model whose
    predictions persist from round to round), so that AR fills proposed in one round can still be the
    arg-max in the next (accepted) and the impact set of a round holds only rows that newly crossed
    tau_high (sometimes none: rejected).  Otherwise every round draws a fresh table."""
    mask_id = V - 1
    cfg = B.DecodeCfg(block_len=bl, prompt_len=prompt_len, gen_len=gen_len, K=K, routes=routes,
                      tau_high=tau_high, tau_plan_lo=band[0], tau_plan_hi=band[1], tau_ar_lo=tau_ar,
                      logit_scale=1.0, n_sparse=n_sparse)
    ocfg = oracle_decode_cfg(cfg)
    R = cfg.R
    rng = np.random.default_rng(seed)
    plan = S.make_plan_vocab(seed + 1, plan_n or V // 4, V, mask_id)
    bitmap = dev(S.plan_bitmap(plan, V).view(np.int32), torch.int32)
    prompts = np.stack([S.make_prompt(seed + 10 + g, prompt_len, V, mask_id) for g in range(G)])
    # library state, initialised by the library itself
    st = B.State(G, cfg)
    st.canvas[:] = mask_id
    st.canvas[:, :, :prompt_len] = dev(prompts, torch.int32)[:, None, :]
    ost = [O.initial_state(prompts[g], ocfg, mask_id) for g in range(G)]
    margin = np.inf
    seen = {"accept": 0, "reject": 0, "plan": 0, "ar": 0, "wide": 0, "wide_accept": 0}
    table = S.make_boosted_logits(seed + 3, G * R, V, boost_hi, mask_id).reshape(G, 1, R, V) if persistent else None
    for rnd in range(rounds):
        if persistent:
            lg = np.repeat(table, 1 + K, axis=1)
            lg[:, :1] += rng.standard_normal((G, 1, R, V)).astype(np.float32) * round_jitter
            lg[:, 1:] += rng.standard_normal((G, K, R, V)).astype(np.float32) * jitter
            lg = S.bf16_round(lg)
        else:
            lg = draft_consistent_logits(rng, G, K, R, V, mask_id, boost_hi, jitter)
        B.epilogue(dev(lg, dtype), st, bitmap, V, mask_id)
        torch.cuda.synchronize()
        for g in range(G):
            if ost[g].done:
                continue
            n = ost[g].drafts.n
            wp = O.window_positions(ocfg, ost[g].k_active)
            conf = np.zeros((1 + n, R), np.float32); tok = np.full((1 + n, R), -1, np.int32)
            ok = wp < ocfg.T
            for j in range(1 + n):
                conf[j, ok], tok[j, ok] = O.stage1(lg[g, j][ok], 1.0, mask_id)
            gc, gt = st.conf[g].cpu().numpy(), st.tok[g].cpu().numpy()
            assert np.array_equal(gt[: 1 + n], tok), f"round {rnd} group {g}: top-1 tokens"
            np.testing.assert_allclose(gc[: 1 + n], conf, rtol=CONF_RTOL)
            new, info = O.decide(ost[g], conf, tok, ocfg, mask_id, plan)
            margin = min(margin, info.margin)
            if info.margin >= 1e-5:
                assert_state_equals(st, g, new, info, cfg, where=f"seed {seed} round {rnd} group {g}")
            seen["accept"] += sum(info.accept); seen["reject"] += len(info.accept) - sum(info.accept)
            seen["plan"] += info.route == 1; seen["ar"] += info.route == 2
            seen["wide"] += new.ws == 2; seen["wide_accept"] += sum(info.accept) if ost[g].ws == 2 else 0
            ost[g] = new
        if margin < 1e-5:
            return margin, seen
    return margin, seen


def walk_seeds(first_seed, **kw):
    for seed in range(first_seed, first_seed + 20):
        margin, seen = run_two_rounds(seed, **kw)
        if margin >= 1e-5:
            return seed, seen
    pytest.fail("no seed with decision margin >= 1e-5")


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_epilogue_rounds_match_oracle_small_vocab(dtype):
    tot = {"accept": 0, "reject": 0, "plan": 0, "ar": 0}
    for first in (100, 200, 300):
        seed, seen = walk_seeds(first, G=5, K=4, bl=32, gen_len=96, V=4096, dtype=dtype)
        for k in tot:
            tot[k] += seen[k]
    assert all(v > 0 for v in tot.values()), tot      # both routes, both outcomes were exercised


@pytest.mark.parametrize("n_sparse,bl,gen_len,rounds", [(16, 16, 64, 5), (6, 16, 48, 8), (32, 32, 64, 4),
                                                        (3, 8, 8, 4)])
def test_epilogue_early_cross_block_revelation(n_sparse, bl, gen_len, rounds):
    """Working sets of two blocks (App. A.4.1): verify, commit and propose all range over both."""
    tot = {"accept": 0, "reject": 0, "wide": 0, "wide_accept": 0}
    for first in (700, 720):
        seed, seen = walk_seeds(first, G=4, K=4, bl=bl, gen_len=gen_len, V=2048, dtype=torch.float32,
                                n_sparse=n_sparse, rounds=rounds, tau_high=0.85)
        for k in tot:
            tot[k] += seen[k]
    if gen_len > bl:
        assert tot["wide"] > 0 and tot["wide_accept"] > 0 and tot["reject"] > 0, tot
    else:
        assert tot["wide"] == 0                        # a single block has nothing to reveal


@pytest.mark.parametrize("routes,K", [(0, 3), (1, 2), (2, 8), (3, 0), (3, 1)])
def test_epilogue_route_switches_and_budgets(routes, K):
    walk_seeds(400 + 10 * routes + K, G=3, K=K, bl=16, gen_len=32, V=2048, dtype=torch.float32,
               routes=routes, tau_high=0.8)


def test_epilogue_single_block_window_and_last_block():
    # gen_len == block_len: the window is one block; finishing it finishes the canvas
    walk_seeds(500, G=4, K=4, bl=64, gen_len=64, V=2048, dtype=torch.bfloat16, boost_hi=24.0)
    # tau_high = 0 commits every mask of the block at once (ends blocks early)
    walk_seeds(510, G=2, K=2, bl=8, gen_len=16, V=1024, dtype=torch.float32, tau_high=0.0,
               band=(0.0, 0.0))


def test_epilogue_full_vocabulary_rows():
    """Full-width rows (V = 126464, bf16), 256-row single-block window, K = 4."""
    seed, seen = walk_seeds(600, G=2, K=4, bl=256, gen_len=256, V=126464, dtype=torch.bfloat16,
                            plan_n=512 * 32, prompt_len=0)
    assert seen["plan"] + seen["ar"] > 0


@pytest.mark.parametrize("routes,first_seed,kw", [
    (1, 610, dict(plan_n=126464 // 2, round_jitter=1.0, jitter=1.0)),   # confidences move between rounds: impact sets form
    (2, 640, dict(tau_ar=1e-4, jitter=0.3))])                            # weak AR fills: some stop being the arg-max
def test_epilogue_full_vocabulary_both_outcomes_on_each_route(routes, first_seed, kw):
    """V = 126464, bf16, predictions that persist between rounds: on the planning route and on the AR
    route drafts are verified at the real vocabulary width, and both outcomes (accepted, rejected) occur."""
    tot = {"accept": 0, "reject": 0, "plan": 0, "ar": 0}
    for k in range(6):
        seed, seen = walk_seeds(first_seed + 5 * k, G=1, K=4, bl=32, gen_len=64, V=126464, dtype=torch.bfloat16,
                                prompt_len=0, routes=routes, rounds=5, persistent=True, **kw)
        for key in tot:
            tot[key] += seen[key]
        if tot["accept"] > 0 and tot["reject"] > 0:
            break
    assert tot["accept"] > 0 and tot["reject"] > 0, tot
    assert tot["plan" if routes == 1 else "ar"] > 0 and tot["ar" if routes == 1 else "plan"] == 0, tot


def test_epilogue_rejects_bad_configuration():
    cfg = B.DecodeCfg(block_len=8, prompt_len=0, gen_len=12, K=2)        # 12 % 8 != 0
    st = B.State(1, B.DecodeCfg(block_len=4, prompt_len=0, gen_len=12, K=2))
    st.cfg = cfg
    lg = torch.zeros(1, 3, 12, 64, device="cuda")
    bm = torch.zeros(2, dtype=torch.int32, device="cuda")
    with pytest.raises(B.PvfError):
        B.epilogue(lg, st, bm, 64, 63)
    st.cfg = B.DecodeCfg(block_len=4, prompt_len=0, gen_len=12, K=2, tau_plan_hi=0.95)  # band above tau_high
    with pytest.raises(B.PvfError):
        B.epilogue(lg, st, bm, 64, 63)
    st.cfg = B.DecodeCfg(block_len=4, prompt_len=0, gen_len=12, K=2, n_sparse=-1)
    with pytest.raises(B.PvfError) as e:
        B.epilogue(lg, st, bm, 64, 63)
    assert e.value.status == -1
