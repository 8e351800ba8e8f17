"""Pins for early cross-block revelation (App. A.4.1, Eq. block_expansion) in the oracle:
the working set becomes {active block's masks} + {whole next block} once at most N_s masks are
left in the active block.  Checked against an independently written threshold decoder, by
brute force over two-block working sets, by closed-form round counts and by schedule equality."""
import itertools

import numpy as np
import pytest
import scipy.special

from oracle import pvf_oracle as O
from synth import inputs as S


def table_fn(V, seed, spread=2.5):
    return lambda canvas: S.table_model_logits(canvas, V, seed=seed, spread=spread)


def top1(row, mask_id):
    ids = [w for w in range(len(row)) if w != mask_id]
    pr = scipy.special.softmax(np.asarray(row, np.float32)[ids].astype(np.float64))
    best = pr.max()
    return min(i for i, p in zip(ids, pr) if p == best), np.float32(best)


def working_set(y, cfg, mask_id):
    """Direct statement of Eq. (block_expansion): indices eligible for replacement."""
    S_ = cfg.block_len
    gen = [cfg.prompt_len + i for i in range(cfg.gen_len)]
    masked = [i for i in gen if y[i] == mask_id]
    k = (masked[0] - cfg.prompt_len) // S_
    blk = lambda b: range(cfg.prompt_len + b * S_, cfg.prompt_len + (b + 1) * S_)
    M_active = [i for i in blk(k) if y[i] == mask_id]
    if cfg.n_sparse > 0 and len(M_active) <= cfg.n_sparse and k + 1 < cfg.gen_len // S_:
        return M_active + [i for i in blk(k + 1) if y[i] == mask_id]
    return M_active


def threshold_decode_sparse(prompt, fn, cfg, mask_id):
    y = np.array(list(prompt) + [mask_id] * cfg.gen_len, dtype=np.int32)
    nfe, trail = 0, []
    while (y == mask_id).any():
        Bt = working_set(y, cfg, mask_id)
        logits = fn(y); nfe += 1
        pred = {i: top1(logits[i], mask_id) for i in Bt}
        hit = [i for i in Bt if pred[i][1] >= np.float32(cfg.tau_high)] or \
              [max(Bt, key=lambda i: (pred[i][1], -i))]
        for i in hit:
            y[i] = pred[i][0]
        trail.append(y.copy())
    return y, nfe, trail


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("ns", [1, 3, 4])
def test_k0_equals_independent_threshold_decoder_with_expansion(seed, ns):
    V, mask_id = 12, 11
    cfg = O.DecodeCfg(block_len=4, prompt_len=3, gen_len=16, tau_high=0.55, tau_plan_lo=0.2,
                      tau_plan_hi=0.5, K=0, n_sparse=ns)
    fn = table_fn(V, seed)
    res = O.decode([1, 2, 3], fn, cfg, 1.0, mask_id, [])
    y, nfe, trail = threshold_decode_sparse([1, 2, 3], fn, cfg, mask_id)
    assert np.array_equal(res.tokens, y) and res.nfe == nfe
    expanded = 0
    prev = np.array([1, 2, 3] + [mask_id] * 16)
    for t in trail:                                     # commits never go beyond active block + 1
        k = (np.flatnonzero(prev == mask_id)[0] - 3) // 4
        changed = np.flatnonzero(t != prev)
        assert changed.max() < 3 + (k + 2) * 4
        expanded += changed.max() >= 3 + (k + 1) * 4
        prev = t
    if ns == 4:
        assert expanded > 0                             # N_s = block length: always expanded


def test_tau_zero_with_full_expansion_commits_two_blocks_per_round():
    V, mask_id = 12, 11
    for n_blocks in (4, 5):
        cfg = O.DecodeCfg(block_len=4, prompt_len=2, gen_len=4 * n_blocks, tau_high=0.0, tau_plan_lo=0.0,
                          tau_plan_hi=0.0, K=2, n_sparse=4)
        res = O.decode([1, 2], table_fn(V, 3), cfg, 1.0, mask_id, range(11))
        assert res.nfe == (n_blocks + 1) // 2
    cfg0 = O.DecodeCfg(block_len=4, prompt_len=2, gen_len=16, tau_high=0.0, tau_plan_lo=0.0, tau_plan_hi=0.0, K=2)
    assert O.decode([1, 2], table_fn(V, 3), cfg0, 1.0, mask_id, range(11)).nfe == 4


@pytest.mark.parametrize("seed", range(8))
def test_schedules_agree_with_expansion(seed):
    V, mask_id = 16, 15
    cfg = O.DecodeCfg(block_len=4, prompt_len=3, gen_len=16, tau_high=0.7, tau_plan_lo=0.15,
                      tau_plan_hi=0.6, tau_ar_lo=0.2, K=3, n_sparse=2)
    plan = sorted(np.random.default_rng(seed).choice(V - 1, 7, replace=False).tolist())
    fn = table_fn(V, seed)
    res = O.decode([4, 5, 6], fn, cfg, 1.0, mask_id, plan)
    y, nfe, trail = O.decode_literal([4, 5, 6], fn, cfg, 1.0, mask_id, plan)
    got = list(res.canvases[1:])
    if not got or not np.array_equal(got[-1], res.tokens):
        got.append(res.tokens)
    assert np.array_equal(res.tokens, y) and len(got) == len(trail)
    assert all(np.array_equal(a, b) for a, b in zip(got, trail))
    assert res.n_base + res.n_plan + res.n_ar == cfg.gen_len


def test_expansion_off_is_the_default_path():
    V, mask_id = 16, 15
    kw = dict(block_len=4, prompt_len=3, gen_len=16, tau_high=0.7, tau_plan_lo=0.15, tau_plan_hi=0.6, K=3)
    for seed in range(4):
        a = O.decode([4, 5, 6], table_fn(V, seed), O.DecodeCfg(**kw), 1.0, mask_id, range(5))
        b = O.decode([4, 5, 6], table_fn(V, seed), O.DecodeCfg(**kw, n_sparse=0), 1.0, mask_id, range(5))
        assert np.array_equal(a.tokens, b.tokens) and a.nfe == b.nfe
    assert O.DecodeCfg(**kw).window_rows == 8 and O.DecodeCfg(**kw, n_sparse=2).window_rows == 16


@pytest.mark.parametrize("seed", range(10))
def test_verify_over_two_block_working_set_matches_brute_force(seed):
    """Impact set, A_j and C_total range over BOTH blocks of an expanded working set."""
    V, mask_id = 6, 5
    cfg = O.DecodeCfg(block_len=3, prompt_len=2, gen_len=9, tau_high=0.45, K=64, n_sparse=2)
    fn = table_fn(V, seed, spread=2.0)
    rng = np.random.default_rng(seed)
    y = np.array([1, 3] + [mask_id] * 9, dtype=np.int32)
    y[2 + int(rng.integers(0, 3))] = int(rng.integers(0, V - 1))        # 2 masks left in block 0 <= N_s
    B = list(range(2, 8))
    masked = [i for i in B if y[i] == mask_id]
    fills = [(i, w) for i in masked for w in range(V - 1)]
    st = O.State(y.copy(), O.Drafts(O.ROUTE_PLAN, fills), 0, False, ws=2)
    conf, tok = O.summaries(st, fn, cfg, 1.0, mask_id)
    _, info = O.decide(st, conf, tok, cfg, mask_id, [])
    base = {i: top1(fn(y)[i], mask_id) for i in B}
    impact = {i for i in B if y[i] == mask_id and base[i][1] >= np.float32(cfg.tau_high)}
    A, C = [], []
    for pos, w in fills:
        z = y.copy(); z[pos] = w
        lg = fn(z)
        pz = {i: top1(lg[i], mask_id) for i in B}
        A.append(int(bool(impact) and all(pz[i][0] == base[i][0] for i in impact)))
        C.append(sum(float(pz[i][1]) for i in B if z[i] == mask_id))
    J = [j for j in range(len(fills)) if A[j]]
    win = 1 + max(J, key=lambda j: (C[j], -j)) if J else 0
    assert info.accept == A and info.winner == win and sorted(info.impact) == sorted(impact)


def test_proposal_uses_expanded_set():
    """Hand-made summaries: with 1 mask left in block 0 and N_s = 1 a confident position of
    block 1 is committed in the same step, and candidates may come from block 1."""
    mask_id, bl = 9, 3
    cfg = O.DecodeCfg(block_len=bl, prompt_len=1, gen_len=9, tau_high=0.8, tau_plan_lo=0.2, tau_plan_hi=0.6,
                      tau_ar_lo=0.1, K=2, n_sparse=1)
    y = np.array([4, 1, 2, mask_id] + [mask_id] * 6, dtype=np.int32)
    conf = np.array([[0.0, 0.0, 0.3, 0.95, 0.4, 0.05, 0, 0, 0]], np.float32)
    tok = np.array([[0, 0, 7, 6, 5, 3, 0, 0, 0]], np.int32)
    new, info = O.decide(O.State(y, O.Drafts(), 0), conf, tok, cfg, mask_id, plan_set=[5])
    assert new.ws == 2 and new.k_active == 0
    assert new.y.tolist() == [4, 1, 2, mask_id, 6, mask_id, mask_id, mask_id, mask_id, mask_id]
    assert info.n_base == 1
    assert (new.drafts.route, new.drafts.fills) == (O.ROUTE_PLAN, [(5, 5)])
    cfg_off = O.DecodeCfg(block_len=bl, prompt_len=1, gen_len=9, tau_high=0.8, tau_plan_lo=0.2, tau_plan_hi=0.6,
                          tau_ar_lo=0.1, K=2, n_sparse=0)
    new, info = O.decide(O.State(y, O.Drafts(), 0), conf[:, :6], tok[:, :6], cfg_off, mask_id, plan_set=[5])
    assert new.ws == 1 and new.y.tolist()[3] == 7 and new.y.tolist()[4] == mask_id    # progress rule inside block 0
