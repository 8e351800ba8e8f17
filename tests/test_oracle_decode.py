"""Pins for the oracle's decision step and decode loop.

* brute force: on tiny canvases with a table-model denoiser every possible draft is
  enumerated and Eqs. (impact_set), (at), C_total and the AR acceptance set are evaluated
  by a second evaluator written here as direct set comprehensions;
* reductions the paper states: no drafts == confidence-threshold decoding (Sec. 2, Sec. 4),
  empty impact set rejects every planning draft (Eq. at), no accepted draft commits the
  base branch (Sec. 4.2, 4.3);
* invariants: absorbing commits, block-causal order, tau_high = 0, route switches,
  slot permutation, token accounting;
* the one-forward-per-round schedule equals Algorithm 1 taken literally.
"""
import itertools

import numpy as np
import pytest
import scipy.special

from oracle import pvf_oracle as O
from synth import inputs as S


# ----------------------------------------------------------------------------- helpers
def table_fn(V, seed, spread=3.0):
    return lambda canvas: S.table_model_logits(canvas, V, seed=seed, spread=spread)


def probs(logits_row, scale, mask_id):
    """softmax over live columns, as a dict id -> probability (library softmax)."""
    ids = [w for w in range(len(logits_row)) if w != mask_id]
    x = np.float32(scale) * np.asarray(logits_row, np.float32)[ids]
    return dict(zip(ids, scipy.special.softmax(x.astype(np.float64))))


def top1(pr):
    best = max(pr.values())
    w = min(k for k, v in pr.items() if v == best)
    return w, np.float32(pr[w])


def threshold_decode(prompt, fn, cfg, scale, mask_id):
    """Confidence-threshold blockwise decoding (Sec. 2 + App. A.1), written independently:
    commit every masked position of the first unfinished block whose top-1 probability is
    >= tau_high; if there is none, the single most confident one."""
    y = np.array(list(prompt) + [mask_id] * cfg.gen_len, dtype=np.int32)
    nfe = 0
    while (y == mask_id).any():
        first = int(np.flatnonzero(y == mask_id)[0])
        k = (first - cfg.prompt_len) // cfg.block_len
        blk = range(cfg.prompt_len + k * cfg.block_len, cfg.prompt_len + (k + 1) * cfg.block_len)
        logits = fn(y); nfe += 1
        pred = {i: top1(probs(logits[i], scale, mask_id)) for i in blk if y[i] == mask_id}
        hit = [i for i in pred if pred[i][1] >= np.float32(cfg.tau_high)]
        if not hit:
            hit = [max(pred, key=lambda i: (pred[i][1], -i))]
        for i in hit:
            y[i] = pred[i][0]
    return y, nfe


def brute_verify(y, route, fills, fn, cfg, scale, mask_id, k_active):
    """Definition-level evaluation of one verify step.  Returns (accept bits, winner)."""
    b0 = cfg.prompt_len + k_active * cfg.block_len
    B = range(b0, b0 + cfg.block_len)
    tau = np.float32(cfg.tau_high)

    def branch(extra):
        z = np.array(y).copy()
        for pos, tok in extra:
            z[pos] = tok
        return z

    z_base = branch([])
    P_base = {i: probs(fn(z_base)[i], scale, mask_id) for i in B}
    if route == O.ROUTE_PLAN:
        S_impact = {i for i in B if z_base[i] == mask_id and top1(P_base[i])[1] >= tau}
        A, C = [], []
        for f in fills:
            z = branch([f])
            Pz = {i: probs(fn(z)[i], scale, mask_id) for i in B}
            A.append(int(len(S_impact) > 0 and
                         all(top1(Pz[i])[0] == top1(P_base[i])[0] for i in S_impact)))
            C.append(sum(float(top1(Pz[i])[1]) for i in B if z[i] == mask_id))
        J = [j for j in range(len(fills)) if A[j]]
        winner = 0 if not J else 1 + max(J, key=lambda j: (C[j], -j))
        return A, winner
    else:
        ok = []
        for k in range(1, len(fills) + 1):
            z = branch(fills[:k])
            lg = fn(z)
            ok.append(int(all(top1(probs(lg[pos], scale, mask_id))[0] == tok
                              for pos, tok in fills[:k])))
        K_AR = [k for k in range(1, len(fills) + 1) if ok[k - 1]]
        return ok, (max(K_AR) if K_AR else 0)


def ref_propose(y, conf_row, tok_row, cfg, mask_id, plan, k_active):
    """Set-comprehension statement of the proposal step given one branch's (p, yhat)."""
    b0 = cfg.prompt_len + k_active * cfg.block_len
    f = np.float32
    M = [i for i in range(b0, b0 + cfg.block_len) if y[i] == mask_id]
    p = {i: f(conf_row[i - b0]) for i in M}
    t = {i: int(tok_row[i - b0]) for i in M}
    S_base = [i for i in M if p[i] >= f(cfg.tau_high)] or [max(M, key=lambda i: (p[i], -i))]
    Rm = [i for i in M if i not in S_base]
    P_plan = [i for i in Rm if t[i] in plan and f(cfg.tau_plan_lo) <= p[i] < f(cfg.tau_plan_hi)]
    ar = [i for i in Rm if p[i] >= f(cfg.tau_ar_lo)]
    if cfg.K > 0 and (cfg.routes & 1) and P_plan:
        sel = sorted(P_plan, key=lambda i: (-p[i], i))[: cfg.K]
        return S_base, O.ROUTE_PLAN, [(i, t[i]) for i in sel]
    if cfg.K > 0 and (cfg.routes & 2) and ar:
        return S_base, O.ROUTE_AR, [(i, t[i]) for i in ar[: cfg.K]]
    return S_base, O.ROUTE_NONE, []


# ----------------------------------------------------------------------------- brute force
@pytest.mark.parametrize("seed", range(12))
def test_verify_matches_brute_force_on_every_draft(seed):
    V, mask_id = 6, 5
    cfg = O.DecodeCfg(block_len=3, prompt_len=2, gen_len=6, tau_high=0.45, K=64)
    rng = np.random.default_rng(seed)
    fn = table_fn(V, seed, spread=2.0)
    y = np.array([1, 3] + [mask_id] * 6, dtype=np.int32)
    k_active = int(rng.integers(0, 2))
    if k_active == 1:
        y[2:5] = rng.integers(0, V - 1, 3)
    b0 = 2 + 3 * k_active
    if rng.random() < 0.5:                                   # sometimes one position already known
        y[b0 + int(rng.integers(0, 3))] = int(rng.integers(0, V - 1))
    masked = [i for i in range(b0, b0 + 3) if y[i] == mask_id]
    # PLAN: every (position, token) single-token draft
    fills = [(i, w) for i in masked for w in range(V - 1)]
    st = O.State(y.copy(), O.Drafts(O.ROUTE_PLAN, fills), k_active)
    conf, tok = O.summaries(st, fn, cfg, 1.0, mask_id)
    _, info = O.decide(st, conf, tok, cfg, mask_id, plan_set=[])
    A, win = brute_verify(y, O.ROUTE_PLAN, fills, fn, cfg, 1.0, mask_id, k_active)
    assert info.accept == A and info.winner == win
    want = y.copy()
    if win:
        want[fills[win - 1][0]] = fills[win - 1][1]
    assert np.array_equal(info.committed, want)
    # AR: every ordered token assignment on the leftmost masked positions
    for toks in itertools.product(range(V - 1), repeat=min(2, len(masked))):
        fills = list(zip(masked, toks))
        st = O.State(y.copy(), O.Drafts(O.ROUTE_AR, fills), k_active)
        conf, tok = O.summaries(st, fn, cfg, 1.0, mask_id)
        _, info = O.decide(st, conf, tok, cfg, mask_id, plan_set=[])
        ok, win = brute_verify(y, O.ROUTE_AR, fills, fn, cfg, 1.0, mask_id, k_active)
        assert info.accept == ok and info.winner == win
        want = y.copy()
        for pos, t in fills[:win]:
            want[pos] = t
        assert np.array_equal(info.committed, want)


def test_brute_force_sees_both_outcomes():
    """The enumeration above must exercise accepted and rejected drafts on both routes."""
    V, mask_id = 6, 5
    cfg = O.DecodeCfg(block_len=3, prompt_len=2, gen_len=6, tau_high=0.45, K=64)
    seen = {(r, a) for r in (1, 2) for a in (0, 1)}
    for seed in range(12):
        fn = table_fn(V, seed, spread=2.0)
        y = np.array([1, 3] + [mask_id] * 6, dtype=np.int32)
        fills = [(i, w) for i in (2, 3, 4) for w in range(V - 1)]
        for route, fl in ((1, fills), (2, [(2, 0), (3, 1)]), (2, [(2, 4), (3, 2)])):
            A, _ = brute_verify(y, route, fl, fn, cfg, 1.0, mask_id, 0)
            seen -= {(route, a) for a in A}
    assert not seen


@pytest.mark.parametrize("seed", range(30))
def test_decide_fuzz_against_set_comprehensions(seed):
    """Random (p, yhat) tables: verify + commit + propose against the second evaluator."""
    rng = np.random.default_rng(100 + seed)
    V, mask_id, bl = 40, 39, 8
    cfg = O.DecodeCfg(block_len=bl, prompt_len=3, gen_len=3 * bl, K=int(rng.integers(1, 5)),
                      tau_high=0.8, tau_plan_lo=0.2, tau_plan_hi=0.6, tau_ar_lo=0.3,
                      routes=int(rng.integers(0, 4)))
    plan = set(rng.choice(V - 1, 12, replace=False).tolist())
    k_active = int(rng.integers(0, 3))
    y = np.full(cfg.T, mask_id, np.int32)
    y[:3 + k_active * bl] = rng.integers(0, V - 1, 3 + k_active * bl)
    b0 = 3 + k_active * bl
    keep = rng.random(bl) < 0.7
    keep[int(rng.integers(0, bl))] = True                     # at least one mask in the block
    y[b0:b0 + bl][~keep] = rng.integers(0, V - 1, int((~keep).sum()))
    masked = [i for i in range(b0, b0 + bl) if y[i] == mask_id]
    route = int(rng.integers(0, 3))
    n = int(rng.integers(0, min(cfg.K, len(masked)) + 1)) if route else 0
    pos = sorted(rng.choice(masked, n, replace=False).tolist())
    fills = [(p, int(rng.integers(0, V - 1))) for p in pos]
    R = cfg.window_rows
    conf = rng.choice(np.array([.05, .15, .25, .35, .5, .7, .85, .95], np.float32), (1 + n, R))
    tok = rng.integers(0, V - 1, (1 + n, R)).astype(np.int32)
    if n and rng.random() < 0.7:                               # make acceptance likely
        tok[1:] = tok[0]
        for k, (p, t) in enumerate(fills):
            tok[k + 1:, p - b0] = t
    st = O.State(y.copy(), O.Drafts(route if n else 0, fills), k_active)
    new, info = O.decide(st, conf, tok, cfg, mask_id, plan)

    # -- second evaluator: verify
    X = [y.copy() for _ in range(1 + n)]
    for j in range(1, n + 1):
        for p, t in ([fills[j - 1]] if route == 1 else fills[:j]):
            X[j][p] = t
    B = range(b0, b0 + bl)
    if n and route == 1:
        imp = {i for i in B if y[i] == mask_id and conf[0, i - b0] >= np.float32(cfg.tau_high)}
        A = [int(bool(imp) and all(tok[j, i - b0] == tok[0, i - b0] for i in imp))
             for j in range(1, n + 1)]
        C = [sum(float(conf[j, i - b0]) for i in B if X[j][i] == mask_id) for j in range(1, n + 1)]
        J = [j for j in range(n) if A[j]]
        win = 1 + max(J, key=lambda j: (C[j], -j)) if J else 0
    elif n:
        A = [int(all(tok[k, p - b0] == t for p, t in fills[:k])) for k in range(1, n + 1)]
        win = max([k for k in range(1, n + 1) if A[k - 1]], default=0)
    else:
        A, win = [], 0
    assert info.accept == A and info.winner == win
    yc = X[win]
    assert np.array_equal(info.committed, yc)
    assert (info.n_plan, info.n_ar) == ((1, 0) if (win and route == 1) else (0, win if route == 2 else 0))
    # -- second evaluator: propose
    if not (yc[3:] == mask_id).any():
        assert new.done
        return
    k_new = k_active if (yc[b0:b0 + bl] == mask_id).any() else k_active + 1
    off = (k_new - k_active) * bl
    S_base, r2, f2 = ref_propose(yc, conf[win, off:], tok[win, off:], cfg, mask_id, plan, k_new)
    want = yc.copy()
    for i in S_base:
        want[i] = tok[win, i - b0]
    assert np.array_equal(new.y, want) and info.n_base == len(S_base)
    assert new.k_active == k_new
    if not (want[3:] == mask_id).any():
        assert new.done and new.drafts.n == 0
    else:
        assert not new.done
        assert (new.drafts.route if new.drafts.n else 0, new.drafts.fills) == (r2, f2)


# ----------------------------------------------------------------------------- reductions
CFG = dict(block_len=4, prompt_len=3, gen_len=12)


@pytest.mark.parametrize("seed", range(6))
def test_no_drafts_is_threshold_decoding(seed):
    V, mask_id = 12, 11
    fn = table_fn(V, seed)
    prompt = [1, 2, 3]
    for kw in (dict(K=0), dict(K=3, routes=0), dict(K=3, routes=2, tau_ar_lo=1.5)):
        cfg = O.DecodeCfg(**CFG, tau_high=0.6, tau_plan_lo=0.2, tau_plan_hi=0.5, **kw)
        res = O.decode(prompt, fn, cfg, 1.0, mask_id, plan_set=[])
        y, nfe = threshold_decode(prompt, fn, cfg, 1.0, mask_id)
        assert np.array_equal(res.tokens, y) and res.nfe == nfe
        assert res.n_plan == 0 and res.n_ar == 0 and res.n_base == cfg.gen_len


@pytest.mark.parametrize("seed", range(4))
def test_tau_high_zero_commits_whole_block_each_round(seed):
    V, mask_id = 12, 11
    cfg = O.DecodeCfg(**CFG, tau_high=0.0, tau_plan_lo=0.0, tau_plan_hi=0.0, K=2)
    res = O.decode([1, 2, 3], table_fn(V, seed), cfg, 1.0, mask_id, plan_set=range(11))
    assert res.nfe == cfg.n_blocks
    assert [r.n_base for r in res.rounds] == [cfg.block_len] * cfg.n_blocks


@pytest.mark.parametrize("seed", range(8))
def test_invariants_over_full_decodes(seed):
    V, mask_id = 16, 15
    rng = np.random.default_rng(seed)
    cfg = O.DecodeCfg(block_len=4, prompt_len=3, gen_len=16, tau_high=0.7, tau_plan_lo=0.15,
                      tau_plan_hi=0.6, tau_ar_lo=0.2, K=3)
    plan = sorted(rng.choice(V - 1, 6, replace=False).tolist())
    prompt = [4, 5, 6]
    res = O.decode(prompt, table_fn(V, seed, spread=2.5), cfg, 1.0, mask_id, plan)
    assert not (res.tokens == mask_id).any()
    assert list(res.tokens[:3]) == prompt
    # token accounting: every generated token is committed exactly once, by one route
    assert res.n_base + res.n_plan + res.n_ar == cfg.gen_len
    prev = np.array(prompt + [mask_id] * cfg.gen_len)
    for y, info in zip(res.canvases + [res.tokens], res.rounds + [None]):
        known = prev != mask_id
        assert np.array_equal(y[known], prev[known])          # absorbing: commits never change
        m = np.flatnonzero(y == mask_id)
        if len(m):                                            # block-causal: nothing beyond the
            k = (m[0] - 3) // 4                               # first unfinished block is touched
            assert (y[3 + (k + 1) * 4:] == mask_id).all()
        if info is not None:
            if info.route == O.ROUTE_PLAN and not info.impact:
                assert info.winner == 0 and not any(info.accept)   # Eq. (at): empty impact set
        prev = y
    routes = {r.route for r in res.rounds}
    assert routes <= {0, 1, 2}


def test_winner_contains_base_branch_and_route_switch():
    V, mask_id = 16, 15
    cfg = O.DecodeCfg(block_len=4, prompt_len=3, gen_len=16, tau_high=0.7, tau_plan_lo=0.15,
                      tau_plan_hi=0.6, tau_ar_lo=0.2, K=3)
    saw = {"plan_acc": 0, "ar_acc": 0, "rej": 0}
    for seed in range(10):
        fn = table_fn(V, seed, spread=2.5)
        # empty planning vocabulary -> only AR drafts ever appear
        res = O.decode([4, 5, 6], fn, cfg, 1.0, mask_id, plan_set=[])
        assert all(r.route in (0, 2) for r in res.rounds) and res.n_plan == 0
        # planning vocabulary = every id -> AR only when no candidate lies in the band
        res = O.decode([4, 5, 6], fn, cfg, 1.0, mask_id, plan_set=range(V - 1))
        st = O.initial_state([4, 5, 6], cfg, mask_id)
        while not st.done:
            X = O.branch_canvases(st.y, st.drafts)
            new, info = O.pvf_round(st, fn, cfg, 1.0, mask_id, range(V - 1))
            base = X[0] != mask_id
            assert np.array_equal(info.committed[base], X[0][base])     # winner contains z_base
            saw["plan_acc"] += info.route == 1 and info.winner > 0
            saw["ar_acc"] += info.route == 2 and info.winner > 0
            saw["rej"] += info.route != 0 and info.winner == 0
            st = new
    assert all(v > 0 for v in saw.values()), saw


@pytest.mark.parametrize("seed", range(6))
def test_permuting_plan_slots_permutes_bits_only(seed):
    V, mask_id = 10, 9
    cfg = O.DecodeCfg(block_len=4, prompt_len=2, gen_len=8, tau_high=0.4, K=8)
    fn = table_fn(V, seed, spread=2.0)
    y = np.array([1, 2] + [mask_id] * 8, np.int32)
    fills = [(2, 3), (3, 1), (4, 7), (5, 0)]
    perm = np.random.default_rng(seed).permutation(4)
    out = []
    for fl in (fills, [fills[i] for i in perm]):
        st = O.State(y.copy(), O.Drafts(O.ROUTE_PLAN, fl), 0)
        out.append(O.pvf_round(st, fn, cfg, 1.0, mask_id, [])[1])
    a, b = out
    assert [a.accept[i] for i in perm] == b.accept
    assert np.array_equal(a.committed, b.committed)            # C_total ties are measure-zero here


# ----------------------------------------------------------------------------- schedule
def _same_trajectory(res, lit_tokens, lit_trail):
    got = [c for c in res.canvases[1:]]
    if not got or not np.array_equal(got[-1], res.tokens):
        got.append(res.tokens)
    assert np.array_equal(res.tokens, lit_tokens)
    assert len(got) == len(lit_trail)
    for a, b in zip(got, lit_trail):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("seed", range(8))
def test_one_forward_per_round_equals_literal_algorithm(seed):
    V, mask_id = 16, 15
    cfg = O.DecodeCfg(block_len=4, prompt_len=3, gen_len=16, tau_high=0.7, tau_plan_lo=0.15,
                      tau_plan_hi=0.6, tau_ar_lo=0.2, K=3)
    plan = sorted(np.random.default_rng(seed).choice(V - 1, 7, replace=False).tolist())
    fn = table_fn(V, seed, spread=2.5)
    res = O.decode([4, 5, 6], fn, cfg, 1.0, mask_id, plan)
    y, nfe, trail = O.decode_literal([4, 5, 6], fn, cfg, 1.0, mask_id, plan)
    _same_trajectory(res, y, trail)
    assert res.nfe <= nfe <= 2 * res.nfe


def test_schedules_agree_on_the_tiny_transformer():
    shape = S.TINY
    mc = O.ModelCfg(shape.n_layers, shape.d_model, shape.n_heads, shape.d_ff, shape.vocab,
                    shape.mask_id, shape.rms_eps, shape.rope_theta, shape.logit_scale)
    w = S.make_weights(shape, seed=0)
    cfg = O.DecodeCfg(block_len=8, prompt_len=16, gen_len=16, K=2)
    prompt = S.make_prompt(1, 16, shape.vocab, shape.mask_id)
    plan = S.make_plan_vocab(2, 64, shape.vocab, shape.mask_id)
    cache = {}

    def fn(canvas):
        key = bytes(np.asarray(canvas, np.int32))
        if key not in cache:
            cache[key] = O.forward(canvas, w, mc)
        return cache[key]

    res = O.decode(prompt, fn, cfg, shape.logit_scale, shape.mask_id, plan)
    y, nfe, trail = O.decode_literal(prompt, fn, cfg, shape.logit_scale, shape.mask_id, plan)
    _same_trajectory(res, y, trail)
    assert res.n_base + res.n_plan + res.n_ar == cfg.gen_len
