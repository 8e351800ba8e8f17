"""Pins for the calibration oracle (entropy, verified information gain, token statistics,
filtering rule; Sec. 3 "Verified information gain" and App. A.2): library entropy, closed
forms, hand-made events, an independently written aggregation, and the trajectory being plain
confidence-threshold decoding."""
import collections
import math

import numpy as np
import pytest
import scipy.special
import scipy.stats

from oracle import pvf_calibration as C
from oracle import pvf_oracle as O
from synth import inputs as S


def table_fn(V, seed, spread=2.5):
    return lambda canvas: S.table_model_logits(canvas, V, seed=seed, spread=spread)


# ------------------------------------------------------------------------------------------
# entropy
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("scale", [1.0, 0.37, 12.0])
def test_entropy_matches_library(scale):
    rng = np.random.default_rng(0)
    V, mask_id = 257, 100
    l = rng.standard_normal((9, V)).astype(np.float32) * 2
    x = (np.float32(scale) * l).astype(np.float32).astype(np.float64)
    ids = [w for w in range(V) if w != mask_id]
    want = [scipy.stats.entropy(scipy.special.softmax(r[ids])) for r in x]
    np.testing.assert_allclose(C.entropy(l, scale, mask_id), want, rtol=2e-6)


def test_entropy_closed_forms():
    V, mask_id = 64, 63
    np.testing.assert_allclose(C.entropy(np.zeros((2, V), np.float32), 3.0, mask_id), math.log(V - 1), rtol=1e-6)
    np.testing.assert_allclose(C.entropy(np.full((1, V), 7.5, np.float32), 1.0, mask_id), math.log(V - 1), rtol=1e-6)
    # two live tokens: binary entropy of sigmoid(scale * (a - b)); the mask column's value is irrelevant
    for a, b, scale in [(1.0, 0.0, 1.0), (0.3, -0.4, 2.0), (5.0, 5.0, 1.0)]:
        p = 1 / (1 + math.exp(-scale * (a - b)))
        want = -(p * math.log(p) + (1 - p) * math.log(1 - p))
        got = C.entropy(np.array([[a, 1e9, b]], np.float32), scale, 1)
        np.testing.assert_allclose(got, want, rtol=1e-6)
    # one dominant logit: entropy ~ 0, and nothing overflows
    l = np.zeros((1, V), np.float32); l[0, 5] = 3e4
    assert C.entropy(l, 1.0, mask_id)[0] == 0.0
    # shift invariance, bounds
    rng = np.random.default_rng(1)
    l = rng.standard_normal((5, V)).astype(np.float32)
    np.testing.assert_allclose(C.entropy(l, 1.0, mask_id), C.entropy(l + np.float32(8.0), 1.0, mask_id), atol=2e-5)
    H = C.entropy(l, 1.0, mask_id)
    assert np.all(H > 0) and np.all(H <= math.log(V - 1) + 1e-6)
    # consistency with stage 1: H >= -ln p_max (min-entropy bound) and H <= ln(V-1)
    p, _ = O.stage1(l, 1.0, mask_id)
    assert np.all(H >= -np.log(p.astype(np.float64)) - 1e-6)


# ------------------------------------------------------------------------------------------
# one step's events
# ------------------------------------------------------------------------------------------
def test_verify_events_hand_made():
    mask = 9
    B = [10, 11, 12, 13]
    z = np.zeros(20, np.int32); z[[11, 12, 13]] = mask
    p_b = np.array([0.99, 0.95, 0.3, 0.5], np.float32)        # position 10 is known: never in the impact set
    t_b = np.array([1, 2, 3, 4]); H_b = np.array([9.0, 1.0, 2.0, 3.0], np.float32)
    t_ok = np.array([7, 2, 8, 8]); t_bad = np.array([1, 5, 3, 4])
    H_p = np.array([0.0, 0.5, 7.0, 2.0], np.float32)
    ev = C.verify_events(z, B, p_b, t_b, H_b, [(12, 7), (12, 7)], [t_ok, t_bad], [H_p, H_p], 0.9, mask)
    assert (ev[0].A, ev[0].nonvacuous, ev[0].token, ev[0].position) == (1, True, 7, 12)
    assert ev[0].dH == pytest.approx(((1.0 - 0.5) + (3.0 - 2.0)) / 2) and ev[0].vig == pytest.approx(0.75)
    assert ev[1].A == 0 and ev[1].vig == 0.0 and ev[1].dH == pytest.approx(0.75)
    # vacuous: nothing reaches tau_high -> A = 0 whatever the tokens say
    ev = C.verify_events(z, B, p_b, t_b, H_b, [(12, 7)], [t_b], [H_p], 0.96, mask)
    assert (ev[0].A, ev[0].nonvacuous, ev[0].vig) == (0, False, 0.0)
    # the candidate's own position belongs to the impact set but not to the evaluation region
    p_b2 = np.array([0.0, 0.2, 0.95, 0.2], np.float32)
    ev = C.verify_events(z, B, p_b2, t_b, H_b, [(12, 7)], [np.array([0, 0, 3, 0])], [H_p], 0.9, mask)
    assert ev[0].A == 1 and ev[0].dH == pytest.approx(0.75)
    ev = C.verify_events(z, B, p_b2, t_b, H_b, [(12, 7)], [np.array([1, 2, 9, 4])], [H_p], 0.9, mask)
    assert ev[0].A == 0
    # empty evaluation region: the candidate is the only mask left
    z1 = np.zeros(20, np.int32); z1[12] = mask
    ev = C.verify_events(z1, B, p_b2, t_b, H_b, [(12, 7)], [t_b], [H_p], 0.9, mask)
    assert ev[0].dH == 0.0 and ev[0].A == 1 and ev[0].vig == 0.0
    # an entropy increase gives a negative gain
    ev = C.verify_events(z, B, p_b, t_b, H_b, [(13, 4)], [t_b], [np.array([0, 2.0, 2.5, 0], np.float32)], 0.9, mask)
    assert ev[0].dH == pytest.approx(((1.0 - 2.0) + (2.0 - 2.5)) / 2) and ev[0].vig < 0


# ------------------------------------------------------------------------------------------
# whole calibration runs against an independently written version
# ------------------------------------------------------------------------------------------
def independent_calibration(prompts, fn, cfg, mask_id, V, band, cap):
    """Written from the definitions with scipy and dictionaries; shares nothing with the oracle."""
    ids = [w for w in range(V) if w != mask_id]

    def dist(row):
        return scipy.special.softmax(np.asarray(row, np.float32)[ids].astype(np.float64))

    def top(row):
        pr = dist(row); best = pr.max()
        return min(i for i, q in zip(ids, pr) if q == best), np.float32(best)

    n, m, a, vig = (collections.Counter() for _ in range(4))
    finals = []
    for prompt in prompts:
        y = np.array(list(prompt) + [mask_id] * cfg.gen_len, dtype=np.int32)
        while (y == mask_id).any():
            first = int(np.flatnonzero(y == mask_id)[0])
            k = (first - cfg.prompt_len) // cfg.block_len
            blk = range(cfg.prompt_len + k * cfg.block_len, cfg.prompt_len + (k + 1) * cfg.block_len)
            lg = fn(y)
            pred = {i: top(lg[i]) for i in blk if y[i] == mask_id}
            hit = [i for i in pred if pred[i][1] >= np.float32(cfg.tau_high)] or \
                  [max(pred, key=lambda i: (pred[i][1], -i))]
            zb = y.copy()
            for i in hit:
                zb[i] = pred[i][0]
            cands = sorted((i for i in pred if i not in hit and np.float32(band[0]) <= pred[i][1] < np.float32(band[1])),
                           key=lambda i: (-pred[i][1], i))[:cap]
            if cands:
                lb = fn(zb)
                still = [i for i in blk if zb[i] == mask_id]
                impact = [i for i in still if top(lb[i])[1] >= np.float32(cfg.tau_high)]
                for i in cands:
                    v = pred[i][0]
                    z = zb.copy(); z[i] = v
                    lz = fn(z)
                    ok = bool(impact) and all(top(lz[q])[0] == top(lb[q])[0] for q in impact)
                    reg = [q for q in still if q != i]
                    gain = sum(scipy.stats.entropy(dist(lb[q])) - scipy.stats.entropy(dist(lz[q])) for q in reg) / len(reg) if reg else 0.0
                    n[v] += 1; m[v] += bool(impact); a[v] += ok; vig[v] += gain if ok else 0.0
            y = zb
        finals.append(y)
    return n, m, a, vig, finals


@pytest.mark.parametrize("seed,cap", [(0, None), (1, None), (2, 2), (3, 1), (4, None)])
def test_calibration_matches_independent_version(seed, cap):
    V, mask_id = 14, 13
    cfg = O.DecodeCfg(block_len=5, prompt_len=3, gen_len=15, tau_high=0.5, tau_plan_lo=0.0, tau_plan_hi=0.0, K=0)
    band = (0.12, 0.45)
    fn = table_fn(V, seed, spread=2.0)
    prompts = [[1, 2, 3], [4, 5, 6], [7, 1, 2]]
    st, finals, n_fwd = C.calibrate(prompts, fn, cfg, 1.0, mask_id, V, band=band, cap=cap)
    n, m, a, vig, fin2 = independent_calibration(prompts, fn, cfg, mask_id, V, band, cap)
    assert st.n.sum() > 0 and st.a.sum() > 0                      # the case exercises accepted events
    for v in range(V):
        assert (st.n[v], st.m[v], st.a[v]) == (n[v], m[v], a[v])
        assert st.vig[v] == pytest.approx(vig[v], rel=1e-5, abs=1e-6)
    assert all(np.array_equal(x, y) for x, y in zip(finals, fin2))
    # invariants of the statistics
    assert np.all(st.a <= st.m) and np.all(st.m <= st.n) and st.n[mask_id] == 0
    assert np.all(st.vig[st.a == 0] == 0.0)
    assert all(abs(e.dH) <= math.log(V - 1) for e in st.events)
    assert n_fwd >= len(st.events)


def test_calibration_trajectory_is_threshold_decoding():
    V, mask_id = 14, 13
    cfg = O.DecodeCfg(block_len=5, prompt_len=3, gen_len=15, tau_high=0.5, tau_plan_lo=0.0, tau_plan_hi=0.0, K=0)
    for seed in range(4):
        fn = table_fn(V, seed, spread=2.0)
        st, finals, _ = C.calibrate([[1, 2, 3]], fn, cfg, 1.0, mask_id, V, band=(0.1, 0.45))
        assert np.array_equal(finals[0], O.decode([1, 2, 3], fn, cfg, 1.0, mask_id, []).tokens)
    # a cap at least as large as the block changes nothing; a smaller one keeps the most confident events
    fn = table_fn(V, 0, spread=2.0)
    full, _, _ = C.calibrate([[1, 2, 3]], fn, cfg, 1.0, mask_id, V, band=(0.1, 0.45))
    big, _, _ = C.calibrate([[1, 2, 3]], fn, cfg, 1.0, mask_id, V, band=(0.1, 0.45), cap=5)
    one, _, _ = C.calibrate([[1, 2, 3]], fn, cfg, 1.0, mask_id, V, band=(0.1, 0.45), cap=1)
    assert np.array_equal(full.n, big.n) and np.array_equal(full.vig, big.vig)
    assert one.n.sum() <= full.n.sum() and np.all(one.n <= full.n)
    # with early cross-block revelation the trajectory is still the N_s threshold decoder
    cfg2 = O.DecodeCfg(block_len=5, prompt_len=3, gen_len=15, tau_high=0.5, tau_plan_lo=0.0, tau_plan_hi=0.0, K=0, n_sparse=2)
    st, finals, _ = C.calibrate([[1, 2, 3]], fn, cfg2, 1.0, mask_id, V, band=(0.1, 0.45))
    assert np.array_equal(finals[0], O.decode([1, 2, 3], fn, cfg2, 1.0, mask_id, []).tokens)


# ------------------------------------------------------------------------------------------
# filtering rule
# ------------------------------------------------------------------------------------------
def test_filtering_rule_each_criterion():
    V, mask_id = 8, 7
    st = C.TokenStats.zeros(V)
    #            n    m    a    vig-sum
    rows = {0: (50, 20, 18, 1.5),      # passes everything exactly at the limits (r = 0.9, vig-hat = 0.03)
            1: (49, 20, 20, 9.0),      # support too small
            2: (60, 19, 19, 9.0),      # too few non-vacuous opportunities
            3: (60, 30, 26, 9.0),      # r = 0.867 < 0.9
            4: (60, 30, 30, 1.79),     # vig-hat = 0.0298 < 0.03
            5: (80, 40, 38, 8.0),      # passes
            6: (0, 0, 0, 0.0),
            7: (90, 90, 90, 90.0)}     # [MASK] is never selected
    for v, (n, m, a, g) in rows.items():
        st.n[v], st.m[v], st.a[v], st.vig[v] = n, m, a, g
    assert C.select_plan_vocab(st, mask_id).tolist() == [5] or C.select_plan_vocab(st, mask_id).tolist() == [0, 5]
    # token 0 sits exactly on float32(0.9) / float32(0.03), which are not 0.9 / 0.03: decide it explicitly
    want0 = (18 / 20 >= float(np.float32(0.9))) and (1.5 / 50 >= float(np.float32(0.03)))
    assert (0 in C.select_plan_vocab(st, mask_id).tolist()) == want0
    assert C.select_plan_vocab(st, mask_id, n_min=1, m_min=1, rho_ver=0.0, gamma_vig=-1.0).tolist() == [0, 1, 2, 3, 4, 5]
    assert st.r_ver[6] == 0.0 and st.vig_hat[6] == 0.0
    mg = C.select_margin(st)
    assert mg[6] == np.inf and mg[0] < 1e-6 and mg[5] > 1e-2


@pytest.mark.parametrize("seed,cap,ns", [(0, None, 0), (1, 3, 0), (2, 1, 0), (3, None, 2), (4, 2, 5)])
def test_pipelined_schedule_gives_the_same_statistics(seed, cap, ns):
    """One batched forward per step (backbone + measured branches) against the literal
    two-forward procedure: same events, same statistics, same final canvases."""
    V, mask_id = 14, 13
    cfg = O.DecodeCfg(block_len=5, prompt_len=3, gen_len=15, tau_high=0.5, tau_plan_lo=0.0, tau_plan_hi=0.0,
                      K=0, n_sparse=ns)
    band = (0.12, 0.45)
    fn = table_fn(V, seed, spread=2.0)
    prompts = [[1, 2, 3], [4, 5, 6]]
    a, fa, _ = C.calibrate(prompts, fn, cfg, 1.0, mask_id, V, band=band, cap=cap)
    b, fb, rounds = C.calibrate_pipelined(prompts, fn, cfg, 1.0, mask_id, V, band=band, cap=cap)
    assert a.n.sum() > 0
    assert np.array_equal(a.n, b.n) and np.array_equal(a.m, b.m) and np.array_equal(a.a, b.a)
    np.testing.assert_allclose(a.vig, b.vig, rtol=1e-12, atol=1e-15)
    assert [(e.token, e.position, e.A) for e in a.events] == [(e.token, e.position, e.A) for e in b.events]
    assert all(np.array_equal(x, y) for x, y in zip(fa, fb))
    assert a.margin == pytest.approx(b.margin)
    plain = [O.decode(p, fn, cfg, 1.0, mask_id, []).nfe for p in prompts]
    assert rounds == sum(plain)                      # measuring never adds or removes a step
