"""Pins for the K/V-cache oracle (oracle/pvf_kvcache.py): the full forward it carries equals
the plain oracle forward; the window forward equals it on the cached canvas, equals an
independently written per-query loop on any canvas, and really is stale outside the window;
decoding with a refresh in every round is plain PVF decoding."""
import math

import numpy as np
import pytest

from oracle import pvf_kvcache as KV
from oracle import pvf_oracle as O
from synth import inputs as S

SHAPE = S.ModelShape(n_layers=2, d_model=32, n_heads=2, d_ff=48, vocab=41, mask_id=40, rope_theta=100.0,
                     logit_scale=30.0)


def model(seed=0, std=0.3):
    w = S.make_weights(SHAPE, seed=seed, std=std)
    cfg = O.ModelCfg(SHAPE.n_layers, SHAPE.d_model, SHAPE.n_heads, SHAPE.d_ff, SHAPE.vocab, SHAPE.mask_id,
                     SHAPE.rms_eps, SHAPE.rope_theta, SHAPE.logit_scale)
    return w, cfg


def canvas(seed, T, n_mask):
    x = S.make_prompt(seed, T, SHAPE.vocab, SHAPE.mask_id).astype(np.int32)
    x[T - n_mask:] = SHAPE.mask_id
    return x


def test_full_forward_equals_plain_oracle_forward():
    w, cfg = model()
    x = canvas(1, 24, 10)
    lg, cache = KV.forward_full(x, w, cfg)
    np.testing.assert_allclose(lg, O.forward(x, w, cfg), rtol=0, atol=1e-6)
    assert len(cache.k) == cfg.n_layers and cache.k[0].shape == (24, cfg.n_heads, cfg.d_model // cfg.n_heads)


@pytest.mark.parametrize("window", [range(8, 16), range(0, 5), range(17, 24), [3, 4, 11, 12, 20]])
def test_window_forward_is_exact_on_the_cached_canvas(window):
    w, cfg = model(seed=2)
    x = canvas(3, 24, 12)
    full, cache = KV.forward_full(x, w, cfg)
    got = KV.forward_window(x, list(window), cache, w, cfg)
    np.testing.assert_allclose(got, full[list(window)], rtol=0, atol=2e-6)


def loop_window_forward(x_new, x_old, window, w, cfg):
    """Per-query, per-head, per-key loops written from the definition: positions outside the
    window keep, in every layer, the keys / values they had in the full forward of x_old."""
    d, H = cfg.d_model, cfg.n_heads
    dh, half = d // H, d // H // 2
    T = len(x_old)

    def norm(v, g):
        return v / math.sqrt(float(np.mean(v * v)) + cfg.rms_eps) * g

    def rot(vec, p):
        out = vec.copy()
        for hh in range(H):
            for i in range(half):
                ang = p * cfg.rope_theta ** (-2.0 * i / dh)
                a, b = vec[hh * dh + i], vec[hh * dh + i + half]
                out[hh * dh + i] = a * math.cos(ang) - b * math.sin(ang)
                out[hh * dh + i + half] = b * math.cos(ang) + a * math.sin(ang)
        return out

    def layer_qkv(hrow, p, lw):
        qkv = lw["wqkv"].astype(np.float64) @ norm(hrow, lw["attn_norm"].astype(np.float64))
        return rot(qkv[:d], p), rot(qkv[d:2 * d], p), qkv[2 * d:]

    # full forward of the old canvas, keeping every layer's keys and values
    h_old = [w["embed"][t].astype(np.float64) for t in x_old]
    h_new = {p: w["embed"][x_new[p]].astype(np.float64) for p in window}
    for lw in w["layers"]:
        old = [layer_qkv(h_old[p], p, lw) for p in range(T)]
        new = {p: layer_qkv(h_new[p], p, lw) for p in window}

        def attend(q, keys, vals):
            o = np.zeros(d)
            for hh in range(H):
                sl = slice(hh * dh, (hh + 1) * dh)
                sc = np.array([q[sl] @ keys[t][sl] / math.sqrt(dh) for t in range(T)])
                pr = np.exp(sc - sc.max()); pr /= pr.sum()
                o[sl] = sum(pr[t] * vals[t][sl] for t in range(T))
            return o

        def rest(hrow, o):
            hrow = hrow + lw["wo"].astype(np.float64) @ o
            f = norm(hrow, lw["ffn_norm"].astype(np.float64))
            gu = lw["w_gate_up"].astype(np.float64) @ f
            g, u = gu[: cfg.d_ff], gu[cfg.d_ff:]
            return hrow + lw["w_down"].astype(np.float64) @ (g / (1 + np.exp(-g)) * u)

        keys_o, vals_o = [o_[1] for o_ in old], [o_[2] for o_ in old]
        keys_n = [new[p][1] if p in new else keys_o[p] for p in range(T)]
        vals_n = [new[p][2] if p in new else vals_o[p] for p in range(T)]
        h_new = {p: rest(h_new[p], attend(new[p][0], keys_n, vals_n)) for p in window}
        h_old = [rest(h_old[p], attend(old[p][0], keys_o, vals_o)) for p in range(T)]
    out = []
    for p in window:
        out.append(w["out_head"].astype(np.float64) @ norm(h_new[p], w["final_norm"].astype(np.float64)))
    return np.array(out)


def test_window_forward_matches_loop_definition_and_is_stale_outside():
    w, cfg = model(seed=4)
    x_old = canvas(5, 14, 8)
    x_new = x_old.copy()
    window = [6, 7, 8, 9]
    x_new[7], x_new[9] = 3, 17                    # committed inside the window since the refresh
    _, cache = KV.forward_full(x_old, w, cfg)
    got = KV.forward_window(x_new, window, cache, w, cfg)
    np.testing.assert_allclose(got, loop_window_forward(x_new, x_old, window, w, cfg), rtol=0, atol=5e-6)
    exact = O.forward(x_new, w, cfg)[window]
    assert np.abs(got - exact).max() > 1e-4        # an approximation: the other rows did not see the commits
    # a change OUTSIDE the window is invisible to the window forward (it reads the cache there)
    x_far = x_new.copy(); x_far[1] = 9
    np.testing.assert_array_equal(KV.forward_window(x_far, window, cache, w, cfg), got)


@pytest.mark.parametrize("seed", range(3))
def test_refresh_every_round_is_plain_decoding(seed):
    """With a refresh in every round the backbone always gets the exact forward: without drafts
    that is plain threshold decoding; with drafts the backbone's own summaries are still exact
    (the drafts, forwarded against the cache, are the only approximation)."""
    w, cfg = model(seed=10 + seed)
    plan = list(range(0, 40, 3))
    prompt = S.make_prompt(seed, 6, SHAPE.vocab, SHAPE.mask_id)
    fn = lambda c: O.forward(c, w, cfg)
    d0 = O.DecodeCfg(block_len=4, prompt_len=6, gen_len=12, tau_high=0.6, tau_plan_lo=0.1, tau_plan_hi=0.5, K=0)
    plain = O.decode(prompt, fn, d0, SHAPE.logit_scale, SHAPE.mask_id, plan)
    forced = KV.decode_cached(prompt, w, cfg, d0, SHAPE.logit_scale, SHAPE.mask_id, plan, force_refresh=True)
    assert np.array_equal(forced.tokens, plain.tokens) and forced.nfe == plain.nfe == forced.n_refresh
    d2 = O.DecodeCfg(block_len=4, prompt_len=6, gen_len=12, tau_high=0.6, tau_plan_lo=0.1, tau_plan_hi=0.5,
                     tau_ar_lo=0.2, K=2)
    st, cache = O.initial_state(prompt, d2, SHAPE.mask_id), None
    for _ in range(4):
        if st.done:
            break
        conf, tok, cache, refreshed = KV.cached_summaries(st, cache, w, cfg, d2, SHAPE.logit_scale, SHAPE.mask_id, True)
        exact_c, exact_t = O.summaries(st, fn, d2, SHAPE.logit_scale, SHAPE.mask_id)
        assert refreshed and np.array_equal(tok[0], exact_t[0])
        np.testing.assert_allclose(conf[0], exact_c[0], rtol=1e-5)
        # a draft is forwarded on its window rows against the backbone's fresh cache
        if st.drafts.n:
            X = O.branch_canvases(st.y, st.drafts)
            wp = O.window_positions(d2, st.k_active); ok = wp < d2.T
            lg = KV.forward_window(X[1], wp[ok], cache, w, cfg)
            c1, t1 = O.stage1(lg, SHAPE.logit_scale, SHAPE.mask_id)
            assert np.array_equal(tok[1][ok], t1) and np.array_equal(conf[1][ok], c1)
        st, _ = O.decide(st, conf, tok, d2, SHAPE.mask_id, plan)


@pytest.mark.parametrize("seed,ns", [(0, 0), (1, 0), (2, 2)])
def test_cached_decoding_invariants(seed, ns):
    w, cfg = model(seed=20 + seed)
    dcfg = O.DecodeCfg(block_len=4, prompt_len=6, gen_len=16, tau_high=0.6, tau_plan_lo=0.1, tau_plan_hi=0.5,
                       tau_ar_lo=0.2, K=3, n_sparse=ns)
    prompt = S.make_prompt(seed, 6, SHAPE.vocab, SHAPE.mask_id)
    res = KV.decode_cached(prompt, w, cfg, dcfg, SHAPE.logit_scale, SHAPE.mask_id, list(range(0, 40, 2)))
    assert not np.any(res.tokens == SHAPE.mask_id) and np.array_equal(res.tokens[:6], prompt)
    assert sum(r.n_base + r.n_plan + r.n_ar for r in res.rounds) == dcfg.gen_len
    # one refresh per distinct active block that a round started in, never more than the block count
    blocks = [0] + [s.k_active for s in res.states[:-1]]
    assert res.n_refresh == len(set(blocks)) <= dcfg.n_blocks and res.n_refresh < res.nfe
    # committed tokens never change afterwards
    prev = np.array(list(prompt) + [SHAPE.mask_id] * dcfg.gen_len)
    for s in res.states:
        keep = prev != SHAPE.mask_id
        assert np.array_equal(s.y[keep], prev[keep])
        prev = s.y
    # the first round is a refresh, hence identical to plain decoding's first round
    fn = lambda c: O.forward(c, w, cfg)
    st0 = O.initial_state(prompt, dcfg, SHAPE.mask_id)
    first, _ = O.pvf_round(st0, fn, dcfg, SHAPE.logit_scale, SHAPE.mask_id, list(range(0, 40, 2)))
    assert np.array_equal(first.y, res.states[0].y)
