"""Pins for the Random / Planning single-extra-commit oracle (App. A.3.1)."""
import collections

import numpy as np
import pytest

from oracle import pvf_ablation as A
from oracle import pvf_oracle as O
from synth import inputs as S


def table_fn(V, seed, spread=2.5):
    return lambda canvas: S.table_model_logits(canvas, V, seed=seed, spread=spread)


def test_generator_matches_published_splitmix64_vector():
    # first outputs of SplitMix64 seeded with 0 (the vector quoted with the reference implementation)
    g = 0x9E3779B97F4A7C15
    want = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F, 0xF88BB8A8724C81EC]
    assert [A.splitmix64((i * g) & ((1 << 64) - 1)) for i in range(4)] == want
    assert A.draw(0, 0, 0) == want[0]
    assert len({A.draw(s, g_, n) for s in range(3) for g_ in range(3) for n in range(50)}) == 450


def test_empty_bin_is_threshold_decoding():
    V, mask_id = 16, 15
    for seed in range(4):
        fn = table_fn(V, seed)
        cfg = O.DecodeCfg(block_len=4, prompt_len=3, gen_len=16, tau_high=0.7, tau_plan_lo=0.0, tau_plan_hi=0.0, K=0)
        ref = O.decode([4, 5, 6], fn, O.DecodeCfg(block_len=4, prompt_len=3, gen_len=16, tau_high=0.7, tau_plan_lo=0.0,
                                                  tau_plan_hi=0.0, K=0), 1.0, mask_id, [])
        for mode in (A.MODE_RANDOM, A.MODE_PLANNING):
            got = A.decode_extra([4, 5, 6], fn, cfg, 1.0, mask_id, range(8), mode, seed=1)
            assert np.array_equal(got.tokens, ref.tokens) and got.nfe == ref.nfe and got.n_extra == 0


def step(p, yhat, mode, seed, plan, y=None, tau=(0.2, 0.6)):
    mask = 99
    B = list(range(4, 12))
    if y is None:
        y = np.array([1, 2, 3, 4] + [mask] * 8 + [mask] * 4, dtype=np.int32)
    cfg = O.DecodeCfg(block_len=8, prompt_len=4, gen_len=12 if len(y) == 16 else 8, tau_high=0.9, tau_plan_lo=tau[0],
                      tau_plan_hi=tau[1], K=0)
    return A.extra_step(y, np.array(p, np.float32), np.array(yhat), B, cfg, mask, plan, mode, seed, 0)


def test_hand_made_steps():
    mask = 99
    p = [0.95, 0.2, 0.6, 0.61, 0.19, 0.4, 0.92, 0.3]
    yhat = [10, 11, 12, 13, 14, 15, 16, 17]
    # threshold commits positions 4 and 10; eligible (closed bin [0.2, 0.6]) = rows 1, 2, 5, 7 -> positions 5, 6, 9, 11
    picks = collections.Counter()
    for seed in range(400):
        z, info = step(p, yhat, A.MODE_RANDOM, seed, [])
        assert info.base == [4, 10] and z[4] == 10 and z[10] == 16
        assert info.extra in (5, 6, 9, 11) and z[info.extra] == yhat[info.extra - 4] and not info.from_plan
        assert int((z == mask).sum()) == 12 - 3
        picks[info.extra] += 1
    assert set(picks) == {5, 6, 9, 11} and min(picks.values()) > 60            # uniform over the 4 eligible (expected 100)
    # Planning: only rows whose token is a planning token, here rows 2 and 7 (tokens 12, 17)
    picks = collections.Counter()
    for seed in range(200):
        z, info = step(p, yhat, A.MODE_PLANNING, seed, [12, 17, 16, 13])          # 16 and 13 are not eligible rows
        assert info.extra in (6, 11) and info.from_plan
        picks[info.extra] += 1
    assert min(picks.values()) > 60
    # fallback: no eligible planning token -> the Random pool, and the same draw as the Random decoder
    for seed in range(20):
        z1, i1 = step(p, yhat, A.MODE_PLANNING, seed, [10, 13, 14])
        z2, i2 = step(p, yhat, A.MODE_RANDOM, seed, [])
        assert i1.extra == i2.extra and not i1.from_plan and np.array_equal(z1, z2)
    # nothing eligible: a plain threshold step; nothing above the threshold: progress rule, then the extra commit
    z, info = step([0.95, 0.1, 0.7, 0.61, 0.19, 0.8, 0.92, 0.1], yhat, A.MODE_RANDOM, 3, [])
    assert info.extra == -1 and info.base == [4, 10]
    z, info = step([0.5, 0.3, 0.1, 0.1, 0.1, 0.1, 0.1, 0.1], yhat, A.MODE_RANDOM, 3, [])
    assert info.base == [4] and info.extra == 5
    # the draw is keyed by the number of masks: a different canvas fill gives an independent draw, same canvas the same
    assert step(p, yhat, A.MODE_RANDOM, 7, [])[1].extra == step(p, yhat, A.MODE_RANDOM, 7, [])[1].extra


@pytest.mark.parametrize("mode", [A.MODE_RANDOM, A.MODE_PLANNING])
def test_decode_invariants(mode):
    V, mask_id = 16, 15
    nfe_thr, nfe_x = 0, 0
    for seed in range(6):
        fn = table_fn(V, seed)
        cfg = O.DecodeCfg(block_len=4, prompt_len=3, gen_len=16, tau_high=0.7, tau_plan_lo=0.1, tau_plan_hi=0.6, K=0)
        res = A.decode_extra([4, 5, 6], fn, cfg, 1.0, mask_id, range(0, 15, 2), mode, seed=seed)
        assert not np.any(res.tokens == mask_id)
        assert sum(len(s.base) + (s.extra >= 0) for s in res.steps) == cfg.gen_len
        assert all(0.1 <= s.extra_conf <= 0.6 for s in res.steps if s.extra >= 0)
        if mode == A.MODE_PLANNING:
            assert all(int(res.tokens[s.extra]) % 2 == 0 for s in res.steps if s.from_plan)
        nfe_x += res.nfe
        nfe_thr += O.decode([4, 5, 6], fn, O.DecodeCfg(block_len=4, prompt_len=3, gen_len=16, tau_high=0.7, tau_plan_lo=0.0,
                                                       tau_plan_hi=0.0, K=0), 1.0, mask_id, []).nfe
    assert nfe_x < nfe_thr                     # an extra commit per iteration shortens decoding
