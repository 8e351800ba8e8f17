"""Pins for the oracle's stage 1 (top-1 token and its softmax probability, Sec. 3):
closed forms, a library softmax, and the tie / mask-column readings."""
import math

import numpy as np
import pytest
import scipy.special

from oracle import pvf_oracle as O


def test_one_hot_row_closed_form():
    # row [a, 0, ..., 0] with N live columns: p = e^a / (e^a + N - 1)
    V, mask_id = 1000, 999
    for a in (0.5, 3.0, 9.0, 15.0):
        row = np.zeros((1, V), np.float32)
        row[0, 17] = a
        p, t = O.stage1(row, 1.0, mask_id)
        N = V - 1
        a32 = float(np.float32(a))
        assert t[0] == 17
        assert p[0] == np.float32(math.exp(a32) / (math.exp(a32) + N - 1))


def test_threshold_crossing_closed_form():
    # p >= tau  <=>  a >= ln(tau (N-1) / (1 - tau))
    V, mask_id, tau = 4096, 4095, 0.9
    N = V - 1
    a_star = math.log(tau * (N - 1) / (1 - tau))
    for da, above in ((-1e-3, False), (+1e-3, True)):
        row = np.zeros((1, V), np.float32)
        row[0, 5] = a_star + da
        p, _ = O.stage1(row, 1.0, mask_id)
        assert (p[0] >= np.float32(tau)) == above


def test_geometric_row_closed_form():
    # l_w = -c w over live ids 0..N-1 (mask is the last id): Z = (1 - r^N) / (1 - r), r = e^-c
    V, mask_id = 513, 512
    c = 0.03125  # exact in float32, so fl32(l_w) = -c w exactly
    row = (-c * np.arange(V, dtype=np.float64)).astype(np.float32)[None, :]
    p, t = O.stage1(row, 1.0, mask_id)
    r, N = math.exp(-c), V - 1
    Z = (1 - r ** N) / (1 - r)
    assert t[0] == 0
    assert abs(float(p[0]) - 1 / Z) <= 1e-7 / Z


def test_uniform_row_and_bounds():
    V = 777
    for mask_id, want in ((0, 1), (5, 0)):
        p, t = O.stage1(np.full((1, V), 2.5, np.float32), 3.0, mask_id)
        assert t[0] == want                       # lowest live id
        assert p[0] == np.float32(1.0 / (V - 1))
    rng = np.random.default_rng(0)
    p, _ = O.stage1(rng.standard_normal((50, V)).astype(np.float32) * 4, 1.0, 3)
    assert np.all(p >= np.float32(1.0 / (V - 1))) and np.all(p <= 1.0)


def test_mask_column_is_never_predicted_and_carries_no_mass():
    V, mask_id = 64, 10
    rng = np.random.default_rng(1)
    l = rng.standard_normal((8, V)).astype(np.float32)
    l[:, mask_id] = 50.0                          # would win and swallow all mass if counted
    p, t = O.stage1(l, 1.0, mask_id)
    keep = np.delete(l, mask_id, axis=1).astype(np.float64)
    sm = scipy.special.softmax(keep, axis=1)
    ids = np.delete(np.arange(V), mask_id)
    assert np.array_equal(t, ids[sm.argmax(1)])
    np.testing.assert_allclose(p, sm.max(1), rtol=1e-6)


def test_ties_take_lowest_id():
    l = np.zeros((1, 100), np.float32)
    l[0, [70, 30, 55]] = 4.0
    p, t = O.stage1(l, 1.0, 99)
    assert t[0] == 30
    assert abs(float(p[0]) - 1.0 / (3 + 96 * math.exp(-4.0))) < 1e-7


@pytest.mark.parametrize("scale", [1.0, 20.0, 0.37])
def test_matches_library_softmax(scale):
    import torch
    rng = np.random.default_rng(2)
    V, mask_id = 4096, 4095
    l = rng.standard_normal((64, V)).astype(np.float32)
    l[np.arange(64), rng.integers(0, V - 1, 64)] += rng.uniform(0, 12, 64).astype(np.float32)
    p, t = O.stage1(l, scale, mask_id)
    x = (torch.tensor(scale, dtype=torch.float32) * torch.from_numpy(l))[:, :mask_id]
    sm = torch.softmax(x.double(), dim=-1)
    pm, tm = sm.max(-1)
    assert np.array_equal(t, tm.numpy().astype(np.int32))
    np.testing.assert_allclose(p, pm.numpy(), rtol=2e-7)


def test_scale_is_applied_to_logits_before_softmax():
    rng = np.random.default_rng(3)
    l = rng.standard_normal((4, 300)).astype(np.float32)
    p2, t2 = O.stage1(l, 4.0, 299)               # power of two: fl32(4 l) == 4 l exactly
    p1, t1 = O.stage1(4.0 * l, 1.0, 299)
    assert np.array_equal(p1, p2) and np.array_equal(t1, t2)
    p0, _ = O.stage1(l, 1.0, 299)
    assert np.all(p2 > p0)                        # sharper distribution
