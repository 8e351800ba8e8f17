"""Pins for the oracle's denoiser forward: the same network composed from PyTorch CPU
library ops (with the rotary embedding written in complex form), plus structural
invariants that a wrong pairing, a causal mask, a dropped gain or a transposed weight break."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import pvf_oracle as O
from synth import inputs as S

SMALL = S.ModelShape(n_layers=2, d_model=64, n_heads=4, d_ff=96, vocab=97, mask_id=96,
                     rope_theta=10000.0)


def _cfg(shape):
    return O.ModelCfg(shape.n_layers, shape.d_model, shape.n_heads, shape.d_ff, shape.vocab,
                      shape.mask_id, shape.rms_eps, shape.rope_theta, shape.logit_scale)


def _torch_forward(tokens, w, shape):
    """Library composition: F.rms_norm, F.scaled_dot_product_attention, F.silu, F.linear,
    rotary embedding as multiplication of (x_i + i x_{i+dh/2}) by exp(i t theta^(-2i/dh))."""
    t64 = lambda a: torch.from_numpy(np.asarray(a)).double()
    d, H = shape.d_model, shape.n_heads
    dh = d // H
    tok = torch.as_tensor(np.asarray(tokens), dtype=torch.long)
    T = tok.shape[0]
    h = F.embedding(tok, t64(w["embed"]))
    inv = 1.0 / (shape.rope_theta ** (torch.arange(0, dh, 2).double() / dh))
    rot = torch.polar(torch.ones(T, dh // 2).double(), torch.outer(torch.arange(T).double(), inv))

    def rotary(x):                                            # [T, H, dh]
        z = torch.complex(x[..., : dh // 2], x[..., dh // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    for lw in w["layers"]:
        a = F.rms_norm(h, (d,), t64(lw["attn_norm"]), shape.rms_eps)
        q, k, v = F.linear(a, t64(lw["wqkv"])).split(d, dim=-1)
        q, k, v = (x.reshape(T, H, dh) for x in (q, k, v))
        q, k = rotary(q), rotary(k)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                           v.transpose(0, 1)[None], is_causal=False)[0]
        h = h + F.linear(o.transpose(0, 1).reshape(T, d), t64(lw["wo"]))
        f = F.rms_norm(h, (d,), t64(lw["ffn_norm"]), shape.rms_eps)
        g, u = F.linear(f, t64(lw["w_gate_up"])).split(shape.d_ff, dim=-1)
        h = h + F.linear(F.silu(g) * u, t64(lw["w_down"]))
    hn = F.rms_norm(h, (d,), t64(w["final_norm"]), shape.rms_eps)
    return F.linear(hn, t64(w["out_head"])).numpy()


@pytest.mark.parametrize("shape,T", [(SMALL, 23), (S.TINY, 48)])
def test_forward_matches_library_composition(shape, T):
    w = S.make_weights(shape, seed=11, std=0.08)
    tok = S.make_prompt(5, T, shape.vocab, shape.mask_id)
    tok[T // 2:] = shape.mask_id
    got = O.forward(tok, w, _cfg(shape))
    want = _torch_forward(tok, w, shape)
    assert got.dtype == np.float32 and got.shape == (T, shape.vocab)
    np.testing.assert_allclose(got, want, atol=2e-6, rtol=1e-5)


def test_rows_argument_selects_positions():
    w = S.make_weights(SMALL, seed=1, std=0.08)
    tok = S.make_prompt(2, 16, SMALL.vocab, SMALL.mask_id)
    full = O.forward(tok, w, _cfg(SMALL))
    sub = O.forward(tok, w, _cfg(SMALL), rows=[3, 9, 15])
    assert np.array_equal(sub, full[[3, 9, 15]])


def test_rope_identity_at_position_zero_and_norm_preserving():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 2, 16))
    y = O.rope(x, 10000.0)
    assert np.array_equal(y[0], x[0])
    np.testing.assert_allclose((y ** 2).sum(-1), (x ** 2).sum(-1), rtol=1e-12)
    # pair (i, i + dh/2), angle t * theta^(-2i/dh): check one element by hand
    t, i, dh = 3, 2, 16
    ang = t * 10000.0 ** (-2 * i / dh)
    np.testing.assert_allclose(y[t, 1, i], x[t, 1, i] * np.cos(ang) - x[t, 1, i + 8] * np.sin(ang))
    np.testing.assert_allclose(y[t, 1, i + 8], x[t, 1, i + 8] * np.cos(ang) + x[t, 1, i] * np.sin(ang))


def test_rope_scores_depend_on_relative_position_only():
    # shifting every position by a constant must not change the logits
    w = S.make_weights(SMALL, seed=3, std=0.08)
    tok = S.make_prompt(4, 12, SMALL.vocab, SMALL.mask_id)
    a = O.forward(tok, w, _cfg(SMALL))
    b = O.forward(tok, w, _cfg(SMALL), pos_offset=37)
    np.testing.assert_allclose(a, b, atol=1e-5)
    c = O.forward(tok, w, _cfg(SMALL), use_rope=False)
    assert np.abs(a - c).max() > 1e-3             # and the rotation does do something


def test_no_mask_of_any_kind_bidirectional():
    w = S.make_weights(SMALL, seed=4, std=0.08)
    tok = S.make_prompt(6, 10, SMALL.vocab, SMALL.mask_id)
    a = O.forward(tok, w, _cfg(SMALL))
    tok2 = tok.copy()
    tok2[-1] = (tok2[-1] + 1) % (SMALL.vocab - 1)
    b = O.forward(tok2, w, _cfg(SMALL))
    assert np.abs(a[0] - b[0]).max() > 1e-4       # first position sees the last one
    # without rotary embedding the network is permutation-equivariant
    perm = np.random.default_rng(0).permutation(10)
    c = O.forward(tok, w, _cfg(SMALL), use_rope=False)
    d = O.forward(tok[perm], w, _cfg(SMALL), use_rope=False)
    np.testing.assert_allclose(d, c[perm], atol=1e-5)


def test_attention_special_cases():
    rng = np.random.default_rng(5)
    q, k, v = (rng.standard_normal((1, 2, 8)) for _ in range(3))
    assert np.allclose(O.attention(q, k, v), v)                      # T = 1 -> v
    k, v = rng.standard_normal((7, 2, 8)), rng.standard_normal((7, 2, 8))
    out = O.attention(np.zeros((7, 2, 8)), k, v)
    np.testing.assert_allclose(out, np.broadcast_to(v.mean(0), (7, 2, 8)))   # q = 0 -> mean of v
    # one dominant key -> that key's value; also fixes the 1/sqrt(dh) factor via a 2-key case
    q = np.zeros((1, 1, 4)); q[0, 0, 0] = 2.0
    k = np.zeros((2, 1, 4)); k[0, 0, 0] = 3.0
    v = np.zeros((2, 1, 4)); v[0, 0, 1] = 1.0
    wgt = 1.0 / (1.0 + np.exp(-(2.0 * 3.0) / np.sqrt(4.0)))
    np.testing.assert_allclose(O.attention(q, k, v)[0, 0, 1], wgt)


def test_rmsnorm_and_silu_closed_forms():
    x = np.array([[3.0, -4.0, 0.0, 0.0]])
    g = np.array([1.0, 2.0, 3.0, 4.0])
    np.testing.assert_allclose(O.rmsnorm(x, g, 0.0), [[3 / 2.5, -8 / 2.5, 0, 0]])
    np.testing.assert_allclose(O.silu(np.array([0.0, 1.0])), [0.0, 1 / (1 + np.exp(-1.0))])


def test_weight_orientation_single_layer_hand_computation():
    """d=2, H=1, one token: attention returns v, so every matmul can be written out by hand."""
    shape = S.ModelShape(n_layers=1, d_model=2, n_heads=1, d_ff=1, vocab=3, mask_id=2, rms_eps=0.0)
    w = {
        "embed": np.array([[1.0, 2.0], [0.5, -1.0], [0, 0]], np.float32),
        "layers": [{
            "attn_norm": np.array([1.0, 1.0], np.float32),
            "wqkv": np.array([[1, 0], [0, 1], [1, 1], [1, -1], [2, 0], [0, 3]], np.float32),
            "wo": np.array([[1, 2], [3, 4]], np.float32),
            "ffn_norm": np.array([2.0, 0.5], np.float32),
            "w_gate_up": np.array([[1, 1], [1, -1]], np.float32),
            "w_down": np.array([[2.0], [-1.0]], np.float32),
        }],
        "final_norm": np.array([1.0, 1.0], np.float32),
        "out_head": np.array([[1, 0], [0, 1], [1, 1]], np.float32),
    }
    h = np.array([1.0, 2.0])
    a = h / np.sqrt((h ** 2).mean())
    v = np.array([2 * a[0], 3 * a[1]])                      # rows 4,5 of wqkv
    h = h + np.array([1 * v[0] + 2 * v[1], 3 * v[0] + 4 * v[1]])
    f = h / np.sqrt((h ** 2).mean()) * np.array([2.0, 0.5])
    g, u = f[0] + f[1], f[0] - f[1]
    h = h + (g / (1 + np.exp(-g)) * u) * np.array([2.0, -1.0])
    hn = h / np.sqrt((h ** 2).mean())
    want = np.array([hn[0], hn[1], hn[0] + hn[1]])
    got = O.forward([0], w, _cfg(shape))
    np.testing.assert_allclose(got[0], want, rtol=1e-6)
