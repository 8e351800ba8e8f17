"""Seeded generators for every synthetic input used by the tests and the bench.

The paper evaluates on public benchmark prompts with trained LLaDA-8B /
Dream-7B weights and calibrated planning vocabularies; none of those are
available offline, so seeded random stand-ins of the same shapes are used:
normal(0, 0.02) weights, uniform-random prompt ids, a random id set as the
planning vocabulary, and normal(0,1) logit rows with a boosted top-1 entry.

Nothing in this file implements a step of the decoding method.
"""
from __future__ import annotations

from dataclasses import dataclass, asdict
from typing import Dict, List, Sequence

import numpy as np


@dataclass(frozen=True)
class ModelShape:
    """Dimensions of the masked-diffusion denoiser (bidirectional transformer)."""

    n_layers: int
    d_model: int
    n_heads: int
    d_ff: int
    vocab: int
    mask_id: int
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    logit_scale: float = 1.0

    def asdict(self) -> dict:
        return asdict(self)


# 2-layer fp32 model of the small parity configuration.
TINY = ModelShape(n_layers=2, d_model=256, n_heads=4, d_ff=704, vocab=4096,
                  mask_id=4095, rope_theta=10000.0, logit_scale=20.0)

# LLaDA-8B-shaped model (dimensions only; weights are random).
LLADA_8B = ModelShape(n_layers=32, d_model=4096, n_heads=32, d_ff=12288,
                      vocab=126464, mask_id=126336, rope_theta=500000.0,
                      logit_scale=1.0)


# ----------------------------------------------------------------------------
# bf16 helpers (format conversion only: round-to-nearest-even on the top 16 bits)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """float32 array whose every value is exactly representable in bf16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x)).reshape(np.shape(x))


# ----------------------------------------------------------------------------
# model weights
# ----------------------------------------------------------------------------
def make_weights(shape: ModelShape, seed: int = 0, std: float = 0.02,
                 round_to_bf16: bool = False,
                 n_layers: int | None = None) -> Dict[str, object]:
    """Random-init weights in a fixed draw order.

    All matrices are stored [out_features, in_features] (the product is
    ``x @ W.T``):  embed [V,d], per layer attn_norm [d], wqkv [3d,d] (rows
    q|k|v), wo [d,d], ffn_norm [d], w_gate_up [2ff,d] (rows gate|up),
    w_down [d,ff]; then final_norm [d] and out_head [V,d].  Norm gains are
    drawn as 1 + N(0, 0.1) so that a dropped or misplaced gain is visible.
    """
    rng = np.random.default_rng(seed)
    d, ff, V = shape.d_model, shape.d_ff, shape.vocab
    L = shape.n_layers if n_layers is None else n_layers

    def mat(r, c):
        w = rng.standard_normal((r, c), dtype=np.float32) * np.float32(std)
        return bf16_round(w) if round_to_bf16 else w

    def gain():
        g = (1.0 + 0.1 * rng.standard_normal(d, dtype=np.float32)).astype(np.float32)
        return bf16_round(g) if round_to_bf16 else g

    w: Dict[str, object] = {"embed": mat(V, d)}
    layers: List[Dict[str, np.ndarray]] = []
    for _ in range(L):
        layers.append({
            "attn_norm": gain(),
            "wqkv": mat(3 * d, d),
            "wo": mat(d, d),
            "ffn_norm": gain(),
            "w_gate_up": mat(2 * ff, d),
            "w_down": mat(d, ff),
        })
    w["layers"] = layers
    w["final_norm"] = gain()
    w["out_head"] = mat(V, d)
    return w


def make_consistent_weights(shape: ModelShape, seed: int = 0, mix: float = 1.0, std: float = 0.02,
                            round_to_bf16: bool = False) -> Dict[str, object]:
    """Weights of a synthetic denoiser whose predictions are self-consistent: unit-variance embeddings, output
    head = std * embedding, and the two projections that write into the residual stream (wo, w_down) scaled
    by `mix`; everything else as make_weights draws it.  A committed token then predicts itself at its own
    position, and masked positions differ by what the layers mix in from the rest of the canvas."""
    w = make_weights(shape, seed=seed, std=std, round_to_bf16=round_to_bf16)
    rng = np.random.default_rng(seed + 100)
    emb = rng.standard_normal((shape.vocab, shape.d_model), dtype=np.float32)
    head = (emb * np.float32(std)).astype(np.float32)
    w["embed"] = bf16_round(emb) if round_to_bf16 else emb
    w["out_head"] = bf16_round(head) if round_to_bf16 else head
    for lw in w["layers"]:
        for name in ("wo", "w_down"):
            m = (lw[name] * np.float32(mix)).astype(np.float32)
            lw[name] = bf16_round(m) if round_to_bf16 else m
    return w


def prior_plan_vocab(w: Dict[str, object], n: int, mask_id: int) -> np.ndarray:
    """n token ids (sorted) that the output head scores highest on the bare [MASK] embedding: the tokens such a
    model predicts most readily at a masked position.  Stand-in for a calibrated planning vocabulary."""
    e = np.asarray(w["embed"][mask_id], dtype=np.float64)
    score = np.asarray(w["out_head"], dtype=np.float64) @ (e / np.sqrt(np.mean(e * e)))
    score[mask_id] = -np.inf
    return np.sort(np.argsort(-score, kind="stable")[:n]).astype(np.int32)


# ----------------------------------------------------------------------------
# prompts, planning vocabulary
# ----------------------------------------------------------------------------
def make_prompt(seed: int, n: int, vocab: int, mask_id: int) -> np.ndarray:
    """n uniform-random token ids, none equal to the mask id."""
    rng = np.random.default_rng(seed)
    ids = rng.integers(0, vocab - 1, size=n, dtype=np.int64)
    ids = np.where(ids >= mask_id, ids + 1, ids)  # skip mask_id, stay < vocab
    return ids.astype(np.int32)


def make_plan_vocab(seed: int, n: int, vocab: int, mask_id: int) -> np.ndarray:
    """n distinct token ids (sorted), none equal to the mask id."""
    rng = np.random.default_rng(seed)
    ids = rng.choice(vocab - 1, size=n, replace=False).astype(np.int64)
    ids = np.where(ids >= mask_id, ids + 1, ids)
    return np.sort(ids).astype(np.int32)


def plan_bitmap(ids: Sequence[int], vocab: int) -> np.ndarray:
    """Membership bitmap: bit (id & 31) of word (id >> 5), ceil(V/32) uint32 words."""
    words = np.zeros((vocab + 31) // 32, dtype=np.uint32)
    for t in np.asarray(ids, dtype=np.int64):
        words[t >> 5] |= np.uint32(1) << np.uint32(t & 31)
    return words


# ----------------------------------------------------------------------------
# logit tables
# ----------------------------------------------------------------------------
def make_boosted_logits(seed: int, rows: int, vocab: int, boost_hi: float = 12.0,
                        mask_id: int | None = None) -> np.ndarray:
    """[rows, vocab] float32, every value bf16-representable.

    Each row is N(0,1) noise plus a boost b ~ U[0, boost_hi] at one uniformly
    chosen id (never the mask id), so max-softmax confidences range from
    near-uniform to near-one-hot.
    """
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, vocab), dtype=np.float32)
    ids = rng.integers(0, vocab, size=rows)
    if mask_id is not None:
        ids = np.where(ids == mask_id, (ids + 1) % vocab, ids)
    b = rng.uniform(0.0, boost_hi, size=rows).astype(np.float32)
    x[np.arange(rows), ids] += b
    return bf16_round(x)


def table_model_logits(canvas: Sequence[int], vocab: int, seed: int = 0,
                       spread: float = 3.0, mix: float = 0.35) -> np.ndarray:
    """A stand-in 'denoiser' for brute-force tests: logits [T, vocab] = a fixed
    pseudo-random table (depends on seed and position only) plus a smaller
    pseudo-random function of the whole canvas, so that every position sees every
    other position (like a bidirectional model) yet predictions are partly stable
    when one token changes."""
    T = len(canvas)
    static = np.random.default_rng([int(seed), 7919]).standard_normal((T, vocab))
    key = [int(seed)] + [int(t) for t in canvas]
    dyn = np.random.default_rng(key).standard_normal((T, vocab))
    return ((static + mix * dyn) * spread).astype(np.float32)
