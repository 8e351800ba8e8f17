"""Synthetic workloads of benchmark size, materialised directly in HBM.

The paper measures on trained LLaDA-8B-Instruct weights and benchmark prompts; neither is
available offline, so the benchmark model has the same dimensions with random-init weights
(N(0, 0.02^2) matrices, unit norm gains) drawn on the device by the library's counter-based
generator, and the prompts are uniform-random token ids.
"""
from __future__ import annotations

from typing import Dict

import numpy as np
import torch

from . import binding as B

# dimensions of the LLaDA-8B-shaped benchmark model
LLADA_8B = dict(n_layers=32, d_model=4096, n_heads=32, d_ff=12288, vocab=126464, mask_id=126336,
                rms_eps=1e-5, rope_theta=500000.0)


def random_model(dims: Dict, seed: int = 0, dtype=torch.bfloat16, std: float = 0.02,
                 device="cuda") -> Dict:
    """Random-init weights in the layout include/pvf.h documents; distinct stream per tensor."""
    d, ff, V, L = dims["d_model"], dims["d_ff"], dims["vocab"], dims["n_layers"]
    k = [seed * 1000003]

    def mat(r, c):
        t = torch.empty(r, c, dtype=dtype, device=device)
        k[0] += 1
        B.fill_normal(t, k[0], 0.0, std)
        return t

    def ones():
        return torch.ones(d, dtype=dtype, device=device)

    w = {"embed": mat(V, d), "layers": []}
    for _ in range(L):
        w["layers"].append({"attn_norm": ones(), "wqkv": mat(3 * d, d), "wo": mat(d, d),
                            "ffn_norm": ones(), "w_gate_up": mat(2 * ff, d), "w_down": mat(d, ff)})
    w["final_norm"] = ones()
    w["out_head"] = mat(V, d)
    return w


def consistent_model(dims: Dict, seed: int = 0, mix: float = 0.25, dtype=torch.bfloat16, std: float = 0.02,
                     device="cuda") -> Dict:
    """A second synthetic model of the same shape whose predictions are SELF-CONSISTENT: a committed token
    predicts itself at its own position, and a masked position's prediction moves only a little when one
    other position is filled -- the two properties of a trained denoiser that the draft checks of
    Sec. 4.2 / 4.3 rest on and that a random-init model lacks.  Construction (no training, no data):
    unit-variance embeddings, output head = std * embedding (tied up to the scale), and the two
    projections that write into the residual stream (wo, w_down) damped by `mix`, so that the token's own
    embedding dominates the stream at committed positions while masked positions are told apart by what
    the layers mix in from the rest of the canvas.  Everything else is drawn like random_model."""
    d, ff, V, L = dims["d_model"], dims["d_ff"], dims["vocab"], dims["n_layers"]
    k = [seed * 1000003 + 500000]

    def mat(r, c, s):
        t = torch.empty(r, c, dtype=dtype, device=device)
        k[0] += 1
        B.fill_normal(t, k[0], 0.0, s)
        return t

    def ones():
        return torch.ones(d, dtype=dtype, device=device)

    w = {"embed": mat(V, d, 1.0), "layers": []}
    for _ in range(L):
        w["layers"].append({"attn_norm": ones(), "wqkv": mat(3 * d, d, std), "wo": mat(d, d, std * mix),
                            "ffn_norm": ones(), "w_gate_up": mat(2 * ff, d, std), "w_down": mat(d, ff, std * mix)})
    w["final_norm"] = ones()
    w["out_head"] = (w["embed"].float() * std).to(dtype)
    return w


def prior_plan_bitmap(weights: Dict, n: int, mask_id: int) -> torch.Tensor:
    """Planning vocabulary for consistent_model: the n token ids its output head scores highest on the bare
    [MASK] embedding, i.e. the tokens it predicts most readily at a masked position before any context is
    mixed in.  A stand-in for the calibrated vocabulary of App. A.2, which needs the paper's corpora."""
    e = weights["embed"][mask_id].float()
    score = weights["out_head"].float() @ (e / e.pow(2).mean().sqrt())
    score[mask_id] = float("-inf")
    ids = torch.topk(score, n).indices.cpu().numpy().astype(np.int64)
    V = weights["out_head"].shape[0]
    words = np.zeros((V + 31) // 32, dtype=np.uint32)
    np.bitwise_or.at(words, ids >> 5, (np.uint32(1) << (ids & 31).astype(np.uint32)))
    return torch.from_numpy(words.view(np.int32)).to(weights["embed"].device)


def make_context(dims: Dict, weights: Dict, max_seqs: int, max_T: int, max_rows: int) -> B.Context:
    return B.Context(dims["n_layers"], dims["d_model"], dims["n_heads"], dims["d_ff"], dims["vocab"],
                     dims["mask_id"], weights, max_seqs, max_T, max_rows, rms_eps=dims["rms_eps"],
                     rope_theta=dims["rope_theta"])


def random_prompts(G: int, n: int, vocab: int, mask_id: int, seed: int, device="cuda") -> torch.Tensor:
    rng = np.random.default_rng(seed)
    ids = rng.integers(0, vocab - 1, size=(G, n), dtype=np.int64)
    ids = np.where(ids >= mask_id, ids + 1, ids).astype(np.int32)
    return torch.from_numpy(ids).to(device)


def random_plan_bitmap(n: int, vocab: int, mask_id: int, seed: int, device="cuda") -> torch.Tensor:
    rng = np.random.default_rng(seed)
    ids = rng.choice(vocab - 1, size=n, replace=False).astype(np.int64)
    ids = np.where(ids >= mask_id, ids + 1, ids)
    words = np.zeros((vocab + 31) // 32, dtype=np.uint32)
    np.bitwise_or.at(words, ids >> 5, (np.uint32(1) << (ids & 31).astype(np.uint32)))
    return torch.from_numpy(words.view(np.int32)).to(device)


def flops_per_round(dims: Dict, n_seq: int, T: int, R: int) -> float:
    """Algorithmic FLOPs of one batched forward: linear layers + attention + output head on R rows."""
    d, ff, V, L = dims["d_model"], dims["d_ff"], dims["vocab"], dims["n_layers"]
    M = n_seq * T
    linear = 2.0 * M * (3 * d * d + d * d + 3 * d * ff) * L
    attn = 4.0 * n_seq * T * T * d * L
    head = 2.0 * n_seq * R * d * V
    return linear + attn + head
