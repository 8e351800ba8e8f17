"""Test helper: the denoiser forward in float64 with a round-to-bf16 at every point where a bf16
pipeline stores an activation tensor.

It answers one question for the GPU parity tests: how far must ANY forward that keeps its activations
in bf16 between its matrix products sit from the exact (float64) forward, however well its kernels
are written?  `forward_bf16_storage` is the float64 composition of tests' oracle (same architecture,
same order of operations) with `r()` = round-to-nearest-even to bf16 applied to
    the normed input of each projection, q / k / v, the rotated q and k, the softmax weights that
    multiply v, the attention output, the residual stream after each of its two updates, the
    SwiGLU output, the normed window rows, the logits.
It is NOT the oracle (the oracle is oracle/pvf_oracle.py and has no rounding anywhere) and it shares
no code with the HIP path; the GPU tests use it (a) to derive the bound that replaces the 5e-2
max-abs bar at the full model width and (b) as a second, much closer reference for the bf16 kernels.
"""
from __future__ import annotations

from typing import Dict, Optional, Sequence

import numpy as np


def r(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bf16 value (ties to even), returned as float64."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    u = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return u.view(np.float32).astype(np.float64).reshape(np.shape(x))


def _rmsnorm(x, gain, eps):
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * gain


def _rope(x, theta, pos):
    T, H, dh = x.shape
    half = dh // 2
    inv = theta ** (-2.0 * np.arange(half, dtype=np.float64) / dh)
    ang = pos[:, None] * inv[None, :]
    # the table the kernels read is float32
    c = np.cos(ang).astype(np.float32).astype(np.float64)[:, None, :]
    s = np.sin(ang).astype(np.float32).astype(np.float64)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def forward_bf16_storage(tokens: Sequence[int], weights: Dict, n_layers: int, d_model: int, n_heads: int,
                         d_ff: int, rms_eps: float, rope_theta: float,
                         rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """Logits [len(rows), V] (bf16 values as float32) of one canvas; weights must hold bf16 values."""
    f64 = np.float64
    tok = np.asarray(tokens, dtype=np.int64)
    T, d, H = tok.shape[0], d_model, n_heads
    dh = d // H
    pos = np.arange(T, dtype=f64)
    h = weights["embed"][tok].astype(f64)
    for lw in weights["layers"][:n_layers]:
        a = r(_rmsnorm(h, lw["attn_norm"].astype(f64), rms_eps))
        qkv = r(a @ lw["wqkv"].astype(f64).T)
        q = r(_rope(qkv[:, :d].reshape(T, H, dh), rope_theta, pos))
        k = r(_rope(qkv[:, d:2 * d].reshape(T, H, dh), rope_theta, pos))
        v = qkv[:, 2 * d:].reshape(T, H, dh)
        o = np.empty((T, H, dh))
        for hd in range(H):
            s = (q[:, hd] @ k[:, hd].T) / np.sqrt(float(dh))
            p = r(np.exp(s - s.max(axis=-1, keepdims=True)))      # the weights enter the matrix product in bf16
            o[:, hd] = (p @ v[:, hd]) / p.sum(axis=-1, keepdims=True)
        o = r(o.reshape(T, d))
        h = r(h + o @ lw["wo"].astype(f64).T)
        f = r(_rmsnorm(h, lw["ffn_norm"].astype(f64), rms_eps))
        gu = f @ lw["w_gate_up"].astype(f64).T
        g, u = gu[:, :d_ff], gu[:, d_ff:]
        act = r(g / (1.0 + np.exp(-g)) * u)
        h = r(h + act @ lw["w_down"].astype(f64).T)
    if rows is not None:
        h = h[np.asarray(rows, dtype=np.int64)]
    hn = r(_rmsnorm(h, weights["final_norm"].astype(f64), rms_eps))
    return r(hn @ weights["out_head"].astype(f64).T).astype(np.float32)
