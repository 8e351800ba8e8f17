"""CPU oracle for PVF decoding with a block-level K/V cache.

TEST INFRASTRUCTURE ONLY (same rules as pvf_oracle.py).

The paper measures tokens/s "under KV cache" in the manner of block-wise diffusion decoders
(Sec. 5.1): while a block is being decoded, the keys and values of all positions are kept
from a full forward made when the block was entered, and each denoising step recomputes only
the positions of the working window.  The paper gives no further detail, so the scheme is
fixed here (readings):

  K1  refresh: in the first round, and in every round whose active block differs from the
      block the cache was made for, the BACKBONE canvas gets the exact full forward; its
      per-layer rotated keys and values become the cache.  The drafts of such a round are
      forwarded like in any other round (K2), against the cache just made.
  K2  otherwise: for a canvas of the batch only the window rows (the rows whose logits
      the decision step reads: 2 blocks from the active block, 4 with early cross-block
      revelation, cut at the end of the canvas) run through the layers.  In every layer their
      queries attend to all T positions: keys / values of window positions are the ones just
      computed for this canvas, those of all other positions come from the cache.
  K3  the hidden states of positions outside the window are therefore frozen at refresh time:
      an approximation.  It is exact whenever the canvas equals the cached canvas.
  K4  drafts share the backbone's cache (they differ from it only inside the window).

Arithmetic as in pvf_oracle.py (float64 inside, float32 logits).

Parity status: pinned by tests/test_oracle_kvcache.py (equality with the full forward on the
cached canvas, an independently written per-query loop, refresh-every-round == plain decoding,
staleness really coming from the cached canvas).  Speed-ups on trained models: parity unpinned.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import pvf_oracle as O


@dataclass
class KVCache:
    k: List[np.ndarray]      # per layer [T, H, dh] keys after the rotary embedding
    v: List[np.ndarray]      # per layer [T, H, dh]
    block: int = -1          # active block the cache was made for


def _layer_rows(h: np.ndarray, pos: np.ndarray, lw: Dict, cfg: O.ModelCfg):
    """q, k, v [n, H, dh] (q, k rotated) of the rows h [n, d] sitting at canvas positions pos."""
    d, H = cfg.d_model, cfg.n_heads
    dh = d // H
    f64 = np.float64
    a = O.rmsnorm(h, lw["attn_norm"].astype(f64), cfg.rms_eps)
    qkv = a @ lw["wqkv"].astype(f64).T
    n = h.shape[0]
    q, k, v = (qkv[:, i * d:(i + 1) * d].reshape(n, H, dh) for i in range(3))
    p = pos.astype(f64)
    return O.rope(q, cfg.rope_theta, p), O.rope(k, cfg.rope_theta, p), v


def _attend(q: np.ndarray, k_all: np.ndarray, v_all: np.ndarray) -> np.ndarray:
    """softmax(q k^T / sqrt(dh)) v for queries q [n, H, dh] over keys k_all [T, H, dh]."""
    n, H, dh = q.shape
    out = np.empty_like(q)
    for h in range(H):
        s = (q[:, h, :] @ k_all[:, h, :].T) / np.sqrt(float(dh))
        s = s - s.max(axis=-1, keepdims=True)
        e = np.exp(s)
        out[:, h, :] = (e / e.sum(axis=-1, keepdims=True)) @ v_all[:, h, :]
    return out


def _ffn(h: np.ndarray, lw: Dict, cfg: O.ModelCfg) -> np.ndarray:
    f64 = np.float64
    f = O.rmsnorm(h, lw["ffn_norm"].astype(f64), cfg.rms_eps)
    gu = f @ lw["w_gate_up"].astype(f64).T
    return h + (O.silu(gu[:, : cfg.d_ff]) * gu[:, cfg.d_ff:]) @ lw["w_down"].astype(f64).T


def forward_full(tokens: Sequence[int], weights: Dict, cfg: O.ModelCfg) -> Tuple[np.ndarray, KVCache]:
    """Exact forward of one canvas; returns (logits [T, V] float32, its K/V per layer)."""
    tok = np.asarray(tokens, dtype=np.int64)
    T = tok.shape[0]
    pos = np.arange(T)
    h = weights["embed"][tok].astype(np.float64)
    cache = KVCache([], [])
    for lw in weights["layers"][: cfg.n_layers]:
        q, k, v = _layer_rows(h, pos, lw, cfg)
        cache.k.append(k); cache.v.append(v)
        h = h + _attend(q, k, v).reshape(T, cfg.d_model) @ lw["wo"].astype(np.float64).T
        h = _ffn(h, lw, cfg)
    hn = O.rmsnorm(h, weights["final_norm"].astype(np.float64), cfg.rms_eps)
    return (hn @ weights["out_head"].astype(np.float64).T).astype(np.float32), cache


def forward_window(tokens: Sequence[int], window: Sequence[int], cache: KVCache, weights: Dict,
                   cfg: O.ModelCfg) -> np.ndarray:
    """Logits [len(window), V] (float32) of the window positions of `tokens` (reading K2)."""
    tok = np.asarray(tokens, dtype=np.int64)
    w = np.asarray(window, dtype=np.int64)
    h = weights["embed"][tok[w]].astype(np.float64)
    for li, lw in enumerate(weights["layers"][: cfg.n_layers]):
        q, k, v = _layer_rows(h, w, lw, cfg)
        k_all, v_all = cache.k[li].copy(), cache.v[li].copy()
        k_all[w], v_all[w] = k, v
        h = h + _attend(q, k_all, v_all).reshape(len(w), cfg.d_model) @ lw["wo"].astype(np.float64).T
        h = _ffn(h, lw, cfg)
    hn = O.rmsnorm(h, weights["final_norm"].astype(np.float64), cfg.rms_eps)
    return (hn @ weights["out_head"].astype(np.float64).T).astype(np.float32)


@dataclass
class CachedDecodeResult:
    tokens: np.ndarray
    nfe: int
    n_refresh: int
    rounds: List[O.RoundInfo]
    margin: float
    states: List[O.State]            # state after each round


def cached_summaries(state: O.State, cache: Optional[KVCache], weights: Dict, mcfg: O.ModelCfg,
                     cfg: O.DecodeCfg, scale: float, mask_id: int, force_refresh: bool = False
                     ) -> Tuple[np.ndarray, np.ndarray, KVCache, bool]:
    """Stage-1 summaries [1+K_t, R] of one round under readings K1/K2.
    Returns (conf, tok, cache to use from now on, whether this round refreshed)."""
    wp = O.window_positions(cfg, state.k_active)
    ok = wp < cfg.T
    X = O.branch_canvases(state.y, state.drafts)
    conf = np.zeros((len(X), cfg.window_rows), np.float32)
    tok = np.full((len(X), cfg.window_rows), -1, np.int32)
    refresh = force_refresh or cache is None or cache.block != state.k_active
    for j, x in enumerate(X):
        if refresh and j == 0:
            lg, cache = forward_full(x, weights, mcfg)
            lg = lg[wp[ok]]
            cache.block = state.k_active
        else:
            lg = forward_window(x, wp[ok], cache, weights, mcfg)
        conf[j, ok], tok[j, ok] = O.stage1(lg, scale, mask_id)
    return conf, tok, cache, refresh


def decode_cached(prompt: Sequence[int], weights: Dict, mcfg: O.ModelCfg, cfg: O.DecodeCfg, scale: float,
                  mask_id: int, plan_set: Sequence[int], force_refresh: bool = False) -> CachedDecodeResult:
    """Algorithm 1 (one batched forward per round) on top of the block-level K/V cache."""
    st = O.initial_state(prompt, cfg, mask_id)
    cache: Optional[KVCache] = None
    rounds, states, n_refresh = [], [], 0
    while not st.done:
        conf, tok, cache, refreshed = cached_summaries(st, cache, weights, mcfg, cfg, scale, mask_id, force_refresh)
        n_refresh += int(refreshed)
        st, info = O.decide(st, conf, tok, cfg, mask_id, plan_set)
        rounds.append(info); states.append(st)
        assert len(rounds) <= cfg.gen_len + 1
    return CachedDecodeResult(st.y, len(rounds), n_refresh, rounds, min([r.margin for r in rounds], default=np.inf), states)
