"""CPU oracle for Plan-Verify-Fill (PVF) decoding of a masked diffusion LM.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
GPU library must compute.  It shares no code with the HIP path and is imported
only by tests, by the smoke check and by the bench's CPU-baseline leg.

What follows the paper and where:
  * top-1 token / confidence per masked position ........ Sec. 3 (definitions of y-hat, p)
  * base set, base branch ............................... Sec. 3 ("Base branch and impact set")
  * impact set .......................................... Eq. (impact_set)
  * planning branch ..................................... Eq. (plan_branch)
  * verified compatibility A ............................ Eq. (at)
  * planning candidates, Top-K .......................... Sec. 4.1
  * Filter 1 / Filter 2 (C_total) ....................... Sec. 4.2
  * AR fallback construction and verification ........... Sec. 4.3
  * decode loop and route switch ........................ Algorithm 1
  * blockwise semi-autoregressive constraint ............ App. A.1
  * confidence-threshold decoding ....................... Sec. 2
The denoiser architecture is not given in the paper; `forward` is a pre-norm
bidirectional transformer (RMSNorm, rotary embedding with rotate-half pairing,
full multi-head attention without any mask, SwiGLU FFN, untied output head).

Arithmetic: inputs (weights, logits) are float32 values; every product, sum,
exponential and softmax here is evaluated in float64; logits and confidences
are rounded to float32 at the interface and every threshold comparison is done
on those float32 values.

Readings taken where the paper is silent (all listed again in the design notes):
  R1  progress: if no masked position of the active block reaches tau_high, the
      single most confident one is committed (lowest index on ties).
  R2  one forward per round: the accepted branch's own forward output is
      P(.|y_t) and is reused for the next proposal (`decode`); the two-forward
      literal schedule is `decode_literal` and must give the same sequence.
  R3  arg-max ties -> lowest token id;  R4  the [MASK] column is never predicted.
  R5  Top-K ties -> lower position;  R6  Filter-2 ties -> lower draft slot.
  R7  the impact set does not exclude the candidate's own position.
  R8  AR candidates: filter by tau_AR, then the first K by position.
  R9  after a planning round in which every draft is rejected, only the base
      branch is committed (no AR attempt in the same round).
  R10 blocks tile the generation region only; gen_len % block_len == 0.
  R11 early cross-block revelation (App. A.4.1, Eq. block_expansion): the working set of a step
      is fixed when the step's proposal is made, from the canvas before the base commits; the
      same set is used for the base commit, the candidates, the impact set and C_total of that
      step.  "Active block" everywhere above means this working set.

Parity status: every function below is pinned by tests/test_oracle_*.py
(closed forms, library special cases, invariants, brute force).  Absolute
NFE / tokens-per-forward values on trained models are parity unpinned: they
need weights and prompts that are not available offline.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np

ROUTE_NONE = 0
ROUTE_PLAN = 1
ROUTE_AR = 2
ROUTES_BIT_PLAN = 1
ROUTES_BIT_AR = 2


# =============================================================================
# configuration
# =============================================================================
@dataclass
class ModelCfg:
    n_layers: int
    d_model: int
    n_heads: int
    d_ff: int
    vocab: int
    mask_id: int
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    logit_scale: float = 1.0


@dataclass
class DecodeCfg:
    """Hyper-parameters of Algorithm 1 (defaults: the GSM8K / MMLU-Pro row of the
    hyper-parameter table, K=3)."""
    block_len: int
    prompt_len: int
    gen_len: int
    tau_high: float = 0.9
    tau_plan_lo: float = 0.2
    tau_plan_hi: float = 0.65
    tau_ar_lo: float = 0.1
    K: int = 3
    routes: int = ROUTES_BIT_PLAN | ROUTES_BIT_AR
    n_sparse: int = 0      # N_s of Eq. (block_expansion); 0 = early cross-block revelation off

    @property
    def T(self) -> int:
        return self.prompt_len + self.gen_len

    @property
    def n_blocks(self) -> int:
        return self.gen_len // self.block_len

    @property
    def window_rows(self) -> int:
        """Rows scored per canvas, starting at the active block k.  Without early revelation the
        next working block is k or k+1 (2 blocks of rows); with it the working set of this round
        can be {k, k+1} and the next one {k+2, k+3} (4 blocks of rows)."""
        return min((4 if self.n_sparse > 0 else 2) * self.block_len, self.gen_len)

    def check(self) -> None:
        assert self.block_len > 0 and self.gen_len % self.block_len == 0
        assert self.K >= 0 and self.prompt_len >= 0 and self.n_sparse >= 0
        assert self.tau_plan_lo <= self.tau_plan_hi <= self.tau_high


# =============================================================================
# denoiser forward  P_theta(. | canvas)      (architecture: see module docstring)
# =============================================================================
def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope(x: np.ndarray, theta: float, pos: Optional[np.ndarray] = None) -> np.ndarray:
    """Rotary embedding on x [T, H, dh]; dimension i is paired with i + dh/2 and the
    pair at canvas position t is rotated by the angle t * theta**(-2i/dh)."""
    T, H, dh = x.shape
    half = dh // 2
    if pos is None:
        pos = np.arange(T, dtype=np.float64)
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / dh)
    ang = pos[:, None] * inv_freq[None, :]            # [T, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """softmax(q k^T / sqrt(dh)) v over ALL keys (no causal or padding mask).
    q, k, v: [T, H, dh] -> [T, H, dh]."""
    T, H, dh = q.shape
    out = np.empty_like(q)
    for h in range(H):
        s = (q[:, h, :] @ k[:, h, :].T) / np.sqrt(float(dh))   # [Tq, Tk]
        s = s - s.max(axis=-1, keepdims=True)
        e = np.exp(s)
        out[:, h, :] = (e / e.sum(axis=-1, keepdims=True)) @ v[:, h, :]
    return out


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def forward_hidden(tokens: Sequence[int], weights: Dict, cfg: ModelCfg,
                   use_rope: bool = True, pos_offset: int = 0) -> np.ndarray:
    """Final-norm hidden state [T, d] (float64) of one canvas."""
    tok = np.asarray(tokens, dtype=np.int64)
    T = tok.shape[0]
    d, H = cfg.d_model, cfg.n_heads
    dh = d // H
    f64 = np.float64
    h = weights["embed"][tok].astype(f64)                       # [T, d]
    pos = np.arange(T, dtype=f64) + float(pos_offset)
    for lw in weights["layers"][: cfg.n_layers]:
        a = rmsnorm(h, lw["attn_norm"].astype(f64), cfg.rms_eps)
        qkv = a @ lw["wqkv"].astype(f64).T                      # [T, 3d]
        q = qkv[:, 0 * d:1 * d].reshape(T, H, dh)
        k = qkv[:, 1 * d:2 * d].reshape(T, H, dh)
        v = qkv[:, 2 * d:3 * d].reshape(T, H, dh)
        if use_rope:
            q, k = rope(q, cfg.rope_theta, pos), rope(k, cfg.rope_theta, pos)
        o = attention(q, k, v).reshape(T, d)
        h = h + o @ lw["wo"].astype(f64).T
        f = rmsnorm(h, lw["ffn_norm"].astype(f64), cfg.rms_eps)
        gu = f @ lw["w_gate_up"].astype(f64).T                  # [T, 2ff]
        g, u = gu[:, : cfg.d_ff], gu[:, cfg.d_ff:]
        h = h + (silu(g) * u) @ lw["w_down"].astype(f64).T
    return rmsnorm(h, weights["final_norm"].astype(f64), cfg.rms_eps)


def forward(tokens: Sequence[int], weights: Dict, cfg: ModelCfg,
            rows: Optional[Sequence[int]] = None, **kw) -> np.ndarray:
    """Unscaled logits (float32) of one canvas: [T, V], or [len(rows), V] for the
    requested positions only.  The confidence temperature `logit_scale` is NOT
    applied here; it belongs to `stage1`."""
    hn = forward_hidden(tokens, weights, cfg, **kw)
    if rows is not None:
        hn = hn[np.asarray(rows, dtype=np.int64)]
    return (hn @ weights["out_head"].astype(np.float64).T).astype(np.float32)


# =============================================================================
# stage 1: top-1 token and its probability for each logits row
# =============================================================================
def stage1(logits: np.ndarray, scale: float, mask_id: int) -> Tuple[np.ndarray, np.ndarray]:
    """logits [n, V] (float32 values) -> (p [n] float32, yhat [n] int32).

    x_w = fl32(scale * l_w) for every w != mask_id;  yhat = lowest-id arg-max of x;
    p = softmax(x)[yhat] = 1 / sum_w exp(x_w - max x), summed in float64."""
    l32 = np.asarray(logits, dtype=np.float32)
    x = (np.float32(scale) * l32).astype(np.float32)
    x[:, mask_id] = -np.inf
    yhat = np.argmax(x, axis=1)                 # first occurrence = lowest id
    m = x[np.arange(x.shape[0]), yhat].astype(np.float64)
    Z = np.exp(x.astype(np.float64) - m[:, None]).sum(axis=1)
    return (1.0 / Z).astype(np.float32), yhat.astype(np.int32)


# =============================================================================
# round state and the decision step (verify -> commit -> propose)
# =============================================================================
@dataclass
class Drafts:
    """Drafts attached to a backbone canvas.  `fills` = [(position, token)], length K_t.
    PLAN: draft j (1-based) = backbone + fills[j-1].   AR: draft k = backbone + fills[:k]."""
    route: int = ROUTE_NONE
    fills: List[Tuple[int, int]] = field(default_factory=list)

    @property
    def n(self) -> int:
        return len(self.fills) if self.route != ROUTE_NONE else 0


@dataclass
class State:
    y: np.ndarray                    # backbone canvas [T] (= z_base of the coming forward)
    drafts: Drafts
    k_active: int = 0
    done: bool = False
    ws: int = 1                      # blocks in the working set B_t this batch was formed on (1 or 2)


@dataclass
class RoundInfo:
    accept: List[int]                # A_j (PLAN) or ok_k (AR) for each draft of this batch
    winner: int                      # 0 = base branch, else draft slot
    route: int                       # route of the batch that was verified
    n_base: int = 0                  # tokens committed by the threshold (incl. progress rule)
    n_plan: int = 0
    n_ar: int = 0
    impact: List[int] = field(default_factory=list)
    c_total: List[float] = field(default_factory=list)
    margin: float = np.inf           # smallest relative distance of any decision from flipping
    committed: Optional[np.ndarray] = None   # y_t: the canvas right after the verify/commit step


def _margin_cmp(info: RoundInfo, a: float, b: float) -> None:
    """Records how far a comparison a <> b is from flipping, relative to the larger operand
    (a perturbation of the logits by e moves a probability p by about 2 e p (1 - p))."""
    a, b = float(a), float(b)
    den = max(abs(a), abs(b))
    info.margin = min(info.margin, abs(a - b) / den if den > 0 else 0.0)


def branch_canvases(y: np.ndarray, drafts: Drafts) -> List[np.ndarray]:
    """[X_0 = backbone, X_1 .. X_Kt] per Eq. (plan_branch) / the AR-branch definition."""
    out = [y.copy()]
    for j in range(1, drafts.n + 1):
        x = y.copy()
        picks = [drafts.fills[j - 1]] if drafts.route == ROUTE_PLAN else drafts.fills[:j]
        for pos, tok in picks:
            x[pos] = tok
        out.append(x)
    return out


def first_masked_block(y: np.ndarray, cfg: DecodeCfg, mask_id: int) -> int:
    """Index of the first block of the generation region holding a mask; -1 if none."""
    for b in range(cfg.n_blocks):
        lo = cfg.prompt_len + b * cfg.block_len
        if np.any(y[lo: lo + cfg.block_len] == mask_id):
            return b
    return -1


def working_blocks(y: np.ndarray, k: int, cfg: DecodeCfg, mask_id: int) -> int:
    """Eq. (block_expansion): the working set is the active block k, plus the whole next block
    when at most N_s masks are left in block k (and a next block exists).  Returns 1 or 2."""
    if cfg.n_sparse <= 0 or k + 1 >= cfg.n_blocks:
        return 1
    lo = cfg.prompt_len + k * cfg.block_len
    return 2 if int(np.sum(y[lo: lo + cfg.block_len] == mask_id)) <= cfg.n_sparse else 1


def window_positions(cfg: DecodeCfg, k_active: int) -> np.ndarray:
    """Canvas positions of the R scored rows; entries >= T mark rows that do not exist."""
    return cfg.prompt_len + k_active * cfg.block_len + np.arange(cfg.window_rows)


def decide(state: State, conf: np.ndarray, tok: np.ndarray, cfg: DecodeCfg,
           mask_id: int, plan_set: Sequence[int]) -> Tuple[State, RoundInfo]:
    """Verify this batch's drafts, commit the winner, then propose the next batch.

    conf, tok: [1+K_t, R] stage-1 summaries of X_0..X_Kt on the window rows that
    start at the first position of block `state.k_active`."""
    f32 = np.float32
    plan = set(int(t) for t in plan_set)
    bl = cfg.block_len
    X = branch_canvases(state.y, state.drafts)
    w0 = cfg.prompt_len + state.k_active * bl              # canvas position of window row 0
    B = list(range(w0, w0 + state.ws * bl))                # working set this batch was formed on
    dr = state.drafts
    info = RoundInfo(accept=[0] * dr.n, winner=0, route=dr.route if dr.n else ROUTE_NONE)

    # ---- verify ------------------------------------------------------------
    if dr.n and dr.route == ROUTE_PLAN:
        impact = []
        for i in B:
            if X[0][i] == mask_id:
                _margin_cmp(info, conf[0, i - w0], f32(cfg.tau_high))
                if f32(conf[0, i - w0]) >= f32(cfg.tau_high):
                    impact.append(i)
        info.impact = impact
        best_c = None
        for j in range(1, dr.n + 1):
            ok = len(impact) > 0 and all(tok[j, i - w0] == tok[0, i - w0] for i in impact)
            info.accept[j - 1] = int(ok)
            c = float(sum(np.float64(conf[j, i - w0]) for i in B if X[j][i] == mask_id))
            info.c_total.append(c)
            if ok:
                if best_c is not None:
                    _margin_cmp(info, c, best_c)
                if best_c is None or c > best_c:           # strict: ties keep the lower slot
                    best_c, info.winner = c, j
    elif dr.n and dr.route == ROUTE_AR:
        for k in range(1, dr.n + 1):
            ok = all(tok[k, pos - w0] == t for pos, t in dr.fills[:k])
            info.accept[k - 1] = int(ok)
            if ok:
                info.winner = k                            # longest passing extension

    # ---- commit --------------------------------------------------------------
    y = X[info.winner].copy()
    if info.winner:
        if dr.route == ROUTE_PLAN:
            info.n_plan = 1
        else:
            info.n_ar = info.winner
    info.committed = y.copy()
    k_new = first_masked_block(y, cfg, mask_id)
    if k_new < 0:
        return State(y, Drafts(), state.k_active, True), info
    assert state.k_active <= k_new <= state.k_active + state.ws

    # ---- propose from the winner's own predictions ----------------------------
    cw, tw = conf[info.winner], tok[info.winner]
    b0 = cfg.prompt_len + k_new * bl
    ws_new = working_blocks(y, k_new, cfg, mask_id)         # decided on y_t, before the base commits
    M = [i for i in range(b0, b0 + ws_new * bl) if y[i] == mask_id]
    for i in M:
        _margin_cmp(info, cw[i - w0], f32(cfg.tau_high))
    S_base = [i for i in M if f32(cw[i - w0]) >= f32(cfg.tau_high)]
    if not S_base:                                          # R1: progress rule
        best = M[0]
        for i in M[1:]:
            if cw[i - w0] > cw[best - w0]:
                best = i
        for i in M:
            if i != best:
                _margin_cmp(info, cw[i - w0], cw[best - w0])
        S_base = [best]
    for i in S_base:
        y[i] = tw[i - w0]
    info.n_base = len(S_base)
    if first_masked_block(y, cfg, mask_id) < 0:
        return State(y, Drafts(), k_new, True, ws_new), info   # nothing left: no further forward

    Rm = [i for i in M if i not in S_base]
    nxt = Drafts()
    if cfg.K > 0 and (cfg.routes & ROUTES_BIT_PLAN):
        cand = []
        for i in Rm:
            if int(tw[i - w0]) in plan:
                _margin_cmp(info, cw[i - w0], f32(cfg.tau_plan_lo))
                _margin_cmp(info, cw[i - w0], f32(cfg.tau_plan_hi))
                if f32(cfg.tau_plan_lo) <= f32(cw[i - w0]) < f32(cfg.tau_plan_hi):
                    cand.append(i)
        if cand:
            cand.sort(key=lambda i: (-float(cw[i - w0]), i))
            if len(cand) > cfg.K:                           # the cut between kept and dropped
                _margin_cmp(info, cw[cand[cfg.K - 1] - w0], cw[cand[cfg.K] - w0])
            for a, b in zip(cand[: cfg.K], cand[1: cfg.K]):  # order among kept sets the slots
                _margin_cmp(info, cw[a - w0], cw[b - w0])
            nxt = Drafts(ROUTE_PLAN, [(i, int(tw[i - w0])) for i in cand[: cfg.K]])
    if nxt.n == 0 and cfg.K > 0 and (cfg.routes & ROUTES_BIT_AR):
        cand = []
        for i in Rm:
            _margin_cmp(info, cw[i - w0], f32(cfg.tau_ar_lo))
            if f32(cw[i - w0]) >= f32(cfg.tau_ar_lo):
                cand.append(i)
        if cand:
            nxt = Drafts(ROUTE_AR, [(i, int(tw[i - w0])) for i in sorted(cand)[: cfg.K]])
    return State(y, nxt, k_new, False, ws_new), info


# =============================================================================
# one round and the decode loops
# =============================================================================
ForwardFn = Callable[[np.ndarray], np.ndarray]      # canvas [T] -> unscaled logits [T, V]


def initial_state(prompt: Sequence[int], cfg: DecodeCfg, mask_id: int) -> State:
    cfg.check()
    y = np.full(cfg.T, mask_id, dtype=np.int32)
    y[: cfg.prompt_len] = np.asarray(prompt, dtype=np.int32)
    assert not np.any(y[: cfg.prompt_len] == mask_id)
    return State(y, Drafts(), 0, cfg.gen_len == 0)


def summaries(state: State, forward_fn: ForwardFn, cfg: DecodeCfg, scale: float,
              mask_id: int) -> Tuple[np.ndarray, np.ndarray]:
    """Forward every canvas of the batch on its own and reduce the window rows with stage 1.
    Rows past the end of the canvas get p = 0, token = -1."""
    wp = window_positions(cfg, state.k_active)
    ok = wp < cfg.T
    X = branch_canvases(state.y, state.drafts)
    conf = np.zeros((len(X), cfg.window_rows), dtype=np.float32)
    tok = np.full((len(X), cfg.window_rows), -1, dtype=np.int32)
    for j, x in enumerate(X):
        logits = forward_fn(x)
        conf[j, ok], tok[j, ok] = stage1(logits[wp[ok]], scale, mask_id)
    return conf, tok


def pvf_round(state: State, forward_fn: ForwardFn, cfg: DecodeCfg, scale: float,
              mask_id: int, plan_set: Sequence[int]) -> Tuple[State, RoundInfo]:
    """One PVF round = one batched forward over {backbone, drafts} + the decision step."""
    conf, tok = summaries(state, forward_fn, cfg, scale, mask_id)
    return decide(state, conf, tok, cfg, mask_id, plan_set)


@dataclass
class DecodeResult:
    tokens: np.ndarray
    nfe: int
    rounds: List[RoundInfo]
    canvases: List[np.ndarray]        # y_t after each round's verify/commit step
    margin: float

    @property
    def n_base(self): return sum(r.n_base for r in self.rounds)
    @property
    def n_plan(self): return sum(r.n_plan for r in self.rounds)
    @property
    def n_ar(self): return sum(r.n_ar for r in self.rounds)


def decode(prompt: Sequence[int], forward_fn: ForwardFn, cfg: DecodeCfg, scale: float,
           mask_id: int, plan_set: Sequence[int], max_rounds: int = 100000) -> DecodeResult:
    """Algorithm 1 with one forward per round (reading R2)."""
    st = initial_state(prompt, cfg, mask_id)
    rounds: List[RoundInfo] = []
    canv: List[np.ndarray] = []
    while not st.done:
        assert len(rounds) < max_rounds
        st, info = pvf_round(st, forward_fn, cfg, scale, mask_id, plan_set)
        rounds.append(info)
        canv.append(info.committed)
    margin = min([r.margin for r in rounds], default=np.inf)
    return DecodeResult(st.y, len(rounds), rounds, canv, margin)


def decode_literal(prompt: Sequence[int], forward_fn: ForwardFn, cfg: DecodeCfg, scale: float,
                   mask_id: int, plan_set: Sequence[int]) -> Tuple[np.ndarray, int, List[np.ndarray]]:
    """Algorithm 1 taken line by line: each iteration first forwards y_{t-1} to get the
    predictions on the active block, forms the base branch and the candidates, and then
    spends a second (batched) forward on {z_base, drafts} to verify them.
    Returns (tokens, number of forwards, list of y_t after each iteration)."""
    f32 = np.float32
    plan = set(int(t) for t in plan_set)
    cfg.check()
    y = np.full(cfg.T, mask_id, dtype=np.int32)
    y[: cfg.prompt_len] = np.asarray(prompt, dtype=np.int32)
    nfe, trail = 0, []
    while np.any(y == mask_id):
        k = first_masked_block(y, cfg, mask_id)
        b0 = cfg.prompt_len + k * cfg.block_len
        B = list(range(b0, b0 + working_blocks(y, k, cfg, mask_id) * cfg.block_len))
        p, yh = stage1(forward_fn(y)[B], scale, mask_id); nfe += 1
        M = [i for i in B if y[i] == mask_id]
        S_base = [i for i in M if f32(p[i - b0]) >= f32(cfg.tau_high)]
        if not S_base:
            S_base = [max(M, key=lambda i: (float(p[i - b0]), -i))]
        z = y.copy()
        for i in S_base:
            z[i] = yh[i - b0]
        if not np.any(z == mask_id):
            y = z; trail.append(y.copy()); break
        Rm = [i for i in M if i not in S_base]
        P_plan = [i for i in Rm if int(yh[i - b0]) in plan
                  and f32(cfg.tau_plan_lo) <= f32(p[i - b0]) < f32(cfg.tau_plan_hi)]
        if cfg.K > 0 and (cfg.routes & ROUTES_BIT_PLAN) and P_plan:
            top = sorted(P_plan, key=lambda i: (-float(p[i - b0]), i))[: cfg.K]
            branches = []
            for i in top:
                zz = z.copy(); zz[i] = yh[i - b0]; branches.append(zz)
            outs = [stage1(forward_fn(c)[B], scale, mask_id) for c in [z] + branches]; nfe += 1
            pb, yb = outs[0]
            impact = [i for i in B if z[i] == mask_id and f32(pb[i - b0]) >= f32(cfg.tau_high)]
            best, best_c = None, None
            for j, zz in enumerate(branches, start=1):
                pj, yj = outs[j]
                if impact and all(yj[i - b0] == yb[i - b0] for i in impact):
                    c = float(sum(np.float64(pj[i - b0]) for i in B if zz[i] == mask_id))
                    if best is None or c > best_c:
                        best, best_c = zz, c
            y = best if best is not None else z
        else:
            ar = [i for i in Rm if f32(p[i - b0]) >= f32(cfg.tau_ar_lo)][: cfg.K] \
                if (cfg.K > 0 and (cfg.routes & ROUTES_BIT_AR)) else []
            if ar:
                branches = []
                for k_ in range(1, len(ar) + 1):
                    zz = z.copy()
                    for i in ar[:k_]:
                        zz[i] = yh[i - b0]
                    branches.append(zz)
                nfe += 1
                y = z
                for k_, zz in enumerate(branches, start=1):
                    _, yk = stage1(forward_fn(zz)[B], scale, mask_id)
                    if all(yk[i - b0] == yh[i - b0] for i in ar[:k_]):
                        y = zz
            else:
                y = z
        trail.append(y.copy())
    return y, nfe, trail
