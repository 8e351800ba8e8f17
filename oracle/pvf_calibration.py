"""CPU oracle for the offline side of PVF: entropy, verified information gain and the
construction of the planning-token vocabulary.

TEST INFRASTRUCTURE ONLY (same rules as pvf_oracle.py: no code shared with the HIP path;
imported only by tests, the smoke check and the bench's CPU-baseline leg).

What follows the paper and where:
  * H_i(z): Shannon entropy (natural log) of the token distribution at position i .. Sec. 3
    ("Verified information gain")
  * evaluation region R_t^j, d_{t,i}^j, Delta H_t^j, VIG_t^j = A_t^j * Delta H_t^j .... Sec. 3
  * calibration trajectory and calibration band C_t^cal ............................ App. A.2
  * token statistics n_v, m_v, r_v^ver, VIG-hat(v) ................................. App. A.2
    ("Token-level aggregation")
  * filtering rule for P^plan ...................................................... App. A.2
    ("Filtering rule"; defaults n_min 50, m_min 20, rho_ver 0.9, gamma_vig 0.03, band
    [0.15, 0.25))

Arithmetic: as in pvf_oracle.py -- float32 values at the interface, float64 inside.  The
probabilities are those of stage 1: softmax of fl32(scale * logit) over every token except
[MASK] (reading R4 there).

Readings:
  C1  the calibration trajectory is plain confidence-threshold decoding with the progress rule
      R1; candidate branches are measured and never committed.
  C2  at most `cap` candidates are measured per step, the most confident ones first (ties:
      lower position), because one batched forward holds a bounded number of canvases;
      cap = None measures all of C_t^cal, which is the paper's statement.
  C3  r_v^ver = (sum of A) / m_v and VIG-hat(v) = (sum of VIG) / n_v are formed in float64 and
      compared with the float32 thresholds widened to float64.
  C4  the [MASK] token is never a member of P^plan.

Parity status: pinned by tests/test_oracle_calibration.py (library entropy, closed forms,
hand-made events, brute-force aggregation, trajectory == threshold decoding).  The actual
vocabularies of the paper need its calibration corpora and trained weights: parity unpinned.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

from . import pvf_oracle as O


def entropy(logits: np.ndarray, scale: float, mask_id: int) -> np.ndarray:
    """logits [n, V] (float32 values) -> H [n] float32, H = - sum_w p_w ln p_w with
    p = softmax(fl32(scale * l)) over w != mask_id and 0 ln 0 = 0."""
    l32 = np.asarray(logits, dtype=np.float32)
    x = (np.float32(scale) * l32).astype(np.float32).astype(np.float64)
    x = np.delete(x, mask_id, axis=1)
    x = x - x.max(axis=1, keepdims=True)
    e = np.exp(x)
    p = e / e.sum(axis=1, keepdims=True)
    with np.errstate(divide="ignore", invalid="ignore"):
        t = np.where(p > 0, p * np.log(p), 0.0)
    return (-t.sum(axis=1)).astype(np.float32)


@dataclass
class Event:
    """One measured calibration candidate (t, j)."""
    token: int          # v = predicted token at the candidate position
    position: int
    nonvacuous: bool    # |S_impact| > 0
    A: int              # verified compatibility, Eq. (at)
    dH: float           # Delta H_t^j (0 if the evaluation region is empty)

    @property
    def vig(self) -> float:
        return self.A * self.dH


def verify_events(z_base: np.ndarray, B: Sequence[int], p_base: np.ndarray, t_base: np.ndarray,
                  H_base: np.ndarray, cands: Sequence[Tuple[int, int]],
                  t_plan: Sequence[np.ndarray], H_plan: Sequence[np.ndarray],
                  tau_high: float, mask_id: int) -> List[Event]:
    """Scores the candidates of one step.  All per-position arrays are indexed like B.

    z_base: base-branch canvas; (p_base, t_base, H_base): top-1 probability / token / entropy
    under z_base; cands[j] = (position, token); (t_plan[j], H_plan[j]): top-1 token / entropy
    under the planning branch z_plan,j = z_base with cands[j] written in."""
    f32 = np.float32
    B = list(B)
    masked = [q for q in range(len(B)) if z_base[B[q]] == mask_id]
    impact = [q for q in masked if f32(p_base[q]) >= f32(tau_high)]
    out = []
    for j, (pos, v) in enumerate(cands):
        A = int(len(impact) > 0 and all(int(t_plan[j][q]) == int(t_base[q]) for q in impact))
        region = [q for q in masked if B[q] != pos]
        dH = float(np.mean([float(H_base[q]) - float(H_plan[j][q]) for q in region])) if region else 0.0
        out.append(Event(int(v), int(pos), len(impact) > 0, A, dH))
    return out


@dataclass
class TokenStats:
    n: np.ndarray       # [V] int64   support
    m: np.ndarray       # [V] int64   non-vacuous verification opportunities
    a: np.ndarray       # [V] int64   sum of A over the events
    vig: np.ndarray     # [V] float64 sum of VIG over the events
    events: List[Event] = field(default_factory=list)
    margin: float = np.inf   # smallest relative distance of any threshold comparison from flipping

    def cmp(self, a: float, b: float) -> None:
        a, b = float(a), float(b)
        den = max(abs(a), abs(b))
        self.margin = min(self.margin, abs(a - b) / den if den > 0 else 0.0)

    @staticmethod
    def zeros(V: int) -> "TokenStats":
        return TokenStats(np.zeros(V, np.int64), np.zeros(V, np.int64), np.zeros(V, np.int64), np.zeros(V, np.float64))

    def add(self, ev: Event) -> None:
        self.n[ev.token] += 1
        self.m[ev.token] += int(ev.nonvacuous)
        self.a[ev.token] += ev.A
        self.vig[ev.token] += ev.vig
        self.events.append(ev)

    @property
    def r_ver(self) -> np.ndarray:
        return np.where(self.m > 0, self.a / np.maximum(self.m, 1), 0.0)

    @property
    def vig_hat(self) -> np.ndarray:
        return np.where(self.n > 0, self.vig / np.maximum(self.n, 1), 0.0)


def calibrate(prompts: Sequence[Sequence[int]], forward_fn: O.ForwardFn, cfg: O.DecodeCfg, scale: float,
              mask_id: int, vocab: int, band: Tuple[float, float] = (0.15, 0.25),
              cap: Optional[int] = None, stats: Optional[TokenStats] = None
              ) -> Tuple[TokenStats, List[np.ndarray], int]:
    """Runs the calibration trajectory of every prompt and aggregates the token statistics.
    Returns (stats, final canvases, number of canvases forwarded)."""
    f32 = np.float32
    stats = stats or TokenStats.zeros(vocab)
    finals, n_fwd = [], 0
    for prompt in prompts:
        y = O.initial_state(prompt, cfg, mask_id).y
        while np.any(y == mask_id):
            k = O.first_masked_block(y, cfg, mask_id)
            lo = cfg.prompt_len + k * cfg.block_len
            B = list(range(lo, lo + O.working_blocks(y, k, cfg, mask_id) * cfg.block_len))
            p, yhat = O.stage1(forward_fn(y)[B], scale, mask_id); n_fwd += 1
            M = [q for q in range(len(B)) if y[B[q]] == mask_id]
            base = [q for q in M if p[q] >= f32(cfg.tau_high)]
            for q in M:
                stats.cmp(p[q], cfg.tau_high)
            if not base:
                base = [min(M, key=lambda q: (-float(p[q]), q))]
                for q in M:
                    if q != base[0]:
                        stats.cmp(p[q], p[base[0]])
            z_base = y.copy()
            for q in base:
                z_base[B[q]] = yhat[q]
            cal = [q for q in M if q not in base and f32(band[0]) <= p[q] < f32(band[1])]
            for q in M:
                if q not in base:
                    stats.cmp(p[q], band[0]); stats.cmp(p[q], band[1])
            cal.sort(key=lambda q: (-float(p[q]), q))
            if cap is not None:
                if len(cal) > cap:
                    stats.cmp(p[cal[cap - 1]], p[cal[cap]])
                cal = cal[:cap]
            if cal:
                lb = forward_fn(z_base)[B]; n_fwd += 1
                p_b, t_b = O.stage1(lb, scale, mask_id)
                H_b = entropy(lb, scale, mask_id)
                for q in range(len(B)):
                    if z_base[B[q]] == mask_id:
                        stats.cmp(p_b[q], cfg.tau_high)
                t_pl, H_pl, cands = [], [], []
                for q in cal:
                    z = z_base.copy(); z[B[q]] = yhat[q]
                    lj = forward_fn(z)[B]; n_fwd += 1
                    t_pl.append(O.stage1(lj, scale, mask_id)[1]); H_pl.append(entropy(lj, scale, mask_id))
                    cands.append((B[q], int(yhat[q])))
                for ev in verify_events(z_base, B, p_b, t_b, H_b, cands, t_pl, H_pl, cfg.tau_high, mask_id):
                    stats.add(ev)
            y = z_base
        finals.append(y)
    return stats, finals, n_fwd


def select_plan_vocab(stats: TokenStats, mask_id: int, n_min: int = 50, m_min: int = 20,
                      rho_ver: float = 0.9, gamma_vig: float = 0.03) -> np.ndarray:
    """The filtering rule: sorted ids of P^plan."""
    keep = ((stats.n >= n_min) & (stats.m >= m_min)
            & (stats.r_ver >= float(np.float32(rho_ver))) & (stats.vig_hat >= float(np.float32(gamma_vig))))
    keep[mask_id] = False
    return np.flatnonzero(keep).astype(np.int32)


def select_margin(stats: TokenStats, rho_ver: float = 0.9, gamma_vig: float = 0.03) -> np.ndarray:
    """Per token: relative distance of its two float comparisons from flipping (inf where the
    integer tests alone decide).  Tests skip tokens whose margin is below the float32 noise."""
    with np.errstate(divide="ignore", invalid="ignore"):
        d1 = np.abs(stats.r_ver - float(np.float32(rho_ver))) / max(float(rho_ver), 1e-30)
        d2 = np.abs(stats.vig_hat - float(np.float32(gamma_vig))) / np.maximum(np.abs(stats.vig_hat), abs(float(gamma_vig)))
    d2 = np.where(np.isfinite(d2), d2, np.inf)
    return np.where(stats.n > 0, np.minimum(d1, d2), np.inf)


# =============================================================================
# the same trajectory with one batched forward per step (reading R2 of pvf_oracle.py)
# =============================================================================
ROUTE_CAL = 3


def cal_summaries(state: O.State, forward_fn: O.ForwardFn, cfg: O.DecodeCfg, scale: float,
                  mask_id: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(p, yhat, H) [1+K_t, R] of the backbone and of every measured branch on the window rows."""
    wp = O.window_positions(cfg, state.k_active)
    ok = wp < cfg.T
    X = O.branch_canvases(state.y, O.Drafts(O.ROUTE_PLAN, state.drafts.fills) if state.drafts.n else O.Drafts())
    conf = np.zeros((len(X), cfg.window_rows), np.float32)
    tok = np.full((len(X), cfg.window_rows), -1, np.int32)
    ent = np.zeros((len(X), cfg.window_rows), np.float32)
    for j, x in enumerate(X):
        lg = forward_fn(x)[wp[ok]]
        conf[j, ok], tok[j, ok] = O.stage1(lg, scale, mask_id)
        ent[j, ok] = entropy(lg, scale, mask_id)
    return conf, tok, ent


def cal_decide(state: O.State, conf: np.ndarray, tok: np.ndarray, ent: np.ndarray, cfg: O.DecodeCfg,
               mask_id: int, band: Tuple[float, float], cap: Optional[int],
               stats: Optional[TokenStats] = None) -> Tuple[O.State, List[Event]]:
    """One step of the pipelined calibration trajectory: measure this batch's branches against
    the backbone (= z_base of the step that proposed them), then do the next step's threshold
    commit on the backbone's own predictions and pick its candidates.  state.drafts holds the
    candidates as fills with route ROUTE_CAL; nothing but base tokens is ever committed."""
    f32 = np.float32
    bl = cfg.block_len
    w0 = cfg.prompt_len + state.k_active * bl
    events: List[Event] = []
    if state.drafts.n:
        B = list(range(w0, w0 + state.ws * bl))
        n = len(B)
        if stats is not None:
            for q in range(n):
                if state.y[B[q]] == mask_id:
                    stats.cmp(conf[0][q], cfg.tau_high)
        events = verify_events(state.y, B, conf[0][:n], tok[0][:n], ent[0][:n], state.drafts.fills,
                               [tok[j][:n] for j in range(1, 1 + state.drafts.n)],
                               [ent[j][:n] for j in range(1, 1 + state.drafts.n)], cfg.tau_high, mask_id)
    # the threshold step of plain decoding (commit, block advance, working set) on the backbone row
    plain = O.DecodeCfg(block_len=bl, prompt_len=cfg.prompt_len, gen_len=cfg.gen_len, tau_high=cfg.tau_high,
                        tau_plan_lo=0.0, tau_plan_hi=0.0, tau_ar_lo=cfg.tau_ar_lo, K=0, routes=0, n_sparse=cfg.n_sparse)
    before = state.y.copy()
    new, info = O.decide(O.State(state.y.copy(), O.Drafts(), state.k_active, state.done, state.ws),
                         conf[:1], tok[:1], plain, mask_id, [])
    if stats is not None:
        stats.margin = min(stats.margin, info.margin)
    fills: List[Tuple[int, int]] = []
    if not new.done:
        lo = cfg.prompt_len + new.k_active * bl
        cand = [i for i in range(lo, lo + new.ws * bl)
                if new.y[i] == mask_id and f32(band[0]) <= conf[0][i - w0] < f32(band[1])]
        if stats is not None:
            for i in range(lo, lo + new.ws * bl):
                if new.y[i] == mask_id:
                    stats.cmp(conf[0][i - w0], band[0]); stats.cmp(conf[0][i - w0], band[1])
        cand.sort(key=lambda i: (-float(conf[0][i - w0]), i))
        if cap is not None:
            if stats is not None and len(cand) > cap:
                stats.cmp(conf[0][cand[cap - 1] - w0], conf[0][cand[cap] - w0])
            cand = cand[:cap]
        fills = [(i, int(tok[0][i - w0])) for i in cand]
    assert np.all((before == new.y) | (before == mask_id))
    return O.State(new.y, O.Drafts(ROUTE_CAL if fills else O.ROUTE_NONE, fills), new.k_active, new.done, new.ws), events


def calibrate_pipelined(prompts: Sequence[Sequence[int]], forward_fn: O.ForwardFn, cfg: O.DecodeCfg,
                        scale: float, mask_id: int, vocab: int, band: Tuple[float, float] = (0.15, 0.25),
                        cap: Optional[int] = None) -> Tuple[TokenStats, List[np.ndarray], int]:
    """`calibrate` with one batched forward per step.  Returns (stats, finals, rounds)."""
    stats = TokenStats.zeros(vocab)
    finals, rounds = [], 0
    for prompt in prompts:
        st = O.initial_state(prompt, cfg, mask_id)
        while not st.done:
            conf, tok, ent = cal_summaries(st, forward_fn, cfg, scale, mask_id)
            st, events = cal_decide(st, conf, tok, ent, cfg, mask_id, band, cap, stats)
            for ev in events:
                stats.add(ev)
            rounds += 1
        finals.append(st.y)
    return stats, finals, rounds
