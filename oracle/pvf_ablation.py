"""CPU oracle for the Random / Planning single-extra-commit decoders of the paper's ablation.

TEST INFRASTRUCTURE ONLY (same rules as pvf_oracle.py).

App. A.3.1 ("Planning tokens beyond high-confidence decoding"): every decoding iteration first
commits all masked positions of the working block that pass the confidence threshold, then
commits exactly ONE more token among the remaining masked positions whose top-1 confidence lies
in the CLOSED bin [tau_l, tau_u]:
  Random    one eligible position, uniformly at random;
  Planning  one position, uniformly at random, among the eligible ones whose top-1 token is a
            planning token; if there is none, the Random rule.
No drafts are verified: these decoders isolate WHICH low-confidence token is committed.

Readings:
  X1  the threshold step keeps the progress rule R1 of pvf_oracle.py (the paper's baseline
      never stalls on its benchmarks; a random model can).
  X2  "uniformly at random" is realised by a counter-based generator so that the GPU library
      and this oracle draw the same numbers: u = splitmix64(seed * 2^32 + group * 2^20 + n_masked),
      where n_masked is the number of masked canvas positions at the start of the iteration
      (it strictly decreases, so no key repeats), and the pick is the (u mod count)-th eligible
      position in canvas order.  The modulo bias is below 2^-50.
  X3  if no position is eligible the iteration is a plain threshold iteration.

Parity status: pinned by tests/test_oracle_ablation.py (generator against the published
SplitMix64 vector, empty bin == threshold decoding, eligibility and fallback on hand-made
steps, uniformity over seeds).  The paper's accuracy / NFE figures: parity unpinned.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np

from . import pvf_oracle as O

MODE_RANDOM = 1
MODE_PLANNING = 2
_M64 = (1 << 64) - 1


def splitmix64(x: int) -> int:
    """One step of the SplitMix64 generator started at state x (Steele, Lea, Flood 2014)."""
    z = (x + 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def draw(seed: int, group: int, n_masked: int) -> int:
    return splitmix64(((seed & 0xFFFFFFFF) << 32) + ((group & 0xFFF) << 20) + (n_masked & 0xFFFFF))


@dataclass
class StepInfo:
    base: List[int]                    # positions committed by the threshold (or the progress rule)
    extra: int = -1                    # position of the extra commit, -1 if none
    extra_conf: float = 0.0
    from_plan: bool = False            # the extra commit came from the planning subset
    margin: float = np.inf


def extra_step(y: np.ndarray, p: np.ndarray, yhat: np.ndarray, B: Sequence[int], cfg: O.DecodeCfg,
               mask_id: int, plan_set: Sequence[int], mode: int, seed: int, group: int
               ) -> Tuple[np.ndarray, StepInfo]:
    """One iteration on the working set B given its predictions (p, yhat indexed like B)."""
    f32 = np.float32
    plan = set(int(t) for t in plan_set)
    info = StepInfo([])

    def cmp(a, b):
        a, b = float(a), float(b)
        den = max(abs(a), abs(b))
        info.margin = min(info.margin, abs(a - b) / den if den > 0 else 0.0)

    n_masked = int(np.sum(y == mask_id))
    M = [q for q in range(len(B)) if y[B[q]] == mask_id]
    base = [q for q in M if p[q] >= f32(cfg.tau_high)]
    for q in M:
        cmp(p[q], cfg.tau_high)
    if not base:
        base = [min(M, key=lambda q: (-float(p[q]), q))]
        for q in M:
            if q != base[0]:
                cmp(p[q], p[base[0]])
    z = y.copy()
    for q in base:
        z[B[q]] = yhat[q]
    info.base = [B[q] for q in base]
    rest = [q for q in M if q not in base]
    elig = [q for q in rest if f32(cfg.tau_plan_lo) <= p[q] <= f32(cfg.tau_plan_hi)]
    for q in rest:
        cmp(p[q], cfg.tau_plan_lo); cmp(p[q], cfg.tau_plan_hi)
    pool = elig
    if mode == MODE_PLANNING:
        sub = [q for q in elig if int(yhat[q]) in plan]
        if sub:
            pool, info.from_plan = sub, True
    if pool:
        q = pool[draw(seed, group, n_masked) % len(pool)]
        z[B[q]] = yhat[q]
        info.extra, info.extra_conf = B[q], float(p[q])
    return z, info


@dataclass
class AblationResult:
    tokens: np.ndarray
    nfe: int
    steps: List[StepInfo] = field(default_factory=list)

    @property
    def n_extra(self) -> int:
        return sum(s.extra >= 0 for s in self.steps)

    @property
    def avg_extra_conf(self) -> float:
        c = [s.extra_conf for s in self.steps if s.extra >= 0]
        return float(np.mean(c)) if c else 0.0

    @property
    def margin(self) -> float:
        return min([s.margin for s in self.steps], default=np.inf)


def decode_extra(prompt: Sequence[int], forward_fn: O.ForwardFn, cfg: O.DecodeCfg, scale: float, mask_id: int,
                 plan_set: Sequence[int], mode: int, seed: int, group: int = 0) -> AblationResult:
    """Blockwise decoding with the threshold rule plus one extra low-confidence commit per
    iteration; the bin is [cfg.tau_plan_lo, cfg.tau_plan_hi] (closed)."""
    y = O.initial_state(prompt, cfg, mask_id).y
    res = AblationResult(y, 0)
    while np.any(y == mask_id):
        k = O.first_masked_block(y, cfg, mask_id)
        lo = cfg.prompt_len + k * cfg.block_len
        B = list(range(lo, lo + O.working_blocks(y, k, cfg, mask_id) * cfg.block_len))
        p, yhat = O.stage1(forward_fn(y)[B], scale, mask_id)
        y, info = extra_step(y, p, yhat, B, cfg, mask_id, plan_set, mode, seed, group)
        res.steps.append(info)
        res.nfe += 1
    res.tokens = y
    return res
