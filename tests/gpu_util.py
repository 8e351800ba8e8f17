"""Helpers shared by the GPU parity tests: move synthetic inputs to the device and translate
between the library's state buffers and the oracle's State objects."""
from __future__ import annotations

import numpy as np
import torch

from oracle import pvf_oracle as O
from paper_2601_12247_amd import binding as B
from synth import inputs as S


def oracle_model_cfg(shape: S.ModelShape, n_layers=None) -> O.ModelCfg:
    return O.ModelCfg(shape.n_layers if n_layers is None else n_layers, shape.d_model, shape.n_heads,
                      shape.d_ff, shape.vocab, shape.mask_id, shape.rms_eps, shape.rope_theta,
                      shape.logit_scale)


def oracle_decode_cfg(c: B.DecodeCfg) -> O.DecodeCfg:
    return O.DecodeCfg(block_len=c.block_len, prompt_len=c.prompt_len, gen_len=c.gen_len,
                       tau_high=c.tau_high, tau_plan_lo=c.tau_plan_lo, tau_plan_hi=c.tau_plan_hi,
                       tau_ar_lo=c.tau_ar_lo, K=c.K, routes=c.routes, n_sparse=c.n_sparse)


def to_device(w, dtype=torch.float32, device="cuda"):
    def t(a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(device=device, dtype=dtype)
    out = {k: t(v) for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: t(v) for k, v in lw.items()} for lw in w["layers"]]
    return out


def make_context(shape: S.ModelShape, w_dev, max_seqs, max_T, max_rows, n_layers=None) -> B.Context:
    L = shape.n_layers if n_layers is None else n_layers
    return B.Context(L, shape.d_model, shape.n_heads, shape.d_ff, shape.vocab, shape.mask_id, w_dev,
                     max_seqs, max_T, max_rows, rms_eps=shape.rms_eps, rope_theta=shape.rope_theta)


def oracle_state(st: B.State, g: int) -> O.State:
    """The library's state of group g as the oracle's State."""
    n = int(st.n_drafts[g])
    route = int(st.draft_route[g]) if n else 0
    fp, ft = st.fill_pos[g].cpu().numpy(), st.fill_tok[g].cpu().numpy()
    fills = [(int(fp[j]), int(ft[j])) for j in range(n)]
    return O.State(st.canvas[g, 0].cpu().numpy().astype(np.int32).copy(),
                   O.Drafts(route, fills), int(st.k_active[g]), bool(st.done[g]),
                   ws=int(st.n_ws_blocks[g]))


def assert_state_equals(st: B.State, g: int, want: O.State, info: O.RoundInfo, cfg: B.DecodeCfg,
                        where=""):
    """Bit-exact comparison of everything the decision step outputs for group g."""
    K = cfg.K
    got_accept = st.accept[g].cpu().numpy()[:K].tolist()
    assert got_accept == info.accept + [0] * (K - len(info.accept)), f"{where}: accept bits"
    assert int(st.winner[g]) == info.winner, f"{where}: winner"
    assert st.n_commit[g].cpu().numpy().tolist() == [info.n_base, info.n_plan, info.n_ar], f"{where}: commit counts"
    assert bool(st.done[g]) == want.done, f"{where}: done"
    assert np.array_equal(st.canvas[g, 0].cpu().numpy(), want.y), f"{where}: backbone canvas"
    assert int(st.n_drafts[g]) == want.drafts.n, f"{where}: number of drafts"
    if not want.done:
        assert int(st.k_active[g]) == want.k_active, f"{where}: active block"
        assert int(st.n_ws_blocks[g]) == want.ws, f"{where}: working-set blocks"
    if want.drafts.n:
        assert int(st.draft_route[g]) == want.drafts.route, f"{where}: route"
        fp, ft = st.fill_pos[g].cpu().numpy(), st.fill_tok[g].cpu().numpy()
        assert [(int(fp[j]), int(ft[j])) for j in range(want.drafts.n)] == want.drafts.fills, f"{where}: fills"
    X = O.branch_canvases(want.y, want.drafts)
    cv = st.canvas[g].cpu().numpy()
    for j in range(1 + K):
        ref = X[j] if j < len(X) else X[0]
        assert np.array_equal(cv[j], ref), f"{where}: canvas slot {j}"
