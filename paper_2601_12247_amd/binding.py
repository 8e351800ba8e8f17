"""ctypes binding of libpvf.so: the same calls as include/pvf.h, arguments marshalled from
torch tensors (device memory) and Python numbers.  No step of the method runs here.

The library must have been built (paper_2601_12247_amd/build.py); loading fails loudly
otherwise.  There is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpvf.so")

PVF_F32, PVF_BF16 = 0, 1
PVF_ROUTES_PLAN, PVF_ROUTES_AR, PVF_ROUTES_CAL, PVF_ROUTES_XRANDOM, PVF_ROUTES_XPLANNING = 1, 2, 4, 8, 16
PVF_ROUTE_NONE, PVF_ROUTE_PLAN, PVF_ROUTE_AR, PVF_ROUTE_CAL = 0, 1, 2, 3
ROUTE_NONE, ROUTE_PLAN, ROUTE_AR = 0, 1, 2
MAX_K = 32          # PVF_MAX_K of include/pvf.h
STATUS = {0: "PVF_OK", -1: "PVF_EINVAL", -2: "PVF_ESHAPE", -3: "PVF_ENOMEM", -4: "PVF_EHIP",
          -5: "PVF_ENOTIMPL"}

# every symbol include/pvf.h declares
EXPORTS = ["pvf_create", "pvf_destroy", "pvf_last_error", "pvf_workspace_bytes", "pvf_profile_begin",
           "pvf_profile_end", "pvf_forward",
           "pvf_epilogue", "pvf_round", "pvf_state_init", "pvf_decode", "pvf_stage1", "pvf_gemm",
           "pvf_gemm_swiglu", "pvf_rmsnorm", "pvf_rope_attention", "pvf_fill_normal", "pvf_entropy",
           "pvf_plan_vocab_select", "pvf_qkv_attention", "pvf_rope_attention_noalloc", "pvf_round_sync", "pvf_ctx_gemm",
           "pvf_ctx_gemm_swiglu"]


class PvfError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{STATUS.get(status, status)}: {msg}")
        self.status = status


class ModelCfgC(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("d_ff", C.c_int32), ("vocab", C.c_int32), ("dtype", C.c_int32),
                ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("mask_id", C.c_int32)]


class DecodeCfgC(C.Structure):
    _fields_ = [("tau_high", C.c_float), ("tau_plan_lo", C.c_float), ("tau_plan_hi", C.c_float),
                ("tau_ar_lo", C.c_float), ("logit_scale", C.c_float), ("K", C.c_int32),
                ("block_len", C.c_int32), ("prompt_len", C.c_int32), ("gen_len", C.c_int32),
                ("routes", C.c_int32), ("n_sparse", C.c_int32), ("seed", C.c_uint32), ("kv_cache", C.c_int32)]


class WeightsC(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("out_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("attn_norm", C.POINTER(C.c_void_p)), ("wqkv", C.POINTER(C.c_void_p)),
                ("wo", C.POINTER(C.c_void_p)), ("ffn_norm", C.POINTER(C.c_void_p)),
                ("w_gate_up", C.POINTER(C.c_void_p)), ("w_down", C.POINTER(C.c_void_p))]


class StateC(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("canvas", "n_drafts", "draft_route", "fill_pos", "fill_tok", "k_active", "n_ws_blocks",
                 "conf",
                 "tok", "accept", "winner", "n_commit", "done", "ent", "dh", "cal_n", "cal_m", "cal_a",
                 "cal_vig")]


class StatsC(C.Structure):
    _fields_ = [("rounds", C.c_int32), ("seq_forwards", C.c_int32), ("n_base", C.c_int64),
                ("n_plan", C.c_int64), ("n_ar", C.c_int64), ("drafts_proposed", C.c_int64),
                ("drafts_accepted", C.c_int64), ("ms_total", C.c_double)]


PROF_CATEGORIES = ("gemm", "attention", "stage1", "forward", "stage2")


class ProfileC(C.Structure):
    _fields_ = [("ms", C.c_double * 5), ("flops", C.c_double * 5), ("bytes", C.c_double * 5),
                ("launches", C.c_int64 * 5)]


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2601_12247_amd.build` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        L.pvf_last_error.restype = C.c_char_p
        L.pvf_last_error.argtypes = [C.c_void_p]
        L.pvf_workspace_bytes.restype = C.c_int64
        L.pvf_workspace_bytes.argtypes = [C.c_void_p]
        L.pvf_destroy.restype = None
        L.pvf_destroy.argtypes = [C.c_void_p]
        L.pvf_profile_begin.argtypes = [C.c_void_p]
        L.pvf_profile_end.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(ProfileC)]
        L.pvf_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(ModelCfgC), C.POINTER(WeightsC),
                                 C.c_int32, C.c_int32, C.c_int32]
        L.pvf_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                  C.c_void_p, C.c_int32, C.c_void_p]
        L.pvf_epilogue.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                   C.c_int32, C.c_int32, C.c_void_p, C.POINTER(DecodeCfgC),
                                   C.POINTER(StateC)]
        L.pvf_round.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                C.POINTER(DecodeCfgC), C.POINTER(StateC), C.c_int32]
        L.pvf_round_sync.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                     C.POINTER(DecodeCfgC), C.POINTER(StateC), C.c_int32, C.POINTER(C.c_int32)]
        L.pvf_state_init.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                     C.POINTER(DecodeCfgC), C.POINTER(StateC)]
        L.pvf_decode.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                 C.POINTER(DecodeCfgC), C.POINTER(StateC), C.c_void_p,
                                 C.POINTER(StatsC)]
        L.pvf_stage1.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int32,
                                 C.c_int32, C.c_float, C.c_void_p, C.c_void_p]
        L.pvf_entropy.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int32,
                                  C.c_int32, C.c_float, C.c_void_p]
        L.pvf_plan_vocab_select.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_int32, C.c_int32, C.c_uint32, C.c_uint32, C.c_float,
                                            C.c_float, C.c_void_p]
        L.pvf_gemm.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                               C.c_void_p, C.c_int32, C.c_int32, C.c_int32]
        L.pvf_ctx_gemm.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.c_void_p, C.c_int32, C.c_int32, C.c_int32]
        L.pvf_ctx_gemm_swiglu.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_int32, C.c_int32, C.c_int32]
        L.pvf_gemm_swiglu.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_int32, C.c_int32, C.c_int32]
        L.pvf_rmsnorm.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                  C.c_int32, C.c_int32, C.c_float]
        L.pvf_rope_attention.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32,
                                         C.c_int32, C.c_int32, C.c_int32, C.c_float]
        L.pvf_rope_attention_noalloc.argtypes = L.pvf_rope_attention.argtypes
        L.pvf_qkv_attention.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_float]
        L.pvf_fill_normal.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int64, C.c_uint64,
                                      C.c_float, C.c_float]
        for name in EXPORTS:
            fn = getattr(L, name)
            if name not in ("pvf_last_error", "pvf_workspace_bytes", "pvf_destroy"):
                fn.restype = C.c_int32
        _lib = L
    return _lib


def _check(status: int, ctx: Optional[int] = None) -> None:
    if status != 0:
        raise PvfError(status, lib().pvf_last_error(ctx).decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dtype_code(t: torch.dtype) -> int:
    if t == torch.float32:
        return PVF_F32
    if t == torch.bfloat16:
        return PVF_BF16
    raise TypeError(f"unsupported dtype {t}")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensor required"
    return t.data_ptr()


@dataclass
class DecodeCfg:
    block_len: int
    prompt_len: int
    gen_len: int
    tau_high: float = 0.9
    tau_plan_lo: float = 0.2
    tau_plan_hi: float = 0.65
    tau_ar_lo: float = 0.1
    logit_scale: float = 1.0
    K: int = 3
    routes: int = 3
    n_sparse: int = 0
    seed: int = 0
    kv_cache: int = 0

    @property
    def T(self) -> int:
        return self.prompt_len + self.gen_len

    @property
    def R(self) -> int:
        return min((4 if self.n_sparse > 0 else 2) * self.block_len, self.gen_len)

    def c(self) -> DecodeCfgC:
        return DecodeCfgC(self.tau_high, self.tau_plan_lo, self.tau_plan_hi, self.tau_ar_lo,
                          self.logit_scale, self.K, self.block_len, self.prompt_len, self.gen_len,
                          self.routes, self.n_sparse, self.seed, self.kv_cache)


class State:
    """Device buffers of pvf_state for G groups (allocated with torch)."""

    def __init__(self, G: int, cfg: DecodeCfg, device="cuda", vocab: Optional[int] = None):
        K, T, R = cfg.K, cfg.T, cfg.R
        i32 = dict(dtype=torch.int32, device=device)
        self.G, self.cfg = G, cfg
        self.canvas = torch.zeros(G, 1 + K, T, **i32)
        self.n_drafts = torch.zeros(G, **i32)
        self.draft_route = torch.zeros(G, **i32)
        self.fill_pos = torch.full((G, max(K, 1)), -1, **i32)
        self.fill_tok = torch.full((G, max(K, 1)), -1, **i32)
        self.k_active = torch.zeros(G, **i32)
        self.n_ws_blocks = torch.ones(G, **i32)
        self.conf = torch.zeros(G, 1 + K, R, dtype=torch.float32, device=device)
        self.tok = torch.zeros(G, 1 + K, R, **i32)
        self.accept = torch.zeros(G, max(K, 1), dtype=torch.uint8, device=device)
        self.winner = torch.zeros(G, **i32)
        self.n_commit = torch.zeros(G, 3, **i32)
        self.done = torch.zeros(G, **i32)
        # calibration members (App. A.2): allocated only for the calibration trajectory
        self.ent = self.dh = self.cal_n = self.cal_m = self.cal_a = self.cal_vig = None
        if cfg.routes & PVF_ROUTES_CAL:
            assert vocab is not None, "the calibration trajectory needs vocab for the token statistics"
            self.ent = torch.zeros(G, 1 + K, R, dtype=torch.float32, device=device)
            self.dh = torch.zeros(G, max(K, 1), dtype=torch.float64, device=device)
            self.cal_n = torch.zeros(vocab, **i32)
            self.cal_m = torch.zeros(vocab, **i32)
            self.cal_a = torch.zeros(vocab, **i32)
            self.cal_vig = torch.zeros(vocab, dtype=torch.float64, device=device)

    def c(self) -> StateC:
        return StateC(*[_ptr(getattr(self, n)) for n, _ in StateC._fields_])

    def live_seqs(self) -> int:
        """sum over live groups of 1 + n_drafts (synchronises)."""
        nd, dn = self.n_drafts.cpu(), self.done.cpu()
        return int(((1 + nd) * (1 - dn)).sum())


class Context:
    """pvf_ctx: keeps the weight tensors alive and owns the library workspace."""

    def __init__(self, n_layers: int, d_model: int, n_heads: int, d_ff: int, vocab: int,
                 mask_id: int, weights: Dict, max_seqs: int, max_T: int, max_rows: int,
                 rms_eps: float = 1e-5, rope_theta: float = 10000.0):
        self.weights = weights
        dt = weights["embed"].dtype
        self.dtype = dt
        self.vocab, self.mask_id, self.d_model = vocab, mask_id, d_model
        self.model = ModelCfgC(n_layers, d_model, n_heads, d_ff, vocab, _dtype_code(dt), rms_eps,
                               rope_theta, mask_id)
        layers: List[Dict] = weights["layers"]
        assert len(layers) == n_layers

        def arr(name):
            a = (C.c_void_p * n_layers)(*[_ptr(l[name]) for l in layers])
            return a

        self._arrs = {n: arr(n) for n in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down")}
        wc = WeightsC(_ptr(weights["embed"]), _ptr(weights["out_head"]), _ptr(weights["final_norm"]),
                      *[C.cast(self._arrs[n], C.POINTER(C.c_void_p)) for n in
                        ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down")])
        h = C.c_void_p()
        _check(lib().pvf_create(C.byref(h), C.byref(self.model), C.byref(wc), max_seqs, max_T, max_rows))
        self.handle = h

    def close(self):
        if getattr(self, "handle", None):
            lib().pvf_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def workspace_bytes(self) -> int:
        return lib().pvf_workspace_bytes(self.handle)

    def profile_begin(self) -> None:
        _check(lib().pvf_profile_begin(self.handle), self.handle)

    def profile_end(self) -> Dict[str, Dict[str, float]]:
        p = ProfileC()
        _check(lib().pvf_profile_end(self.handle, _stream(), C.byref(p)), self.handle)
        return {name: {"ms": p.ms[i], "flops": p.flops[i], "bytes": p.bytes[i], "launches": p.launches[i]}
                for i, name in enumerate(PROF_CATEGORIES)}

    # ---- GEMMs as the context launches them (weight-streaming kernels for few rows) ----
    def gemm(self, A: torch.Tensor, W: torch.Tensor, residual: Optional[torch.Tensor] = None,
             out: Optional[torch.Tensor] = None) -> torch.Tensor:
        M, K = A.shape
        N = W.shape[0]
        assert W.shape[1] == K and A.dtype == self.dtype
        if out is None:
            out = torch.empty(M, N, dtype=A.dtype, device=A.device)
        _check(lib().pvf_ctx_gemm(self.handle, _stream(), _ptr(A), _ptr(W), _ptr(out), _ptr(residual), M, N, K),
               self.handle)
        return out

    def gemm_swiglu(self, A: torch.Tensor, W: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        M, K = A.shape
        ff = W.shape[0] // 2
        if out is None:
            out = torch.empty(M, ff, dtype=A.dtype, device=A.device)
        _check(lib().pvf_ctx_gemm_swiglu(self.handle, _stream(), _ptr(A), _ptr(W), _ptr(out), M, ff, K), self.handle)
        return out

    # ---- the four calls -------------------------------------------------------------
    def forward(self, tokens: torch.Tensor, row_pos: torch.Tensor) -> torch.Tensor:
        S, T = tokens.shape
        R = row_pos.shape[1]
        logits = torch.empty(S, R, self.vocab, dtype=self.dtype, device=tokens.device)
        _check(lib().pvf_forward(self.handle, _stream(), _ptr(tokens), S, T, _ptr(row_pos), R,
                                 _ptr(logits)), self.handle)
        return logits

    def round(self, state: State, plan_bitmap: torch.Tensor, n_seq: int = 0) -> None:
        cfgc, stc = state.cfg.c(), state.c()
        _check(lib().pvf_round(self.handle, _stream(), state.G, _ptr(plan_bitmap), C.byref(cfgc),
                               C.byref(stc), n_seq), self.handle)

    def round_sync(self, state: State, plan_bitmap: torch.Tensor, n_seq: int = 0):
        """pvf_round_sync: one round and its status words; returns a list of G tuples
        (done, n_drafts, committed by threshold, by planning, by AR)."""
        cfgc, stc = state.cfg.c(), state.c()
        buf = (C.c_int32 * (5 * state.G))()
        _check(lib().pvf_round_sync(self.handle, _stream(), state.G, _ptr(plan_bitmap), C.byref(cfgc),
                                    C.byref(stc), n_seq, buf), self.handle)
        return [tuple(buf[5 * g: 5 * g + 5]) for g in range(state.G)]

    def state_init(self, state: State, prompt: torch.Tensor) -> None:
        cfgc, stc = state.cfg.c(), state.c()
        _check(lib().pvf_state_init(self.handle, _stream(), _ptr(prompt), state.G, C.byref(cfgc),
                                    C.byref(stc)), self.handle)

    def decode(self, state: State, prompt: torch.Tensor, plan_bitmap: torch.Tensor):
        cfgc, stc, stats = state.cfg.c(), state.c(), StatsC()
        out = torch.empty(state.G, state.cfg.T, dtype=torch.int32, device=prompt.device)
        _check(lib().pvf_decode(self.handle, _stream(), _ptr(prompt), state.G, _ptr(plan_bitmap),
                                C.byref(cfgc), C.byref(stc), _ptr(out), C.byref(stats)), self.handle)
        return out, stats


def epilogue(logits: torch.Tensor, state: State, plan_bitmap: torch.Tensor, vocab: int,
             mask_id: int, ctx: Optional[Context] = None) -> None:
    """pvf_epilogue over logits [G, 1+K, R, V]."""
    cfgc, stc = state.cfg.c(), state.c()
    h = ctx.handle if ctx is not None else None
    _check(lib().pvf_epilogue(h, _stream(), _ptr(logits), _dtype_code(logits.dtype), state.G, vocab,
                              mask_id, _ptr(plan_bitmap), C.byref(cfgc), C.byref(stc)), h)


# ---- building blocks ---------------------------------------------------------------------
def stage1(logits: torch.Tensor, mask_id: int, logit_scale: float, conf: Optional[torch.Tensor] = None,
           tok: Optional[torch.Tensor] = None):
    n, V = logits.shape
    if conf is None:
        conf = torch.empty(n, dtype=torch.float32, device=logits.device)
    if tok is None:
        tok = torch.empty(n, dtype=torch.int32, device=logits.device)
    _check(lib().pvf_stage1(_stream(), _ptr(logits), _dtype_code(logits.dtype), n, V, mask_id,
                            logit_scale, _ptr(conf), _ptr(tok)))
    return conf, tok


def entropy(logits: torch.Tensor, mask_id: int, logit_scale: float = 1.0) -> torch.Tensor:
    """H_i (nats) of softmax(logit_scale * logits[i]) over all ids but mask_id; logits [n, V]."""
    n, V = logits.shape
    ent = torch.empty(n, dtype=torch.float32, device=logits.device)
    _check(lib().pvf_entropy(_stream(), _ptr(logits), _dtype_code(logits.dtype), n, V, mask_id,
                             logit_scale, _ptr(ent)))
    return ent


def plan_vocab_select(cal_n: torch.Tensor, cal_m: torch.Tensor, cal_a: torch.Tensor, cal_vig: torch.Tensor,
                      mask_id: int, n_min: int = 50, m_min: int = 20, rho_ver: float = 0.9,
                      gamma_vig: float = 0.03) -> torch.Tensor:
    """Filtering rule of App. A.2 on the accumulated token statistics -> planning bitmap."""
    V = cal_n.numel()
    bitmap = torch.empty((V + 31) // 32, dtype=torch.int32, device=cal_n.device)
    _check(lib().pvf_plan_vocab_select(_stream(), _ptr(cal_n), _ptr(cal_m), _ptr(cal_a), _ptr(cal_vig), V,
                                       mask_id, n_min, m_min, rho_ver, gamma_vig, _ptr(bitmap)))
    return bitmap


def gemm(A: torch.Tensor, W: torch.Tensor, residual: Optional[torch.Tensor] = None,
         out: Optional[torch.Tensor] = None) -> torch.Tensor:
    M, K = A.shape
    N = W.shape[0]
    assert W.shape[1] == K
    if out is None:
        out = torch.empty(M, N, dtype=A.dtype, device=A.device)
    _check(lib().pvf_gemm(_stream(), _dtype_code(A.dtype), _ptr(A), _ptr(W), _ptr(out),
                          _ptr(residual), M, N, K))
    return out


def gemm_swiglu(A: torch.Tensor, W: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    M, K = A.shape
    ff = W.shape[0] // 2
    if out is None:
        out = torch.empty(M, ff, dtype=A.dtype, device=A.device)
    _check(lib().pvf_gemm_swiglu(_stream(), _dtype_code(A.dtype), _ptr(A), _ptr(W), _ptr(out), M, ff, K))
    return out


def rmsnorm(x: torch.Tensor, gain: torch.Tensor, eps: float) -> torch.Tensor:
    M, d = x.shape
    out = torch.empty_like(x)
    _check(lib().pvf_rmsnorm(_stream(), _dtype_code(x.dtype), _ptr(x), _ptr(gain), _ptr(out), M, d, eps))
    return out


def rope_attention(qkv: torch.Tensor, S: int, T: int, n_heads: int, d_head: int,
                   rope_theta: float) -> torch.Tensor:
    """qkv [S*T, 3*d] is rotated in place; returns the attention output [S*T, d]."""
    assert qkv.shape == (S * T, 3 * n_heads * d_head) and qkv.is_contiguous()
    out = torch.empty(S * T, n_heads * d_head, dtype=qkv.dtype, device=qkv.device)
    _check(lib().pvf_rope_attention(_stream(), _dtype_code(qkv.dtype), _ptr(qkv), _ptr(out), S, T,
                                    n_heads, d_head, rope_theta))
    return out


def rope_attention_noalloc(qkv: torch.Tensor, out: torch.Tensor, S: int, T: int, n_heads: int, d_head: int,
                           rope_theta: float) -> torch.Tensor:
    """pvf_rope_attention_noalloc: like rope_attention, into the caller's `out`; the library allocates nothing."""
    assert qkv.shape == (S * T, 3 * n_heads * d_head) and qkv.is_contiguous()
    assert out.shape == (S * T, n_heads * d_head) and out.dtype == qkv.dtype
    _check(lib().pvf_rope_attention_noalloc(_stream(), _dtype_code(qkv.dtype), _ptr(qkv), _ptr(out), S, T,
                                            n_heads, d_head, rope_theta))
    return out


def qkv_attention(x: torch.Tensor, wqkv: torch.Tensor, S: int, T: int, n_heads: int, d_head: int,
                  rope_theta: float, vt: Optional[torch.Tensor] = None):
    """(qkv [S*T, 3d] with q, k rotated; attention output [S*T, d]) of x [S*T, d]; vt [S, H, d_head, T]
    (optional) receives the key-contiguous copy of v where the fused projection epilogue writes one."""
    d = n_heads * d_head
    assert x.shape == (S * T, d) and wqkv.shape == (3 * d, d) and x.is_contiguous() and wqkv.is_contiguous()
    assert wqkv.dtype == x.dtype
    qkv = torch.empty(S * T, 3 * d, dtype=x.dtype, device=x.device)
    out = torch.empty(S * T, d, dtype=x.dtype, device=x.device)
    if vt is not None:
        assert vt.shape == (S, n_heads, d_head, T) and vt.dtype == x.dtype
    _check(lib().pvf_qkv_attention(_stream(), _dtype_code(x.dtype), _ptr(x), _ptr(wqkv), _ptr(qkv), _ptr(vt), _ptr(out),
                                   S, T, n_heads, d_head, rope_theta))
    return qkv, out


def fill_normal(dst: torch.Tensor, seed: int, mean: float = 0.0, std: float = 0.02) -> None:
    _check(lib().pvf_fill_normal(_stream(), _dtype_code(dst.dtype), _ptr(dst), dst.numel(), seed,
                                 mean, std))
