// C-ABI entry points of libpvf: argument validation, workspace, and the order of launches of
// one PVF round (Algorithm 1 with one batched forward per round) and of the decode loop.
#include "common.h"

#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

struct pvf_ctx {
  pvf_model_cfg model;
  pvf_weights w;                       // top-level pointers
  std::vector<const void *> attn_norm, wqkv, wo, ffn_norm, w_gate_up, w_down;
  int max_seqs = 0, max_T = 0, max_rows = 0;
  size_t esize = 4;
  // workspace (device)
  void *h = nullptr, *xn = nullptr, *qkv = nullptr, *att = nullptr, *act = nullptr, *vt = nullptr;
  void *hrows = nullptr, *logits = nullptr;
  float *splitk_ws = nullptr;          // float32 partial sums of the split-K GEMMs (bf16 contexts)
  size_t splitk_floats = 0;
  // RMSNorm folded into the projections (bf16, launches above the split-K range): row sums of squares
  // [d / 128 slots][max rows], and wqkv / w_gate_up with the norm gain folded in (the caller's matrices
  // themselves where every gain is 1)
  float *row_ss = nullptr;
  std::vector<const void *> wqkv_f, w_gate_up_f;
  std::vector<void *> folded_owned;
  int32_t *seq_slot = nullptr, *row_pos = nullptr;
  float2 *cos_sin = nullptr;           // [max_T, d_head/2]
  int32_t *status_host = nullptr;      // pinned, 5*G words per round: done, n_drafts, n_commit[3] of each group
  int32_t *status_dev = nullptr;       // the same words, packed on the device by one small kernel
  int status_cap = 0;
  // block-level K/V cache (decode_cfg.kv_cache): [G][n_layers][T][d] each, row-major like the
  // k / v thirds of the qkv buffer; cache_block[g] = active block the cache of group g is for
  void *kcache = nullptr, *vcache = nullptr;
  int cache_G = 0, cache_T = 0;
  bool cache_vt = false;               // values cached key-contiguous [head][d_head][T] (MFMA window attention)
  std::vector<int> cache_block;
  const void *cache_canvas = nullptr;  // the state (its canvas buffer) the caches were made for
  int32_t *seq_host = nullptr;         // pinned staging of the round's sequence list
  int seq_host_cap = 0;
  int64_t ws_bytes = 0;
  char err[512] = {0};
  // optional per-kernel timing (pvf_profile_begin / pvf_profile_end)
  struct ProfRec { int cat; double flops, bytes; hipEvent_t e0, e1; };
  bool prof_on = false;
  std::vector<ProfRec> prof;
  std::vector<hipEvent_t> ev_pool;
  size_t ev_used = 0;
};

namespace pvf {

static thread_local char g_err[512] = {0};

void set_error(pvf_ctx *ctx, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(ctx ? ctx->err : g_err, 512, fmt, ap);
  va_end(ap);
}

// ---- optional timing of a launch with a pair of HIP events on the launch stream ----------
struct ProfScope {
  pvf_ctx *c; hipStream_t s; bool on; hipEvent_t e1 = nullptr;
  ProfScope(pvf_ctx *ctx, hipStream_t st, int cat, double flops, double bytes) : c(ctx), s(st), on(ctx && ctx->prof_on) {
    if (!on) return;
    auto get = [&]() {
      if (c->ev_used == c->ev_pool.size()) {
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return (hipEvent_t) nullptr;
        c->ev_pool.push_back(e);
      }
      return c->ev_pool[c->ev_used++];
    };
    hipEvent_t e0 = get();
    e1 = get();
    if (!e0 || !e1) { on = false; return; }
    (void)hipEventRecord(e0, s);
    c->prof.push_back({cat, flops, bytes, e0, e1});
  }
  ~ProfScope() { if (on) (void)hipEventRecord(e1, s); }
};

// ---- dispatch between the MFMA kernels and the plain ones -------------------------------
pvf_status launch_gemm_simple(pvf_ctx *, hipStream_t, int, GemmEpilogue, const void *, const void *,
                              void *, const void *, int, int, int);
pvf_status launch_attention_simple(pvf_ctx *, hipStream_t, int, const void *, void *, int, int, int, int);
bool gemm_mfma_supported(int dtype, GemmEpilogue epi, int M, int N, int K);
pvf_status launch_gemm_mfma(pvf_ctx *, hipStream_t, GemmEpilogue, const void *, const void *, void *,
                            const void *, int, int, int, const NormArgs *na = nullptr);
int gemm_mfma_norm_slots(GemmEpilogue epi, int M, int N, int K);
bool gemm_mfma_splitk_supported(int dtype, GemmEpilogue epi, int M, int N, int K, size_t ws_floats);
pvf_status launch_gemm_mfma_splitk(pvf_ctx *, hipStream_t, GemmEpilogue, const void *, const void *, void *, const void *,
                                   int, int, int, float *, size_t);
bool gemm_mfma_qkv_rope_supported(int dtype, int M, int N, int K, int T, int H);
pvf_status launch_gemm_mfma_qkv_rope(pvf_ctx *, hipStream_t, const void *, const void *, void *, void *, const float2 *,
                                     int, int, int, int, int, bool store_v, const NormArgs *na = nullptr);
bool attention_mfma_supported(int dtype, int T, int d_head);
pvf_status launch_attention_mfma(pvf_ctx *, hipStream_t, const void *, const void *, void *, int, int, int);
pvf_status launch_rope_vt(pvf_ctx *, hipStream_t, void *, void *, int, int, int, const float2 *);
bool attention_window_mfma_supported(int dtype, int T, int d_head, int R, int block_len, int prompt_len);
pvf_status launch_rope_vt_rows(pvf_ctx *, hipStream_t, void *, void *, const int32_t *, int, int, int, int, const float2 *);
pvf_status launch_attention_window_mfma(pvf_ctx *, hipStream_t, const void *, const void *, const void *, const void *,
                                        int64_t, const int32_t *, const int32_t *, int, int, int, int, int, int, int, void *);

pvf_status launch_gemm_mfma_splitk_partial(pvf_ctx *, hipStream_t, const void *, const void *, int, int, int, float *, size_t, int *);

static bool fold_norm_enabled() {       // PVF_FOLD_NORM=0: keep the norms as launches of their own (tuning runs)
  static const bool v = [] { const char *e = getenv("PVF_FOLD_NORM"); return !(e && e[0] == '0'); }();
  return v;
}

static bool force_simple() {
  static const bool v = [] { const char *e = getenv("PVF_FORCE_SIMPLE"); return e && e[0] == '1'; }();
  return v;
}

pvf_status launch_gemm(pvf_ctx *ctx, hipStream_t s, int dtype, GemmEpilogue epi, const void *A,
                       const void *W, void *C, const void *residual, int M, int N, int K) {
  if (!force_simple() && ctx && ctx->splitk_ws && gemm_mfma_splitk_supported(dtype, epi, M, N, K, ctx->splitk_floats))
    return launch_gemm_mfma_splitk(ctx, s, epi, A, W, C, residual, M, N, K, ctx->splitk_ws, ctx->splitk_floats);
  if (!force_simple() && gemm_mfma_supported(dtype, epi, M, N, K))
    return launch_gemm_mfma(ctx, s, epi, A, W, C, residual, M, N, K);
  return launch_gemm_simple(ctx, s, dtype, epi, A, W, C, residual, M, N, K);
}

static bool use_attention_mfma(int dtype, int T, int d_head) {
  return !force_simple() && attention_mfma_supported(dtype, T, d_head);
}

// Rotary embedding of q, k (in place) followed by attention.  vt: scratch of S*T*d elements,
// needed only by the MFMA path (key-contiguous copy of v).
static pvf_status launch_rope_attention(pvf_ctx *ctx, hipStream_t s, int dtype, void *qkv, void *vt,
                                        void *out, int S, int T, int n_heads, int d_head,
                                        const float2 *cos_sin) {
  pvf_status st;
  if (use_attention_mfma(dtype, T, d_head)) {
    if ((st = launch_rope_vt(ctx, s, qkv, vt, S, T, n_heads, cos_sin)) != PVF_OK) return st;
    return launch_attention_mfma(ctx, s, qkv, vt, out, S, T, n_heads);
  }
  if ((st = launch_rope(ctx, s, dtype, qkv, S * T, T, n_heads, d_head, cos_sin)) != PVF_OK) return st;
  return launch_attention_simple(ctx, s, dtype, qkv, out, S, T, n_heads, d_head);
}

// ---- validation -----------------------------------------------------------------------
static pvf_status check_decode_cfg(pvf_ctx *ctx, const pvf_decode_cfg *c, int vocab, int mask_id) {
  PVF_REQUIRE(ctx, c != nullptr, PVF_EINVAL, "decode cfg is NULL");
  PVF_REQUIRE(ctx, c->K >= 0 && c->K <= PVF_MAX_K, PVF_EINVAL, "K=%d outside [0,%d]", c->K, PVF_MAX_K);
  PVF_REQUIRE(ctx, c->block_len > 0 && c->gen_len > 0 && c->prompt_len >= 0, PVF_EINVAL,
              "block_len=%d gen_len=%d prompt_len=%d", c->block_len, c->gen_len, c->prompt_len);
  PVF_REQUIRE(ctx, c->gen_len % c->block_len == 0, PVF_EINVAL, "gen_len %% block_len != 0 (%d, %d)", c->gen_len, c->block_len);
  PVF_REQUIRE(ctx, c->tau_plan_lo <= c->tau_plan_hi && c->tau_plan_hi <= c->tau_high, PVF_EINVAL,
              "need tau_plan_lo <= tau_plan_hi <= tau_high (%g, %g, %g)", c->tau_plan_lo, c->tau_plan_hi, c->tau_high);
  PVF_REQUIRE(ctx, c->logit_scale > 0.f && std::isfinite(c->logit_scale), PVF_EINVAL, "logit_scale=%g must be positive", c->logit_scale);
  PVF_REQUIRE(ctx, (c->routes & ~31) == 0, PVF_EINVAL, "routes=%d has unknown bits", c->routes);
  PVF_REQUIRE(ctx, !(c->routes & (PVF_ROUTES_XRANDOM | PVF_ROUTES_XPLANNING)) || c->routes == PVF_ROUTES_XRANDOM ||
                  c->routes == PVF_ROUTES_XPLANNING, PVF_EINVAL,
              "routes=%d: an ablation decoder excludes every other route", c->routes);
  PVF_REQUIRE(ctx, !(c->routes & PVF_ROUTES_CAL) || c->routes == PVF_ROUTES_CAL, PVF_EINVAL,
              "routes=%d: the calibration trajectory excludes the planning and AR routes", c->routes);
  PVF_REQUIRE(ctx, c->n_sparse >= 0, PVF_EINVAL, "n_sparse=%d must be >= 0", c->n_sparse);
  PVF_REQUIRE(ctx, c->kv_cache == 0 || c->kv_cache == 1, PVF_EINVAL, "kv_cache=%d must be 0 or 1", c->kv_cache);
  PVF_REQUIRE(ctx, mask_id >= 0 && mask_id < vocab, PVF_EINVAL, "mask_id=%d outside [0,%d)", mask_id, vocab);
  PVF_REQUIRE(ctx, (int64_t)(1 + c->K) * window_rows(*c) <= PVF_MAX_SUMMARIES, PVF_ESHAPE,
              "(1+K)*R = %lld exceeds %d", (long long)(1 + c->K) * window_rows(*c), PVF_MAX_SUMMARIES);
  return PVF_OK;
}

static pvf_status check_state(pvf_ctx *ctx, const pvf_state *st, const pvf_decode_cfg *cfg) {
  PVF_REQUIRE(ctx, st != nullptr, PVF_EINVAL, "state is NULL");
  if (cfg->routes & PVF_ROUTES_CAL)
    PVF_REQUIRE(ctx, st->ent && st->dh && st->cal_n && st->cal_m && st->cal_a && st->cal_vig, PVF_EINVAL,
                "calibration needs the ent, dh and cal_* members of the state");
  PVF_REQUIRE(ctx, st->canvas && st->n_drafts && st->draft_route && st->fill_pos && st->fill_tok &&
                  st->k_active && st->n_ws_blocks && st->conf && st->tok && st->accept && st->winner && st->n_commit && st->done,
              PVF_EINVAL, "state has a NULL member");
  return PVF_OK;
}

}  // namespace pvf

using namespace pvf;

// =========================================================================================
// context
// =========================================================================================
static void free_ws(pvf_ctx *c) {
  for (hipEvent_t e : c->ev_pool) (void)hipEventDestroy(e);
  c->ev_pool.clear();
  void *ptrs[] = {c->h, c->xn, c->qkv, c->att, c->act, c->vt, c->hrows, c->logits, c->seq_slot, c->row_pos, c->cos_sin,
                  c->kcache, c->vcache, c->splitk_ws, c->status_dev, c->row_ss};
  for (void *p : ptrs) if (p) (void)hipFree(p);
  for (void *p : c->folded_owned) if (p) (void)hipFree(p);
  c->folded_owned.clear();
  if (c->status_host) (void)hipHostFree(c->status_host);
  if (c->seq_host) (void)hipHostFree(c->seq_host);
}

extern "C" pvf_status pvf_create(pvf_ctx **out, const pvf_model_cfg *m, const pvf_weights *w,
                                 int32_t max_seqs, int32_t max_T, int32_t max_rows) {
  PVF_REQUIRE(nullptr, out && m && w, PVF_EINVAL, "pvf_create: NULL argument");
  *out = nullptr;
  PVF_REQUIRE(nullptr, m->dtype == PVF_F32 || m->dtype == PVF_BF16, PVF_EINVAL, "dtype=%d", m->dtype);
  PVF_REQUIRE(nullptr, m->n_layers > 0 && m->d_model > 0 && m->n_heads > 0 && m->d_ff > 0 && m->vocab > 1,
              PVF_EINVAL, "non-positive model dimension");
  PVF_REQUIRE(nullptr, m->d_model % m->n_heads == 0 && (m->d_model / m->n_heads) % 2 == 0, PVF_EINVAL,
              "d_model=%d must split into n_heads=%d even-sized heads", m->d_model, m->n_heads);
  PVF_REQUIRE(nullptr, m->d_model % 8 == 0 && m->d_ff % 8 == 0, PVF_EINVAL, "d_model and d_ff must be multiples of 8");
  PVF_REQUIRE(nullptr, m->mask_id >= 0 && m->mask_id < m->vocab, PVF_EINVAL, "mask_id=%d outside [0,%d)", m->mask_id, m->vocab);
  PVF_REQUIRE(nullptr, m->rms_eps >= 0.f && m->rope_theta > 0.f, PVF_EINVAL, "rms_eps / rope_theta");
  PVF_REQUIRE(nullptr, max_seqs > 0 && max_T > 0 && max_rows > 0 && max_rows <= max_T, PVF_EINVAL,
              "max_seqs=%d max_T=%d max_rows=%d", max_seqs, max_T, max_rows);
  PVF_REQUIRE(nullptr, w->embed && w->out_head && w->final_norm && w->attn_norm && w->wqkv && w->wo &&
                  w->ffn_norm && w->w_gate_up && w->w_down, PVF_EINVAL, "weights has a NULL member");
  for (int l = 0; l < m->n_layers; ++l)
    PVF_REQUIRE(nullptr, w->attn_norm[l] && w->wqkv[l] && w->wo[l] && w->ffn_norm[l] && w->w_gate_up[l] && w->w_down[l],
                PVF_EINVAL, "layer %d has a NULL weight", l);

  pvf_ctx *c = new (std::nothrow) pvf_ctx();
  PVF_REQUIRE(nullptr, c != nullptr, PVF_ENOMEM, "host allocation failed");
  c->model = *m;
  c->w = *w;
  const int L = m->n_layers;
  c->attn_norm.assign(w->attn_norm, w->attn_norm + L);
  c->wqkv.assign(w->wqkv, w->wqkv + L);
  c->wo.assign(w->wo, w->wo + L);
  c->ffn_norm.assign(w->ffn_norm, w->ffn_norm + L);
  c->w_gate_up.assign(w->w_gate_up, w->w_gate_up + L);
  c->w_down.assign(w->w_down, w->w_down + L);
  c->max_seqs = max_seqs; c->max_T = max_T; c->max_rows = max_rows;
  c->esize = m->dtype == PVF_BF16 ? 2 : 4;

  const int64_t M = (int64_t)max_seqs * max_T, d = m->d_model, ff = m->d_ff;
  const int64_t rows = (int64_t)max_seqs * max_rows;
  const int half = m->d_model / m->n_heads / 2;
  struct { void **p; int64_t bytes; } req[] = {
      {&c->h, M * d * (int64_t)c->esize},       {&c->xn, M * d * (int64_t)c->esize},
      {&c->qkv, M * 3 * d * (int64_t)c->esize}, {&c->att, M * d * (int64_t)c->esize},
      {&c->vt, M * d * (int64_t)c->esize},
      {&c->act, M * ff * (int64_t)c->esize},    {&c->hrows, rows * d * (int64_t)c->esize},
      {&c->logits, rows * (int64_t)m->vocab * (int64_t)c->esize},
      {(void **)&c->seq_slot, (int64_t)max_seqs * 4}, {(void **)&c->row_pos, rows * 4},
      {(void **)&c->cos_sin, (int64_t)max_T * half * 8},
      // partial sums of the few-row GEMMs: rows x splits x row length, at most 384 x 49152 floats (up to 384 rows
      // every layer GEMM may split, from there to 640 rows only those with rows of 4096 or less)
      {(void **)&c->splitk_ws, m->dtype == PVF_BF16 ? (int64_t)384 * 49152 * 4 : 0},
      {(void **)&c->row_ss, m->dtype == PVF_BF16 && d % 128 == 0 ? (d / 128) * M * 4 : 0}};
  for (auto &r : req) {
    if (r.bytes == 0) continue;
    hipError_t e = hipMalloc(r.p, (size_t)r.bytes);
    if (e != hipSuccess) {
      set_error(nullptr, "pvf_create: hipMalloc(%lld bytes) failed: %s", (long long)r.bytes, hipGetErrorString(e));
      free_ws(c);
      delete c;
      return e == hipErrorOutOfMemory ? PVF_ENOMEM : PVF_EHIP;
    }
    c->ws_bytes += r.bytes;
  }
  c->splitk_floats = c->splitk_ws ? (size_t)384 * 49152 : 0;
  // rotary table in double precision on the host: angle = pos * theta^(-2i/d_head)
  {
    std::vector<float2> tab((size_t)max_T * half);
    const int dh = 2 * half;
    for (int i = 0; i < half; ++i) {
      const double inv = std::pow((double)m->rope_theta, -2.0 * i / dh);
      for (int t = 0; t < max_T; ++t) {
        const double a = (double)t * inv;
        tab[(size_t)t * half + i] = make_float2((float)std::cos(a), (float)std::sin(a));
      }
    }
    hipError_t e = hipMemcpy(c->cos_sin, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
      set_error(nullptr, "pvf_create: rotary table upload failed: %s", hipGetErrorString(e));
      free_ws(c);
      delete c;
      return PVF_EHIP;
    }
  }
  // Gains folded into the projections that read a normed stream: w'[n][k] = bf16(w[n][k] * gain[k]).  A layer
  // whose gains are all 1 keeps the caller's matrix.
  if (c->row_ss) {
    std::vector<uint16_t> g((size_t)d);
    auto fold = [&](const void *w, const void *gain, int64_t rows, const void **dst) -> pvf_status {
      PVF_HIP_CHECK(nullptr, hipMemcpy(g.data(), gain, (size_t)d * 2, hipMemcpyDeviceToHost));
      bool ones = true;
      for (int64_t i = 0; i < d; ++i) ones = ones && g[(size_t)i] == 0x3f80;
      if (ones) { *dst = w; return PVF_OK; }
      void *p = nullptr;
      hipError_t e = hipMalloc(&p, (size_t)rows * d * 2);
      PVF_REQUIRE(nullptr, e == hipSuccess, e == hipErrorOutOfMemory ? PVF_ENOMEM : PVF_EHIP,
                  "pvf_create: hipMalloc(%lld bytes) for a gain-folded matrix failed: %s", (long long)rows * d * 2, hipGetErrorString(e));
      c->folded_owned.push_back(p);
      c->ws_bytes += rows * d * 2;
      *dst = p;
      return launch_fold_gain(nullptr, nullptr, w, gain, p, rows, (int)d);
    };
    c->wqkv_f.assign(L, nullptr);
    c->w_gate_up_f.assign(L, nullptr);
    for (int l = 0; l < L; ++l) {
      pvf_status st = fold(c->wqkv[l], c->attn_norm[l], 3 * d, &c->wqkv_f[l]);
      if (st == PVF_OK) st = fold(c->w_gate_up[l], c->ffn_norm[l], 2 * ff, &c->w_gate_up_f[l]);
      if (st != PVF_OK) { free_ws(c); delete c; return st; }
    }
    hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) {
      set_error(nullptr, "pvf_create: folding the norm gains failed: %s", hipGetErrorString(e));
      free_ws(c); delete c;
      return PVF_EHIP;
    }
  }
  *out = c;
  return PVF_OK;
}

extern "C" void pvf_destroy(pvf_ctx *ctx) {
  if (!ctx) return;
  free_ws(ctx);
  delete ctx;
}

extern "C" const char *pvf_last_error(const pvf_ctx *ctx) { return ctx ? ctx->err : pvf::g_err; }
extern "C" int64_t pvf_workspace_bytes(const pvf_ctx *ctx) { return ctx ? ctx->ws_bytes : 0; }

// =========================================================================================
// forward
// =========================================================================================
// tokens: [*, T] rows addressed through seq_slot (NULL = identity).  Writes logits [S, R, V].
// capture_spg > 0: the rotated keys and the values of every backbone canvas of the batch (slot
// index divisible by capture_spg) are stored into the context's K/V cache after each layer.
static pvf_status forward_impl(pvf_ctx *c, hipStream_t s, const int32_t *tokens,
                               const int32_t *seq_slot, int S, int T, const int32_t *row_pos,
                               int R, void *logits, int capture_spg = 0) {
  const pvf_model_cfg &m = c->model;
  const int d = m.d_model, H = m.n_heads, dh = d / H, ff = m.d_ff, dt = m.dtype;
  const int M = S * T;
  pvf_status st;
#define RUN(x) do { st = (x); if (st != PVF_OK) return st; } while (0)
#define RUN_GEMM(epi, A, W, C, res, Mm, Nn, Kk)                                                   \
  do {                                                                                            \
    ProfScope ps(c, s, PVF_PROF_GEMM, 2.0 * (Mm) * (double)(Nn) * (Kk) * ((epi) == kEpiSwiglu ? 2 : 1),   \
                 (double)c->esize * ((double)(Mm) * (Kk) + (double)(Nn) * (Kk) * ((epi) == kEpiSwiglu ? 2 : 1) + \
                                     (double)(Mm) * (Nn) * ((epi) == kEpiResidual ? 2 : 1)));             \
    RUN(launch_gemm(c, s, dt, epi, A, W, C, res, Mm, Nn, Kk));                                    \
  } while (0)
  const bool fused_rope = use_attention_mfma(dt, T, dh) && gemm_mfma_qkv_rope_supported(dt, M, 3 * d, d, T, H);
  // Above the split-K range the two norms of a layer are folded into the projections around them: O and down
  // write each row's sum of squares beside h, QKV and gate/up read h itself (gains folded into their weights)
  // and scale their accumulators by 1 / rms.  The xn buffer and the 2 x n_layers norm launches disappear.
  const int slots_o = gemm_mfma_norm_slots(kEpiResidual, M, d, d), slots_down = gemm_mfma_norm_slots(kEpiResidual, M, d, ff);
  const bool fold_norm = !force_simple() && fold_norm_enabled() && fused_rope && c->row_ss && M > 640 && slots_o > 0 && slots_down > 0 &&
                         slots_o <= d / 128 && slots_down <= d / 128 &&
                         gemm_mfma_norm_slots(kEpiQkvRope, M, 3 * d, d) > 0 && gemm_mfma_norm_slots(kEpiSwiglu, M, ff, d) > 0;
  // Up to 640 rows O and down split K: one kernel then adds their partial tiles and the residual and norms the
  // row for the next projection (instead of a reduce kernel followed by a norm kernel).
  const bool split_norm_o_down = !fold_norm && !force_simple() && c->splitk_ws && reduce_residual_rmsnorm_supported(dt, d) &&
                                 gemm_mfma_splitk_supported(dt, kEpiResidual, M, d, d, c->splitk_floats) &&
                                 gemm_mfma_splitk_supported(dt, kEpiResidual, M, d, ff, c->splitk_floats);
  // h += A W^T; with_norm: xn = RMSNorm(h) * gain as well
  auto project_residual_norm = [&](const void *A, const void *W, int Kk, const void *gain, void *out, bool with_norm) -> pvf_status {
    if (split_norm_o_down && with_norm) {
      int splits = 0;
      ProfScope ps(c, s, PVF_PROF_GEMM, 2.0 * M * (double)d * Kk, (double)c->esize * ((double)M * Kk + (double)d * Kk + 2.0 * M * d));
      RUN(launch_gemm_mfma_splitk_partial(c, s, A, W, M, d, Kk, c->splitk_ws, c->splitk_floats, &splits));
      return launch_reduce_residual_rmsnorm(c, s, c->splitk_ws, splits, M, d, c->h, gain, out, m.rms_eps);
    }
    RUN_GEMM(kEpiResidual, A, W, c->h, c->h, M, d, Kk);
    if (with_norm) return launch_rmsnorm(c, s, dt, c->h, gain, out, M, d, m.rms_eps);
    return PVF_OK;
  };
  bool xn_ready = false;
  NormArgs n_in, n_out;
  n_in.ss_in = c->row_ss; n_in.ld = M; n_in.inv_d = 1.0f / (float)d; n_in.eps = m.rms_eps; n_in.n_slots_in = 1;
  n_out.ss_out = c->row_ss; n_out.ld = M;
  RUN(launch_embed(c, s, dt, c->w.embed, tokens, seq_slot, S, T, d, m.vocab, c->h, fold_norm ? c->row_ss : nullptr));
  for (int l = 0; l < m.n_layers; ++l) {
    if (fold_norm) {
      {
        ProfScope ps(c, s, PVF_PROF_GEMM, 2.0 * M * (double)(3 * d) * d,
                     (double)c->esize * ((double)M * d + 3.0 * d * d + (double)M * 2 * d + (double)M * d));
        RUN(launch_gemm_mfma_qkv_rope(c, s, c->h, c->wqkv_f[l], c->qkv, c->vt, c->cos_sin, M, 3 * d, d, T, H,
                                      capture_spg > 0 && !c->cache_vt, &n_in));
      }
      {
        ProfScope ps(c, s, PVF_PROF_ATTENTION, 4.0 * S * (double)T * T * d, 0.0);
        RUN(launch_attention_mfma(c, s, c->qkv, c->vt, c->att, S, T, H));
      }
      if (capture_spg > 0) {
        const int64_t layer_off = (int64_t)l * T * d * c->esize, gstride = (int64_t)m.n_layers * T * d;
        void *vl = (char *)c->vcache + layer_off;
        RUN(launch_kv_store(c, s, dt, c->qkv, c->vt, seq_slot, capture_spg, S, T, d, (char *)c->kcache + layer_off,
                            c->cache_vt ? nullptr : vl, c->cache_vt ? vl : nullptr, gstride));
      }
      {
        ProfScope ps(c, s, PVF_PROF_GEMM, 2.0 * M * (double)d * d, (double)c->esize * ((double)M * d + (double)d * d + 2.0 * M * d));
        RUN(launch_gemm_mfma(c, s, kEpiResidual, c->att, c->wo[l], c->h, c->h, M, d, d, &n_out));
      }
      n_in.n_slots_in = slots_o;
      {
        ProfScope ps(c, s, PVF_PROF_GEMM, 4.0 * M * (double)ff * d, (double)c->esize * ((double)M * d + 2.0 * ff * d + (double)M * ff));
        RUN(launch_gemm_mfma(c, s, kEpiSwiglu, c->h, c->w_gate_up_f[l], c->act, nullptr, M, ff, d, &n_in));
      }
      {
        ProfScope ps(c, s, PVF_PROF_GEMM, 2.0 * M * (double)d * ff, (double)c->esize * ((double)M * ff + (double)d * ff + 2.0 * M * d));
        RUN(launch_gemm_mfma(c, s, kEpiResidual, c->act, c->w_down[l], c->h, c->h, M, d, ff, &n_out));
      }
      n_in.n_slots_in = slots_down;
      continue;
    }
    if (!xn_ready) RUN(launch_rmsnorm(c, s, dt, c->h, c->attn_norm[l], c->xn, M, d, m.rms_eps));
    xn_ready = false;
    if (fused_rope) {
      // the QKV projection rotates q, k and writes the key-contiguous v in its epilogue; the row-major v third
      // has a reader only when the K/V cache keeps its values in that layout
      const bool store_v = capture_spg > 0 && !c->cache_vt;
      {
        ProfScope ps(c, s, PVF_PROF_GEMM, 2.0 * M * (double)(3 * d) * d,
                     (double)c->esize * ((double)M * d + 3.0 * d * d + (double)M * (store_v ? 3 : 2) * d + (double)M * d));   // q, k (, v) + the key-contiguous v
        RUN(launch_gemm_mfma_qkv_rope(c, s, c->xn, c->wqkv[l], c->qkv, c->vt, c->cos_sin, M, 3 * d, d, T, H, store_v));
      }
      ProfScope ps(c, s, PVF_PROF_ATTENTION, 4.0 * S * (double)T * T * d, 0.0);
      RUN(launch_attention_mfma(c, s, c->qkv, c->vt, c->att, S, T, H));
    } else {
      RUN_GEMM(kEpiStore, c->xn, c->wqkv[l], c->qkv, nullptr, M, 3 * d, d);
      ProfScope ps(c, s, PVF_PROF_ATTENTION, 4.0 * S * (double)T * T * d, 0.0);
      RUN(launch_rope_attention(c, s, dt, c->qkv, c->vt, c->att, S, T, H, dh, c->cos_sin));
    }
    if (capture_spg > 0) {
      const int64_t layer_off = (int64_t)l * T * d * c->esize, gstride = (int64_t)m.n_layers * T * d;
      void *vl = (char *)c->vcache + layer_off;
      RUN(launch_kv_store(c, s, dt, c->qkv, c->vt, seq_slot, capture_spg, S, T, d, (char *)c->kcache + layer_off,
                          c->cache_vt ? nullptr : vl, c->cache_vt ? vl : nullptr, gstride));
    }
    RUN(project_residual_norm(c->att, c->wo[l], d, c->ffn_norm[l], c->xn, true));
    RUN_GEMM(kEpiSwiglu, c->xn, c->w_gate_up[l], c->act, nullptr, M, ff, d);
    // the norm that follows the down projection is the next layer's (the final one runs on the gathered rows only)
    const bool has_next = l + 1 < m.n_layers;
    RUN(project_residual_norm(c->act, c->w_down[l], ff, has_next ? c->attn_norm[l + 1] : nullptr, c->xn, has_next));
    xn_ready = has_next;
  }
  RUN(launch_gather_rows(c, s, dt, c->h, row_pos, S, T, R, d, c->hrows));
  RUN(launch_rmsnorm(c, s, dt, c->hrows, c->w.final_norm, c->hrows, S * R, d, m.rms_eps));
  RUN_GEMM(kEpiStore, c->hrows, c->w.out_head, logits, nullptr, S * R, m.vocab, d);
#undef RUN_GEMM
#undef RUN
  return PVF_OK;
}

// Cached round (kv_cache): only the R window rows of each of the S canvases go through the
// layers; keys / values outside the window come from the cache of the canvas' group.
static pvf_status forward_window_impl(pvf_ctx *c, hipStream_t s, const pvf_decode_cfg &cfg, const pvf_state &state,
                                      const int32_t *seq_slot, int S, const int32_t *row_pos, void *logits) {
  const pvf_model_cfg &m = c->model;
  const int d = m.d_model, H = m.n_heads, dh = d / H, ff = m.d_ff, dt = m.dtype;
  const int T = cfg.prompt_len + cfg.gen_len, R = window_rows(cfg);
  const int M = S * R;
  pvf_status st;
#define RUN(x) do { st = (x); if (st != PVF_OK) return st; } while (0)
#define RUN_GEMM(epi, A, W, C, res, Mm, Nn, Kk)                                                   \
  do {                                                                                            \
    ProfScope ps(c, s, PVF_PROF_GEMM, 2.0 * (Mm) * (double)(Nn) * (Kk) * ((epi) == kEpiSwiglu ? 2 : 1),   \
                 (double)c->esize * ((double)(Mm) * (Kk) + (double)(Nn) * (Kk) * ((epi) == kEpiSwiglu ? 2 : 1) + \
                                     (double)(Mm) * (Nn) * ((epi) == kEpiResidual ? 2 : 1)));             \
    RUN(launch_gemm(c, s, dt, epi, A, W, C, res, Mm, Nn, Kk));                                    \
  } while (0)
  RUN(launch_embed_rows(c, s, dt, c->w.embed, state.canvas, seq_slot, row_pos, M, R, T, d, m.vocab, c->h));
  const int64_t gstride = (int64_t)m.n_layers * T * d;
  // h += A W^T, then out = RMSNorm(h) * gain for the next projection.  Where the projection splits K (few rows)
  // one kernel adds the partial tiles and the residual and norms the row; otherwise the residual epilogue and the
  // norm run as two launches.
  const bool fuse_norm = !force_simple() && c->splitk_ws && reduce_residual_rmsnorm_supported(dt, d);
  auto project_residual_norm = [&](const void *A, const void *W, int Kk, const void *gain, void *out) -> pvf_status {
    if (fuse_norm && gemm_mfma_splitk_supported(dt, kEpiResidual, M, d, Kk, c->splitk_floats)) {
      int splits = 0;
      ProfScope ps(c, s, PVF_PROF_GEMM, 2.0 * M * (double)d * Kk, (double)c->esize * ((double)M * Kk + (double)d * Kk + 2.0 * M * d));
      RUN(launch_gemm_mfma_splitk_partial(c, s, A, W, M, d, Kk, c->splitk_ws, c->splitk_floats, &splits));
      return launch_reduce_residual_rmsnorm(c, s, c->splitk_ws, splits, M, d, c->h, gain, out, m.rms_eps);
    }
    RUN_GEMM(kEpiResidual, A, W, c->h, c->h, M, d, Kk);
    return launch_rmsnorm(c, s, dt, c->h, gain, out, M, d, m.rms_eps);
  };
  RUN(launch_rmsnorm(c, s, dt, c->h, c->attn_norm[0], c->xn, M, d, m.rms_eps));
  for (int l = 0; l < m.n_layers; ++l) {
    const int64_t layer_off = (int64_t)l * T * d * c->esize;
    RUN_GEMM(kEpiStore, c->xn, c->wqkv[l], c->qkv, nullptr, M, 3 * d, d);
    {
      ProfScope ps(c, s, PVF_PROF_ATTENTION, 4.0 * S * (double)R * T * d, 0.0);
      if (c->cache_vt) {
        RUN(launch_rope_vt_rows(c, s, c->qkv, c->vt, row_pos, S, R, T, H, c->cos_sin));
        RUN(launch_attention_window_mfma(c, s, c->qkv, c->vt, (const char *)c->kcache + layer_off,
                                         (const char *)c->vcache + layer_off, gstride, seq_slot, state.k_active,
                                         1 + cfg.K, cfg.prompt_len, cfg.block_len, R, S, T, H, c->att));
      } else {
        RUN(launch_rope_rows(c, s, dt, c->qkv, row_pos, M, T, H, dh, c->cos_sin));
        RUN(launch_attention_window(c, s, dt, c->qkv, (const char *)c->kcache + layer_off, (const char *)c->vcache + layer_off,
                                    gstride, cfg, state, seq_slot, S, H, dh, c->att));
      }
    }
    RUN(project_residual_norm(c->att, c->wo[l], d, c->ffn_norm[l], c->xn));
    RUN_GEMM(kEpiSwiglu, c->xn, c->w_gate_up[l], c->act, nullptr, M, ff, d);
    const bool last = l + 1 == m.n_layers;
    RUN(project_residual_norm(c->act, c->w_down[l], ff, last ? c->w.final_norm : c->attn_norm[l + 1], last ? c->hrows : c->xn));
  }
  RUN_GEMM(kEpiStore, c->hrows, c->w.out_head, logits, nullptr, M, m.vocab, d);
#undef RUN_GEMM
#undef RUN
  return PVF_OK;
}

extern "C" pvf_status pvf_forward(pvf_ctx *ctx, void *stream, const int32_t *tokens, int32_t S,
                                  int32_t T, const int32_t *row_pos, int32_t R, void *logits) {
  PVF_REQUIRE(nullptr, ctx != nullptr, PVF_EINVAL, "pvf_forward: ctx is NULL");
  PVF_REQUIRE(ctx, tokens && row_pos && logits, PVF_EINVAL, "pvf_forward: NULL pointer");
  PVF_REQUIRE(ctx, S >= 0 && T > 0 && R >= 0, PVF_EINVAL, "pvf_forward: S=%d T=%d R=%d", S, T, R);
  PVF_REQUIRE(ctx, S <= ctx->max_seqs && T <= ctx->max_T && R <= ctx->max_rows, PVF_ESHAPE,
              "pvf_forward: S=%d T=%d R=%d exceed the context (%d, %d, %d)", S, T, R, ctx->max_seqs, ctx->max_T, ctx->max_rows);
  if (S == 0 || R == 0) return PVF_OK;
  return forward_impl(ctx, (hipStream_t)stream, tokens, nullptr, S, T, row_pos, R, logits);
}

// =========================================================================================
// epilogue
// =========================================================================================
extern "C" pvf_status pvf_stage1(void *stream, const void *logits, int32_t logits_dtype,
                                 int64_t n_rows, int32_t vocab, int32_t mask_id, float logit_scale,
                                 float *conf, int32_t *tok) {
  PVF_REQUIRE(nullptr, n_rows == 0 || (logits && conf && tok), PVF_EINVAL, "pvf_stage1: NULL pointer");
  PVF_REQUIRE(nullptr, logits_dtype == PVF_F32 || logits_dtype == PVF_BF16, PVF_EINVAL, "pvf_stage1: dtype=%d", logits_dtype);
  PVF_REQUIRE(nullptr, n_rows >= 0 && vocab > 1, PVF_EINVAL, "pvf_stage1: n_rows=%lld vocab=%d", (long long)n_rows, vocab);
  PVF_REQUIRE(nullptr, mask_id >= 0 && mask_id < vocab, PVF_EINVAL, "pvf_stage1: mask_id=%d outside [0,%d)", mask_id, vocab);
  PVF_REQUIRE(nullptr, logit_scale > 0.f && std::isfinite(logit_scale), PVF_EINVAL, "pvf_stage1: logit_scale=%g", logit_scale);
  RowFilter rf{};
  return launch_stage1(nullptr, (hipStream_t)stream, logits, logits_dtype, n_rows, vocab, mask_id, logit_scale, rf, conf, tok);
}

extern "C" pvf_status pvf_entropy(void *stream, const void *logits, int32_t logits_dtype,
                                  int64_t n_rows, int32_t vocab, int32_t mask_id, float logit_scale,
                                  float *ent) {
  PVF_REQUIRE(nullptr, n_rows == 0 || (logits && ent), PVF_EINVAL, "pvf_entropy: NULL pointer");
  PVF_REQUIRE(nullptr, logits_dtype == PVF_F32 || logits_dtype == PVF_BF16, PVF_EINVAL, "pvf_entropy: dtype=%d", logits_dtype);
  PVF_REQUIRE(nullptr, n_rows >= 0 && vocab > 1, PVF_EINVAL, "pvf_entropy: n_rows=%lld vocab=%d", (long long)n_rows, vocab);
  PVF_REQUIRE(nullptr, mask_id >= 0 && mask_id < vocab, PVF_EINVAL, "pvf_entropy: mask_id=%d outside [0,%d)", mask_id, vocab);
  PVF_REQUIRE(nullptr, logit_scale > 0.f && std::isfinite(logit_scale), PVF_EINVAL, "pvf_entropy: logit_scale=%g", logit_scale);
  RowFilter rf{};
  return launch_entropy(nullptr, (hipStream_t)stream, logits, logits_dtype, n_rows, vocab, mask_id, logit_scale, rf, ent);
}

extern "C" pvf_status pvf_plan_vocab_select(void *stream, const uint32_t *cal_n, const uint32_t *cal_m,
                                            const uint32_t *cal_a, const double *cal_vig, int32_t vocab,
                                            int32_t mask_id, uint32_t n_min, uint32_t m_min, float rho_ver,
                                            float gamma_vig, uint32_t *plan_bitmap) {
  PVF_REQUIRE(nullptr, cal_n && cal_m && cal_a && cal_vig && plan_bitmap, PVF_EINVAL, "pvf_plan_vocab_select: NULL pointer");
  PVF_REQUIRE(nullptr, vocab > 1 && mask_id >= 0 && mask_id < vocab, PVF_EINVAL, "pvf_plan_vocab_select: vocab=%d mask_id=%d", vocab, mask_id);
  PVF_REQUIRE(nullptr, std::isfinite(rho_ver) && std::isfinite(gamma_vig), PVF_EINVAL, "pvf_plan_vocab_select: thresholds not finite");
  return launch_plan_vocab_select(nullptr, (hipStream_t)stream, cal_n, cal_m, cal_a, cal_vig, vocab, mask_id,
                                  n_min, m_min, rho_ver, gamma_vig, plan_bitmap);
}

static RowFilter make_filter(const pvf_decode_cfg &cfg, const pvf_state &st, const int32_t *seq_slot) {
  RowFilter rf;
  rf.n_drafts = st.n_drafts; rf.done = st.done; rf.k_active = st.k_active; rf.seq_slot = seq_slot;
  rf.slots_per_group = 1 + cfg.K; rf.R = window_rows(cfg);
  rf.prompt_len = cfg.prompt_len; rf.block_len = cfg.block_len; rf.T = cfg.prompt_len + cfg.gen_len;
  return rf;
}

extern "C" pvf_status pvf_epilogue(pvf_ctx *ctx, void *stream, const void *logits, int32_t logits_dtype,
                                   int32_t G, int32_t vocab, int32_t mask_id, const uint32_t *plan_bitmap,
                                   const pvf_decode_cfg *cfg, const pvf_state *state) {
  pvf_status st = check_decode_cfg(ctx, cfg, vocab, mask_id);
  if (st != PVF_OK) return st;
  if ((st = check_state(ctx, state, cfg)) != PVF_OK) return st;
  PVF_REQUIRE(ctx, logits && plan_bitmap, PVF_EINVAL, "pvf_epilogue: NULL pointer");
  PVF_REQUIRE(ctx, logits_dtype == PVF_F32 || logits_dtype == PVF_BF16, PVF_EINVAL, "pvf_epilogue: dtype=%d", logits_dtype);
  PVF_REQUIRE(ctx, G >= 0, PVF_EINVAL, "pvf_epilogue: G=%d", G);
  if (G == 0) return PVF_OK;
  hipStream_t s = (hipStream_t)stream;
  const RowFilter rf = make_filter(*cfg, *state, nullptr);
  const int64_t n_rows = (int64_t)G * (1 + cfg->K) * rf.R;
  {
    ProfScope ps(ctx, s, PVF_PROF_STAGE1, 0.0, (double)n_rows * vocab * (logits_dtype == PVF_BF16 ? 2.0 : 4.0));
    st = launch_stage1(ctx, s, logits, logits_dtype, n_rows, vocab, mask_id, cfg->logit_scale, rf, state->conf, state->tok);
  }
  if (st != PVF_OK) return st;
  if (cfg->routes & PVF_ROUTES_CAL) {
    st = launch_entropy(ctx, s, logits, logits_dtype, n_rows, vocab, mask_id, cfg->logit_scale, rf, state->ent);
    if (st != PVF_OK) return st;
  }
  ProfScope ps(ctx, s, PVF_PROF_STAGE2, 0.0, 0.0);
  return launch_stage2(ctx, s, G, vocab, mask_id, plan_bitmap, *cfg, *state);
}

// =========================================================================================
// round, state init, decode
// =========================================================================================
static pvf_status check_round(pvf_ctx *ctx, int G, const uint32_t *plan_bitmap, const pvf_decode_cfg *cfg,
                              const pvf_state *state) {
  PVF_REQUIRE(nullptr, ctx != nullptr, PVF_EINVAL, "ctx is NULL");
  pvf_status st = check_decode_cfg(ctx, cfg, ctx->model.vocab, ctx->model.mask_id);
  if (st != PVF_OK) return st;
  if ((st = check_state(ctx, state, cfg)) != PVF_OK) return st;
  PVF_REQUIRE(ctx, plan_bitmap != nullptr, PVF_EINVAL, "plan_bitmap is NULL");
  PVF_REQUIRE(ctx, G > 0, PVF_EINVAL, "G=%d", G);
  const int T = cfg->prompt_len + cfg->gen_len;
  PVF_REQUIRE(ctx, (int64_t)G * (1 + cfg->K) <= ctx->max_seqs && T <= ctx->max_T && window_rows(*cfg) <= ctx->max_rows,
              PVF_ESHAPE, "G*(1+K)=%d T=%d R=%d exceed the context (%d, %d, %d)", G * (1 + cfg->K), T,
              window_rows(*cfg), ctx->max_seqs, ctx->max_T, ctx->max_rows);
  return PVF_OK;
}

static pvf_status round_cached_impl(pvf_ctx *ctx, hipStream_t s, int G, const uint32_t *plan_bitmap,
                                    const pvf_decode_cfg &cfg, const pvf_state &state);

static pvf_status round_impl(pvf_ctx *ctx, hipStream_t s, int G, const uint32_t *plan_bitmap,
                             const pvf_decode_cfg &cfg, const pvf_state &state, int n_seq) {
  if (cfg.kv_cache) return round_cached_impl(ctx, s, G, plan_bitmap, cfg, state);
  const int T = cfg.prompt_len + cfg.gen_len, R = window_rows(cfg);
  const int all = G * (1 + cfg.K);
  if (n_seq <= 0 || n_seq > all) n_seq = all;
  pvf_status st = launch_build_batch(ctx, s, G, n_seq, cfg, state, ctx->seq_slot, ctx->row_pos);
  if (st != PVF_OK) return st;
  {
    ProfScope ps(ctx, s, PVF_PROF_FORWARD, 0.0, 0.0);
    st = forward_impl(ctx, s, state.canvas, ctx->seq_slot, n_seq, T, ctx->row_pos, R, ctx->logits);
  }
  if (st != PVF_OK) return st;
  const RowFilter rf = make_filter(cfg, state, ctx->seq_slot);
  {
    ProfScope ps(ctx, s, PVF_PROF_STAGE1, 0.0, (double)n_seq * R * ctx->model.vocab * (double)ctx->esize);
    st = launch_stage1(ctx, s, ctx->logits, ctx->model.dtype, (int64_t)n_seq * R, ctx->model.vocab,
                       ctx->model.mask_id, cfg.logit_scale, rf, state.conf, state.tok);
  }
  if (st != PVF_OK) return st;
  if (cfg.routes & PVF_ROUTES_CAL) {
    st = launch_entropy(ctx, s, ctx->logits, ctx->model.dtype, (int64_t)n_seq * R, ctx->model.vocab,
                        ctx->model.mask_id, cfg.logit_scale, rf, state.ent);
    if (st != PVF_OK) return st;
  }
  ProfScope ps(ctx, s, PVF_PROF_STAGE2, 0.0, 0.0);
  return launch_stage2(ctx, s, G, ctx->model.vocab, ctx->model.mask_id, plan_bitmap, cfg, state);
}

// kv_cache round: the backbone of a group whose active block differs from the block its cache was
// made for (or that has no cache yet) gets the full forward, which also refills the cache; every
// other canvas runs the window forward (after the full one, so it sees the fresh cache).  The sequence list is built on the host from a read-back of the state.
static pvf_status round_cached_impl(pvf_ctx *ctx, hipStream_t s, int G, const uint32_t *plan_bitmap,
                                    const pvf_decode_cfg &cfg, const pvf_state &state) {
  const pvf_model_cfg &m = ctx->model;
  const int T = cfg.prompt_len + cfg.gen_len, R = window_rows(cfg), spg = 1 + cfg.K;
  // cache memory
  const bool want_vt = use_attention_mfma(m.dtype, T, m.d_model / m.n_heads) &&
                       attention_window_mfma_supported(m.dtype, T, m.d_model / m.n_heads, R, cfg.block_len, cfg.prompt_len);
  if (want_vt != ctx->cache_vt) {                          // the value layout changes: every cache is stale
    ctx->cache_vt = want_vt;
    ctx->cache_block.assign(ctx->cache_block.size(), -1);
  }
  if (ctx->cache_G < G || ctx->cache_T != T) {
    if (ctx->kcache) (void)hipFree(ctx->kcache);
    if (ctx->vcache) (void)hipFree(ctx->vcache);
    ctx->kcache = ctx->vcache = nullptr; ctx->cache_G = 0;
    const size_t bytes = (size_t)G * m.n_layers * T * m.d_model * ctx->esize;
    PVF_REQUIRE(ctx, hipMalloc(&ctx->kcache, bytes) == hipSuccess && hipMalloc(&ctx->vcache, bytes) == hipSuccess,
                PVF_ENOMEM, "K/V cache: cannot allocate 2 x %zu bytes", bytes);
    ctx->cache_G = G; ctx->cache_T = T;
    ctx->cache_block.assign(G, -1);
  }
  if ((int)ctx->cache_block.size() < G) ctx->cache_block.resize(G, -1);
  if (ctx->cache_canvas != state.canvas) {                 // another state: its groups' caches are not these
    ctx->cache_canvas = state.canvas;
    ctx->cache_block.assign(ctx->cache_block.size(), -1);
  }
  // state read-back and the two sequence lists
  const int need = 3 * G + G * spg;
  if (ctx->seq_host_cap < need) {
    if (ctx->seq_host) (void)hipHostFree(ctx->seq_host);
    ctx->seq_host = nullptr; ctx->seq_host_cap = 0;
    PVF_HIP_CHECK(ctx, hipHostMalloc((void **)&ctx->seq_host, (size_t)need * sizeof(int32_t), hipHostMallocDefault));
    ctx->seq_host_cap = need;
  }
  int32_t *h_done = ctx->seq_host, *h_nd = h_done + G, *h_ka = h_nd + G, *h_seq = h_ka + G;
  PVF_HIP_CHECK(ctx, hipMemcpyAsync(h_done, state.done, G * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  PVF_HIP_CHECK(ctx, hipMemcpyAsync(h_nd, state.n_drafts, G * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  PVF_HIP_CHECK(ctx, hipMemcpyAsync(h_ka, state.k_active, G * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  PVF_HIP_CHECK(ctx, hipStreamSynchronize(s));
  int n_full = 0, n_win = 0;
  std::vector<int32_t> win, refreshed;
  for (int g = 0; g < G; ++g) {
    if (h_done[g]) continue;
    const int kt = h_nd[g] < 0 ? 0 : (h_nd[g] > cfg.K ? cfg.K : h_nd[g]);
    const bool refresh = ctx->cache_block[g] != h_ka[g];
    for (int j = 0; j <= kt; ++j) {                         // only the backbone of a refreshing group is forwarded in full
      if (refresh && j == 0) h_seq[n_full++] = g * spg + j;
      else win.push_back(g * spg + j);
    }
    if (refresh) { refreshed.push_back(g); ctx->cache_block[g] = -1; }   // valid only once its forward is enqueued
  }
  n_win = (int)win.size();
  for (int i = 0; i < n_win; ++i) h_seq[n_full + i] = win[i];
  const int n_seq = n_full + n_win;
  if (n_seq == 0) return launch_stage2(ctx, s, G, m.vocab, m.mask_id, plan_bitmap, cfg, state);   // all done: reports an empty round
  PVF_HIP_CHECK(ctx, hipMemcpyAsync(ctx->seq_slot, h_seq, n_seq * sizeof(int32_t), hipMemcpyHostToDevice, s));
  pvf_status st = launch_fill_row_pos(ctx, s, cfg, state, ctx->seq_slot, n_seq, ctx->row_pos);
  if (st != PVF_OK) return st;
  {
    ProfScope ps(ctx, s, PVF_PROF_FORWARD, 0.0, 0.0);
    if (n_full) {
      st = forward_impl(ctx, s, state.canvas, ctx->seq_slot, n_full, T, ctx->row_pos, R, ctx->logits, spg);
      if (st != PVF_OK) return st;
      for (int g : refreshed) ctx->cache_block[g] = h_ka[g];
    }
    if (n_win) {
      void *lg = (char *)ctx->logits + (size_t)n_full * R * m.vocab * ctx->esize;
      st = forward_window_impl(ctx, s, cfg, state, ctx->seq_slot + n_full, n_win, ctx->row_pos + (size_t)n_full * R, lg);
      if (st != PVF_OK) return st;
    }
  }
  const RowFilter rf = make_filter(cfg, state, ctx->seq_slot);
  {
    ProfScope ps(ctx, s, PVF_PROF_STAGE1, 0.0, (double)n_seq * R * m.vocab * (double)ctx->esize);
    st = launch_stage1(ctx, s, ctx->logits, m.dtype, (int64_t)n_seq * R, m.vocab, m.mask_id, cfg.logit_scale, rf,
                       state.conf, state.tok);
  }
  if (st != PVF_OK) return st;
  if (cfg.routes & PVF_ROUTES_CAL) {
    st = launch_entropy(ctx, s, ctx->logits, m.dtype, (int64_t)n_seq * R, m.vocab, m.mask_id, cfg.logit_scale, rf, state.ent);
    if (st != PVF_OK) return st;
  }
  ProfScope ps(ctx, s, PVF_PROF_STAGE2, 0.0, 0.0);
  return launch_stage2(ctx, s, G, m.vocab, m.mask_id, plan_bitmap, cfg, state);
}

// One round, then the 5 status words of every group (done, n_drafts, n_commit[3]) packed by one small
// kernel, copied to the context's pinned buffer with one copy, and the stream synchronised.
static pvf_status round_status_impl(pvf_ctx *ctx, hipStream_t s, int G, const uint32_t *plan_bitmap,
                                    const pvf_decode_cfg &cfg, const pvf_state &state, int n_seq) {
  if (ctx->status_cap < 5 * G) {
    if (ctx->status_host) (void)hipHostFree(ctx->status_host);
    if (ctx->status_dev) (void)hipFree(ctx->status_dev);
    ctx->status_host = ctx->status_dev = nullptr; ctx->status_cap = 0;
    PVF_HIP_CHECK(ctx, hipHostMalloc((void **)&ctx->status_host, (size_t)5 * G * sizeof(int32_t), hipHostMallocDefault));
    PVF_HIP_CHECK(ctx, hipMalloc((void **)&ctx->status_dev, (size_t)5 * G * sizeof(int32_t)));
    ctx->status_cap = 5 * G;
  }
  pvf_status st = round_impl(ctx, s, G, plan_bitmap, cfg, state, n_seq);
  if (st != PVF_OK) return st;
  if ((st = launch_pack_status(ctx, s, G, state, ctx->status_dev)) != PVF_OK) return st;
  PVF_HIP_CHECK(ctx, hipMemcpyAsync(ctx->status_host, ctx->status_dev, (size_t)5 * G * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  PVF_HIP_CHECK(ctx, hipStreamSynchronize(s));
  return PVF_OK;
}

extern "C" pvf_status pvf_round_sync(pvf_ctx *ctx, void *stream, int32_t G, const uint32_t *plan_bitmap,
                                     const pvf_decode_cfg *cfg, const pvf_state *state, int32_t n_seq_host,
                                     int32_t *status_host) {
  pvf_status st = check_round(ctx, G, plan_bitmap, cfg, state);
  if (st != PVF_OK) return st;
  PVF_REQUIRE(ctx, status_host != nullptr, PVF_EINVAL, "pvf_round_sync: status_host is NULL");
  if ((st = round_status_impl(ctx, (hipStream_t)stream, G, plan_bitmap, *cfg, *state, n_seq_host)) != PVF_OK) return st;
  memcpy(status_host, ctx->status_host, (size_t)5 * G * sizeof(int32_t));
  return PVF_OK;
}

extern "C" pvf_status pvf_round(pvf_ctx *ctx, void *stream, int32_t G, const uint32_t *plan_bitmap,
                                const pvf_decode_cfg *cfg, const pvf_state *state, int32_t n_seq_host) {
  pvf_status st = check_round(ctx, G, plan_bitmap, cfg, state);
  if (st != PVF_OK) return st;
  return round_impl(ctx, (hipStream_t)stream, G, plan_bitmap, *cfg, *state, n_seq_host);
}

extern "C" pvf_status pvf_state_init(pvf_ctx *ctx, void *stream, const int32_t *prompt, int32_t G,
                                     const pvf_decode_cfg *cfg, const pvf_state *state) {
  PVF_REQUIRE(nullptr, ctx != nullptr, PVF_EINVAL, "ctx is NULL");
  pvf_status st = check_decode_cfg(ctx, cfg, ctx->model.vocab, ctx->model.mask_id);
  if (st != PVF_OK) return st;
  if ((st = check_state(ctx, state, cfg)) != PVF_OK) return st;
  PVF_REQUIRE(ctx, G > 0 && (prompt || cfg->prompt_len == 0), PVF_EINVAL, "pvf_state_init: G=%d prompt=%p", G, (const void *)prompt);
  ctx->cache_block.assign(ctx->cache_block.size(), -1);          // a fresh canvas has no valid K/V cache
  return launch_state_init(ctx, (hipStream_t)stream, prompt, G, ctx->model.mask_id, *cfg, *state);
}

extern "C" pvf_status pvf_decode(pvf_ctx *ctx, void *stream, const int32_t *prompt, int32_t G,
                                 const uint32_t *plan_bitmap, const pvf_decode_cfg *cfg,
                                 const pvf_state *state, int32_t *out_tokens, pvf_stats *stats) {
  pvf_status st = check_round(ctx, G, plan_bitmap, cfg, state);
  if (st != PVF_OK) return st;
  PVF_REQUIRE(ctx, out_tokens && (prompt || cfg->prompt_len == 0), PVF_EINVAL, "pvf_decode: NULL pointer");
  hipStream_t s = (hipStream_t)stream;
  pvf_stats acc;
  memset(&acc, 0, sizeof(acc));
  const auto t0 = std::chrono::steady_clock::now();
  ctx->cache_block.assign(ctx->cache_block.size(), -1);
  if ((st = launch_state_init(ctx, s, prompt, G, ctx->model.mask_id, *cfg, *state)) != PVF_OK) return st;
  int n_seq = G;                                  // first round: backbones only
  const int max_rounds = cfg->gen_len + 2;        // every round commits at least one token per live group
  while (n_seq > 0) {
    PVF_REQUIRE(ctx, acc.rounds < max_rounds, PVF_EINVAL, "pvf_decode: no progress after %d rounds", acc.rounds);
    if ((st = round_status_impl(ctx, s, G, plan_bitmap, *cfg, *state, n_seq)) != PVF_OK) return st;
    acc.rounds += 1;
    acc.seq_forwards += n_seq;
    n_seq = 0;
    for (int g = 0; g < G; ++g) {
      const int32_t *w = ctx->status_host + 5 * g;            // done, n_drafts, n_commit[3]
      acc.n_base += w[2]; acc.n_plan += w[3]; acc.n_ar += w[4];
      acc.drafts_accepted += (w[3] > 0) + w[4];
      if (!w[0]) { n_seq += 1 + w[1]; acc.drafts_proposed += w[1]; }
    }
  }
  if ((st = launch_copy_out(ctx, s, G, cfg->K, cfg->prompt_len + cfg->gen_len, state->canvas, out_tokens)) != PVF_OK) return st;
  PVF_HIP_CHECK(ctx, hipStreamSynchronize(s));
  acc.ms_total = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
  if (stats) *stats = acc;
  return PVF_OK;
}

// =========================================================================================
// per-kernel timing
// =========================================================================================
extern "C" pvf_status pvf_profile_begin(pvf_ctx *ctx) {
  PVF_REQUIRE(nullptr, ctx != nullptr, PVF_EINVAL, "pvf_profile_begin: ctx is NULL");
  ctx->prof.clear();
  ctx->ev_used = 0;
  ctx->prof_on = true;
  return PVF_OK;
}

extern "C" pvf_status pvf_profile_end(pvf_ctx *ctx, void *stream, pvf_profile *out) {
  PVF_REQUIRE(nullptr, ctx != nullptr, PVF_EINVAL, "pvf_profile_end: ctx is NULL");
  PVF_REQUIRE(ctx, out != nullptr, PVF_EINVAL, "pvf_profile_end: out is NULL");
  ctx->prof_on = false;
  PVF_HIP_CHECK(ctx, hipStreamSynchronize((hipStream_t)stream));
  memset(out, 0, sizeof(*out));
  for (const auto &r : ctx->prof) {
    float ms = 0.f;
    PVF_HIP_CHECK(ctx, hipEventElapsedTime(&ms, r.e0, r.e1));
    out->ms[r.cat] += ms; out->flops[r.cat] += r.flops; out->bytes[r.cat] += r.bytes; out->launches[r.cat] += 1;
  }
  ctx->prof.clear();
  ctx->ev_used = 0;
  return PVF_OK;
}

// =========================================================================================
// building blocks
// =========================================================================================
static pvf_status check_dtype(int dtype) {
  PVF_REQUIRE(nullptr, dtype == PVF_F32 || dtype == PVF_BF16, PVF_EINVAL, "dtype=%d", dtype);
  return PVF_OK;
}

extern "C" pvf_status pvf_gemm(void *stream, int32_t dtype, const void *A, const void *W, void *C,
                               const void *residual, int32_t M, int32_t N, int32_t K) {
  if (check_dtype(dtype) != PVF_OK) return PVF_EINVAL;
  PVF_REQUIRE(nullptr, A && W && C && M >= 0 && N >= 0 && K > 0, PVF_EINVAL, "pvf_gemm: bad argument");
  return launch_gemm(nullptr, (hipStream_t)stream, dtype, residual ? kEpiResidual : kEpiStore, A, W, C, residual, M, N, K);
}

extern "C" pvf_status pvf_ctx_gemm(pvf_ctx *ctx, void *stream, const void *A, const void *W, void *C,
                                   const void *residual, int32_t M, int32_t N, int32_t K) {
  PVF_REQUIRE(nullptr, ctx != nullptr, PVF_EINVAL, "pvf_ctx_gemm: ctx is NULL");
  PVF_REQUIRE(ctx, A && W && C && M >= 0 && N >= 0 && K > 0, PVF_EINVAL, "pvf_ctx_gemm: bad argument");
  return launch_gemm(ctx, (hipStream_t)stream, ctx->model.dtype, residual ? kEpiResidual : kEpiStore, A, W, C, residual, M, N, K);
}

extern "C" pvf_status pvf_ctx_gemm_swiglu(pvf_ctx *ctx, void *stream, const void *A, const void *W, void *act,
                                          int32_t M, int32_t ff, int32_t K) {
  PVF_REQUIRE(nullptr, ctx != nullptr, PVF_EINVAL, "pvf_ctx_gemm_swiglu: ctx is NULL");
  PVF_REQUIRE(ctx, A && W && act && M >= 0 && ff >= 0 && K > 0, PVF_EINVAL, "pvf_ctx_gemm_swiglu: bad argument");
  return launch_gemm(ctx, (hipStream_t)stream, ctx->model.dtype, kEpiSwiglu, A, W, act, nullptr, M, ff, K);
}

extern "C" pvf_status pvf_gemm_swiglu(void *stream, int32_t dtype, const void *A, const void *W,
                                      void *act, int32_t M, int32_t ff, int32_t K) {
  if (check_dtype(dtype) != PVF_OK) return PVF_EINVAL;
  PVF_REQUIRE(nullptr, A && W && act && M >= 0 && ff >= 0 && K > 0, PVF_EINVAL, "pvf_gemm_swiglu: bad argument");
  return launch_gemm(nullptr, (hipStream_t)stream, dtype, kEpiSwiglu, A, W, act, nullptr, M, ff, K);
}

extern "C" pvf_status pvf_rmsnorm(void *stream, int32_t dtype, const void *x, const void *gain,
                                  void *out, int32_t M, int32_t d, float eps) {
  if (check_dtype(dtype) != PVF_OK) return PVF_EINVAL;
  PVF_REQUIRE(nullptr, x && gain && out && M >= 0 && d > 0, PVF_EINVAL, "pvf_rmsnorm: bad argument");
  return launch_rmsnorm(nullptr, (hipStream_t)stream, dtype, x, gain, out, M, d, eps);
}

// Builds the rotary table on the host for this call, so it synchronises the stream and
// allocates; it exists for tests, the round itself uses the context's table.
extern "C" pvf_status pvf_rope_attention(void *stream, int32_t dtype, void *qkv, void *out, int32_t S,
                                         int32_t T, int32_t n_heads, int32_t d_head, float rope_theta) {
  if (check_dtype(dtype) != PVF_OK) return PVF_EINVAL;
  PVF_REQUIRE(nullptr, qkv && out && S >= 0 && T > 0 && n_heads > 0 && d_head > 0 && d_head % 2 == 0 && rope_theta > 0.f,
              PVF_EINVAL, "pvf_rope_attention: bad argument");
  if (S == 0) return PVF_OK;
  hipStream_t s = (hipStream_t)stream;
  const int half = d_head / 2;
  std::vector<float2> tab((size_t)T * half);
  for (int i = 0; i < half; ++i) {
    const double inv = std::pow((double)rope_theta, -2.0 * i / d_head);
    for (int t = 0; t < T; ++t)
      tab[(size_t)t * half + i] = make_float2((float)std::cos(t * inv), (float)std::sin(t * inv));
  }
  float2 *dev = nullptr;
  void *vt = nullptr;
  PVF_HIP_CHECK(nullptr, hipMalloc((void **)&dev, tab.size() * sizeof(float2)));
  hipError_t e = hipMemcpy(dev, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice);
  pvf_status st = PVF_OK;
  if (e != hipSuccess) { set_error(nullptr, "rotary table upload: %s", hipGetErrorString(e)); st = PVF_EHIP; }
  if (st == PVF_OK && use_attention_mfma(dtype, T, d_head)) {
    e = hipMalloc(&vt, (size_t)S * T * n_heads * d_head * 2);
    if (e != hipSuccess) { set_error(nullptr, "scratch allocation: %s", hipGetErrorString(e)); st = PVF_EHIP; }
  }
  if (st == PVF_OK) st = launch_rope_attention(nullptr, s, dtype, qkv, vt, out, S, T, n_heads, d_head, dev);
  (void)hipStreamSynchronize(s);
  (void)hipFree(dev);
  if (vt) (void)hipFree(vt);
  return st;
}

// ---- the variant of pvf_rope_attention that allocates nothing ---------------------------------
// Its rotary table and the key-contiguous copy of v live in one file-scope device array.  Each GPU
// holds its own copy of the array at its own address, looked up once per device (with that device
// current) and kept; host code only ever uses the looked-up pointer, never the array's name.
namespace {
constexpr int kNoAllocMaxT = 2048, kNoAllocMaxHalf = 64;
constexpr size_t kNoAllocTabBytes = (size_t)kNoAllocMaxT * kNoAllocMaxHalf * sizeof(float2);   // 1 MiB
constexpr size_t kNoAllocVtBytes = (size_t)16 << 20;                                            // 16 MiB
static __device__ __align__(256) unsigned char scratch[kNoAllocTabBytes + kNoAllocVtBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
unsigned char *g_scratch_ptr[kMaxDevices] = {nullptr};

struct InvFreq { double v[kNoAllocMaxHalf]; };

// tab[t][i] = (cos, sin)(t * inv_freq[i]) evaluated in double precision, like the host-built table
__global__ void __launch_bounds__(256) rope_table_kernel(float2 *tab, int T, int half, InvFreq f) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= T * half) return;
  const double a = (double)(idx / half) * f.v[idx % half];
  tab[idx] = make_float2((float)cos(a), (float)sin(a));
}

pvf_status scratch_of_current_device(unsigned char **out) {
  int dev = -1;
  PVF_HIP_CHECK(nullptr, hipGetDevice(&dev));
  PVF_REQUIRE(nullptr, dev >= 0 && dev < kMaxDevices, PVF_ESHAPE, "device index %d outside [0,%d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    PVF_HIP_CHECK(nullptr, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    PVF_REQUIRE(nullptr, p != nullptr, PVF_EHIP, "hipGetSymbolAddress returned a NULL address");
    g_scratch_ptr[dev] = (unsigned char *)p;
  }
  *out = g_scratch_ptr[dev];
  return PVF_OK;
}
}  // namespace

extern "C" pvf_status pvf_rope_attention_noalloc(void *stream, int32_t dtype, void *qkv, void *out, int32_t S,
                                                 int32_t T, int32_t n_heads, int32_t d_head, float rope_theta) {
  if (check_dtype(dtype) != PVF_OK) return PVF_EINVAL;
  PVF_REQUIRE(nullptr, qkv && out && S >= 0 && T > 0 && n_heads > 0 && d_head > 0 && d_head % 2 == 0 && rope_theta > 0.f,
              PVF_EINVAL, "pvf_rope_attention_noalloc: bad argument");
  const int half = d_head / 2;
  PVF_REQUIRE(nullptr, T <= kNoAllocMaxT && half <= kNoAllocMaxHalf, PVF_ESHAPE,
              "pvf_rope_attention_noalloc: T=%d d_head=%d exceed the static scratch (T <= %d, d_head <= %d)", T, d_head,
              kNoAllocMaxT, 2 * kNoAllocMaxHalf);
  const bool mfma = use_attention_mfma(dtype, T, d_head);
  const size_t vt_bytes = mfma ? (size_t)S * T * n_heads * d_head * 2 : 0;
  PVF_REQUIRE(nullptr, vt_bytes <= kNoAllocVtBytes, PVF_ESHAPE,
              "pvf_rope_attention_noalloc: S*T*n_heads*d_head = %lld elements exceed the static scratch (%lld)",
              (long long)S * T * n_heads * d_head, (long long)(kNoAllocVtBytes / 2));
  if (S == 0) return PVF_OK;
  unsigned char *base = nullptr;
  pvf_status st = scratch_of_current_device(&base);
  if (st != PVF_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  float2 *tab = reinterpret_cast<float2 *>(base);
  void *vt = base + kNoAllocTabBytes;
  InvFreq f;
  for (int i = 0; i < half; ++i) f.v[i] = std::pow((double)rope_theta, -2.0 * i / d_head);
  for (int i = half; i < kNoAllocMaxHalf; ++i) f.v[i] = 0.0;
  rope_table_kernel<<<(T * half + 255) / 256, 256, 0, s>>>(tab, T, half, f);
  PVF_LAUNCH_CHECK(nullptr, "rope_table");
  // every element of tab[0, T*half) and of the vt region the attention reads is rewritten by this call
  return launch_rope_attention(nullptr, s, dtype, qkv, vt, out, S, T, n_heads, d_head, tab);
}

extern "C" pvf_status pvf_qkv_attention(void *stream, int32_t dtype, const void *x, const void *wqkv, void *qkv,
                                        void *vt_caller, void *out, int32_t S, int32_t T, int32_t n_heads,
                                        int32_t d_head, float rope_theta) {
  if (check_dtype(dtype) != PVF_OK) return PVF_EINVAL;
  PVF_REQUIRE(nullptr, x && wqkv && qkv && out && S >= 0 && T > 0 && n_heads > 0 && d_head > 0 && d_head % 2 == 0 &&
                  rope_theta > 0.f, PVF_EINVAL, "pvf_qkv_attention: bad argument");
  if (S == 0) return PVF_OK;
  hipStream_t s = (hipStream_t)stream;
  const int half = d_head / 2, d = n_heads * d_head, M = S * T;
  std::vector<float2> tab((size_t)T * half);
  for (int i = 0; i < half; ++i) {
    const double inv = std::pow((double)rope_theta, -2.0 * i / d_head);
    for (int t = 0; t < T; ++t)
      tab[(size_t)t * half + i] = make_float2((float)std::cos(t * inv), (float)std::sin(t * inv));
  }
  float2 *dev = nullptr;
  void *vt = nullptr;
  PVF_HIP_CHECK(nullptr, hipMalloc((void **)&dev, tab.size() * sizeof(float2)));
  hipError_t e = hipMemcpy(dev, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice);
  pvf_status st = PVF_OK;
  if (e != hipSuccess) { set_error(nullptr, "rotary table upload: %s", hipGetErrorString(e)); st = PVF_EHIP; }
  const bool mfma_att = use_attention_mfma(dtype, T, d_head);
  if (st == PVF_OK && mfma_att) {
    if (vt_caller) vt = vt_caller;
    else {
      e = hipMalloc(&vt, (size_t)M * d * 2);
      if (e != hipSuccess) { set_error(nullptr, "scratch allocation: %s", hipGetErrorString(e)); st = PVF_EHIP; }
    }
  }
  if (st == PVF_OK) {
    if (mfma_att && gemm_mfma_qkv_rope_supported(dtype, M, 3 * d, d, T, n_heads)) {
      st = launch_gemm_mfma_qkv_rope(nullptr, s, x, wqkv, qkv, vt, dev, M, 3 * d, d, T, n_heads, true);
      if (st == PVF_OK) st = launch_attention_mfma(nullptr, s, qkv, vt, out, S, T, n_heads);
    } else {
      st = launch_gemm(nullptr, s, dtype, kEpiStore, x, wqkv, qkv, nullptr, M, 3 * d, d);
      if (st == PVF_OK) st = launch_rope_attention(nullptr, s, dtype, qkv, vt, out, S, T, n_heads, d_head, dev);
    }
  }
  (void)hipStreamSynchronize(s);
  (void)hipFree(dev);
  if (vt && vt != vt_caller) (void)hipFree(vt);
  return st;
}

extern "C" pvf_status pvf_fill_normal(void *stream, int32_t dtype, void *dst, int64_t n, uint64_t seed,
                                      float mean, float std) {
  if (check_dtype(dtype) != PVF_OK) return PVF_EINVAL;
  PVF_REQUIRE(nullptr, dst && n >= 0, PVF_EINVAL, "pvf_fill_normal: bad argument");
  return launch_fill_normal(nullptr, (hipStream_t)stream, dtype, dst, n, seed, mean, std);
}
