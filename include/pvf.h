/*
 * pvf.h -- C ABI of libpvf: one Plan-Verify-Fill (PVF) denoising round for a masked
 * diffusion language model on one AMD MI355X (gfx950), and the decode loop around it.
 *
 * A round (Algorithm 1 of the paper, one forward per round) is
 *   forward   : one batched, non-causal transformer pass over the backbone canvas (the
 *               base branch z_base, Sec. 3) and up to K draft canvases (Eq. plan_branch,
 *               Sec. 4.3), logits produced only for the rows of the active block and the
 *               block after it;
 *   epilogue  : per logits row the top-1 token and its softmax probability (Sec. 3), then
 *               verify the drafts (Eq. impact_set, Eq. at, Filter 1/2 of Sec. 4.2, the AR
 *               acceptance set of Sec. 4.3), commit the winner, and from the winner's own
 *               predictions apply the confidence threshold (Sec. 2) and propose the next
 *               drafts (Sec. 4.1 planning candidates, else Sec. 4.3 AR candidates).
 *
 * Conventions
 *   - "dev" pointers are device memory owned by the CALLER; "host" pointers are host
 *     memory.  The library owns only the workspace inside pvf_ctx.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     enqueue work on it and return without synchronising unless stated otherwise.
 *   - Every call returns a pvf_status; nothing throws or aborts across this boundary.
 *     Arguments are validated before any launch.  pvf_last_error() gives a message for
 *     the last failing call on that context (or on the calling thread if ctx is NULL).
 *   - Matrices are row-major.  Weight matrices are [out_features, in_features], i.e.
 *     y = x * W^T.  dtype 0 = float32, 1 = bfloat16 (storage of weights, activations and
 *     logits; accumulation is always float32).
 *   - Canvas positions: [0, prompt_len) prompt, then gen_len generated tokens split into
 *     gen_len / block_len blocks (App. A.1).  T = prompt_len + gen_len.
 *   - Window: the R = min(c*block_len, gen_len) canvas positions starting at the first
 *     position of the active block, c = 2 (c = 4 when n_sparse > 0); row r of a canvas is
 *     position prompt_len + k_active*block_len + r.  Rows whose position is >= T do not
 *     exist: their summaries are conf = 0, tok = -1.
 *   - Working set B_t: the active block; with n_sparse = N_s > 0 also the whole next block
 *     once the active block holds at most N_s masks (App. A.4.1, Eq. block_expansion).
 *     Impact set, compatibility, C_total, commits and candidates all range over B_t.
 *   - Environment variables, each read once per process; none is needed in normal use:
 *     PVF_GEMM_TILE=<n>   force bf16 GEMM tile shape n wherever a launch can take it
 *                         (tile sweeps; every shape gives bit-identical results),
 *     PVF_FORCE_SIMPLE=1  run bf16 launches on the plain (non-MFMA) kernels,
 *     PVF_FOLD_NORM=0     keep every RMSNorm a launch of its own instead of folding it
 *                         into the projections around it (forwards above 640 rows).
 */
#ifndef PVF_H
#define PVF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  PVF_OK = 0,
  PVF_EINVAL = -1,   /* bad argument value                                   */
  PVF_ESHAPE = -2,   /* shape exceeds what the context was created for       */
  PVF_ENOMEM = -3,   /* workspace allocation failed                          */
  PVF_EHIP = -4,     /* a HIP runtime call failed (message has the HIP text) */
  PVF_ENOTIMPL = -5  /* combination not supported by this build              */
} pvf_status;

enum { PVF_F32 = 0, PVF_BF16 = 1 };
enum { PVF_ROUTE_NONE = 0, PVF_ROUTE_PLAN = 1, PVF_ROUTE_AR = 2, PVF_ROUTE_CAL = 3 };
enum { PVF_ROUTES_PLAN = 1, PVF_ROUTES_AR = 2, PVF_ROUTES_CAL = 4, PVF_ROUTES_XRANDOM = 8, PVF_ROUTES_XPLANNING = 16 };

typedef struct pvf_ctx pvf_ctx;

/* Denoiser P_theta (Sec. 2).  The paper does not fix the architecture; this library runs a
 * pre-norm bidirectional transformer: RMSNorm, rotary embedding (dimension i paired with
 * i + d_head/2, angle pos * rope_theta^(-2i/d_head)), full multi-head attention with no
 * mask, SwiGLU FFN, untied output head. */
typedef struct {
  int32_t n_layers, d_model, n_heads, d_ff, vocab;
  int32_t dtype;        /* PVF_F32 or PVF_BF16 */
  float rms_eps, rope_theta;
  int32_t mask_id;      /* id of the absorbing [MASK] token, in [0, vocab) */
} pvf_model_cfg;

/* Hyper-parameters of Algorithm 1 (hyper-parameter table of the appendix). */
typedef struct {
  float tau_high;       /* commit threshold (Sec. 2)                                  */
  float tau_plan_lo;    /* planning band [lo, hi) (Sec. 4.1); lo <= hi <= tau_high     */
  float tau_plan_hi;
  float tau_ar_lo;      /* AR fallback threshold (Sec. 4.3)                            */
  float logit_scale;    /* > 0; probabilities are softmax(logit_scale * logits)        */
  int32_t K;            /* draft budget per canvas group, 0..PVF_MAX_K                 */
  int32_t block_len;    /* tokens per block; gen_len % block_len == 0                  */
  int32_t prompt_len;
  int32_t gen_len;
  int32_t routes;       /* bit 0 planning route, bit 1 AR route; 0 = threshold decoding; */
                        /* PVF_ROUTES_CAL alone = calibration trajectory (App. A.2):    */
                        /* threshold decoding whose drafts are the non-base masks with  */
                        /* confidence in [tau_plan_lo, tau_plan_hi) (the calibration    */
                        /* band, any token, the K most confident); they are measured    */
                        /* (A_j, Delta H_j) into the token statistics, never committed. */
                        /* PVF_ROUTES_XRANDOM / PVF_ROUTES_XPLANNING alone = the two    */
                        /* ablation decoders of App. A.3.1: threshold decoding plus ONE */
                        /* extra commit per round among the remaining masks whose       */
                        /* confidence lies in the closed bin [tau_plan_lo, tau_plan_hi],*/
                        /* uniformly at random (XPLANNING: among those whose token is a */
                        /* planning token, if any).  The pick is the (u mod count)-th   */
                        /* eligible position in canvas order, u = SplitMix64 step of    */
                        /* seed * 2^32 + (group & 0xFFF) * 2^20 + masked positions left */
                        /* on the canvas; n_commit[.][1] counts these commits           */
  int32_t n_sparse;     /* early cross-block revelation threshold N_s (App. A.4.1);     */
                        /* 0 = off: the working set is always the active block alone   */
  uint32_t seed;        /* seed of the ablation decoders' generator                    */
  int32_t kv_cache;     /* 1 = block-level K/V cache (Sec. 5.1, "under KV cache"), used */
                        /* by pvf_round / pvf_decode: a group's backbone canvas gets    */
                        /* the exact full forward in the first round and whenever its   */
                        /* active block has changed, and that forward's per-layer       */
                        /* rotated keys and values are kept; every other canvas (all    */
                        /* drafts; the backbone in the other rounds) runs only its      */
                        /* window rows through the layers, attending to the cached      */
                        /* keys / values outside the window.                            */
                        /* 0 = every round is a full forward (exact)                    */
} pvf_decode_cfg;

#define PVF_MAX_K 32
#define PVF_MAX_SUMMARIES 8192   /* (1+K) * R must not exceed this */

/* Weights, all dev, in cfg.dtype.  Per-layer entries are HOST arrays of n_layers dev pointers.
 *   embed [vocab, d]   out_head [vocab, d]   final_norm [d]
 *   attn_norm [d]  wqkv [3d, d] (rows: q | k | v)  wo [d, d]
 *   ffn_norm [d]   w_gate_up [2*d_ff, d] (rows: gate | up)  w_down [d, d_ff]
 * The library keeps the pointers (not copies); they must stay valid until pvf_destroy. */
typedef struct {
  const void *embed, *out_head, *final_norm;
  const void *const *attn_norm, *const *wqkv, *const *wo;
  const void *const *ffn_norm, *const *w_gate_up, *const *w_down;
} pvf_weights;

/* Decoding state of G canvas groups, all dev, read-modify-write by the epilogue.
 * One group = one backbone canvas plus its draft slots; slot 0 is the backbone. */
typedef struct {
  int32_t *canvas;      /* [G, 1+K, T]  in: this round's batch X_0..X_K; out: next batch  */
  int32_t *n_drafts;    /* [G]          in: K_t of this batch;  out: K_{t+1}              */
  int32_t *draft_route; /* [G]          PVF_ROUTE_* of the drafts (in/out)                */
  int32_t *fill_pos;    /* [G, K]       canvas position of candidate j (in/out)           */
  int32_t *fill_tok;    /* [G, K]       token of candidate j (in/out).  Planning draft j  */
                        /*              = backbone + fill j; AR draft k = backbone +      */
                        /*              fills 1..k                                        */
  int32_t *k_active;    /* [G]          index of the active block (in/out)                */
  int32_t *n_ws_blocks; /* [G]          blocks in the working set the batch was formed on: */
                        /*              1, or 2 after early cross-block revelation (in/out) */
  float   *conf;        /* [G, 1+K, R]  out: top-1 probability per window row             */
  int32_t *tok;         /* [G, 1+K, R]  out: top-1 token per window row                   */
  uint8_t *accept;      /* [G, K]       out: A_j (planning) / pass bit (AR) of THIS batch */
  int32_t *winner;      /* [G]          out: 0 = base branch, else the committed slot     */
  int32_t *n_commit;    /* [G, 3]       out: tokens committed this round by the           */
                        /*              threshold / planning route / AR route             */
  int32_t *done;        /* [G]          in/out: 1 once the canvas holds no mask; a done    */
                        /*              group is skipped                                  */
  /* Calibration only (routes == PVF_ROUTES_CAL); may be NULL otherwise.  Sec. 3 "Verified
   * information gain", App. A.2 "Token-level aggregation". */
  float   *ent;         /* [G, 1+K, R]  out: entropy H_i (nats) per window row             */
  double  *dh;          /* [G, K]       out: Delta H_j of THIS batch's drafts              */
  uint32_t *cal_n;      /* [vocab]      in/out accumulators over all measured events whose  */
  uint32_t *cal_m;      /*              candidate token is v: n_v (events), m_v (events     */
  uint32_t *cal_a;      /*              with a non-empty impact set), sum of A_j, and       */
  double  *cal_vig;     /* [vocab]      sum of VIG_j = A_j * Delta H_j.  The caller zeroes  */
                        /*              them before the first round.  The three counters    */
                        /*              are exact; cal_vig is added with float64 atomics,   */
                        /*              so when several events of one round carry the same  */
                        /*              token the order of the adds, and with it the last   */
                        /*              bits of that sum, is not fixed.                     */
} pvf_state;

typedef struct {
  int32_t rounds;       /* forward passes issued (NFE of the batch)                        */
  int32_t seq_forwards; /* canvases forwarded, summed over rounds                          */
  int64_t n_base, n_plan, n_ar;   /* tokens committed by each route, summed over groups   */
  int64_t drafts_proposed, drafts_accepted;
  double  ms_total;     /* wall time of the loop (host clock, includes the per-round sync) */
} pvf_stats;

/* ---- context ------------------------------------------------------------------------- */

/* Allocates the activation workspace for at most max_seqs canvases of at most max_T tokens
 * with at most max_rows logits rows each.  Returns PVF_ENOMEM / PVF_EHIP on failure. */
pvf_status pvf_create(pvf_ctx **out, const pvf_model_cfg *model, const pvf_weights *weights,
                      int32_t max_seqs, int32_t max_T, int32_t max_rows);
void pvf_destroy(pvf_ctx *ctx);
/* Static or context-owned string, never freed by the caller. */
const char *pvf_last_error(const pvf_ctx *ctx);
/* Bytes of device workspace the context holds. */
int64_t pvf_workspace_bytes(const pvf_ctx *ctx);

/* ---- per-kernel timing ------------------------------------------------------------------
 * Between pvf_profile_begin and pvf_profile_end every GEMM, attention (rotary + attention) and
 * epilogue stage-1 launch the context makes, and per round the whole forward and stage 2, are
 * bracketed by a pair of HIP events on the launch stream (about 6 us of host time per pair: time
 * throughput in a pass without it).  pvf_profile_end synchronises the stream and returns, per category, the summed
 * event-to-event time, the algorithmic work (flops / bytes) and the number of launches. */
enum { PVF_PROF_GEMM = 0, PVF_PROF_ATTENTION = 1, PVF_PROF_STAGE1 = 2,
       PVF_PROF_FORWARD = 3,   /* the whole batched forward of a round (encloses the GEMM and attention launches) */
       PVF_PROF_STAGE2 = 4,    /* verify / commit / propose + next canvases */
       PVF_PROF_NCAT = 5 };
typedef struct {
  double ms[PVF_PROF_NCAT], flops[PVF_PROF_NCAT], bytes[PVF_PROF_NCAT];
  int64_t launches[PVF_PROF_NCAT];
} pvf_profile;
pvf_status pvf_profile_begin(pvf_ctx *ctx);
pvf_status pvf_profile_end(pvf_ctx *ctx, void *stream, pvf_profile *out);

/* ---- the four calls of the path -------------------------------------------------------- */

/* P_theta(. | canvas) for S canvases in one batch (Sec. 4.1, "one batched forward pass").
 *   tokens  dev int32 [S, T]
 *   row_pos dev int32 [S, R]  canvas positions whose logits are wanted; a negative entry
 *                             yields a row of zeros
 *   logits  dev [S, R, vocab] in model dtype, unscaled (logit_scale is applied by the
 *                             epilogue). */
pvf_status pvf_forward(pvf_ctx *ctx, void *stream, const int32_t *tokens, int32_t S, int32_t T,
                       const int32_t *row_pos, int32_t R, void *logits);

/* Decision epilogue over logits [G, 1+K, R, vocab] (logits_dtype PVF_F32 / PVF_BF16), R the
 * window size defined above.  Slots above n_drafts[g] and done groups are not read.
 * plan_bitmap: dev, ceil(vocab/32) words, bit (id & 31) of word (id >> 5) set iff id is in
 * the planning vocabulary P^plan (Sec. 3).  ctx may be NULL (no workspace is used). */
pvf_status pvf_epilogue(pvf_ctx *ctx, void *stream, const void *logits, int32_t logits_dtype,
                        int32_t G, int32_t vocab, int32_t mask_id, const uint32_t *plan_bitmap,
                        const pvf_decode_cfg *cfg, const pvf_state *state);

/* With cfg->kv_cache = 1 the context keeps, per group, the cache and the block it was made for;
 * pvf_state_init invalidates it, and so does a round on a state other than the one the caches were
 * made for (states are told apart by their canvas buffer; a caller who rewrites a canvas in place
 * between rounds must call pvf_state_init or run one round with kv_cache = 0).  Such a round first reads done / n_drafts / k_active back
 * (one stream synchronisation) to split the groups into refreshing and cached ones; the
 * cache memory (2 * n_layers * T * d_model elements per group) is allocated on first use.
 *
 * forward + epilogue on the same stream, no synchronisation in between.  n_seq_host: if
 * > 0, the caller's count of live canvases sum_g (done[g] ? 0 : 1 + n_drafts[g]) as read
 * from the state after the previous round; only those are forwarded.  If <= 0 all
 * G*(1+K) slots are forwarded (same results, more work). */
pvf_status pvf_round(pvf_ctx *ctx, void *stream, int32_t G, const uint32_t *plan_bitmap,
                     const pvf_decode_cfg *cfg, const pvf_state *state, int32_t n_seq_host);

/* pvf_round, then the per-group status words read back with ONE copy and the stream synchronised:
 * status_host (host, 5*G int32) = { done, n_drafts, n_commit[0..2] } of every group after the round.
 * sum over live groups of 1 + n_drafts is the next round's n_seq_host.  pvf_decode loops over this. */
pvf_status pvf_round_sync(pvf_ctx *ctx, void *stream, int32_t G, const uint32_t *plan_bitmap,
                          const pvf_decode_cfg *cfg, const pvf_state *state, int32_t n_seq_host,
                          int32_t *status_host);

/* y_0 = [prompt | MASK^gen_len] in every slot, no drafts, k_active = 0, n_ws_blocks = 1, done = 0.
 *   prompt dev int32 [G, prompt_len]; must not contain mask_id (not checked on device). */
pvf_status pvf_state_init(pvf_ctx *ctx, void *stream, const int32_t *prompt, int32_t G,
                          const pvf_decode_cfg *cfg, const pvf_state *state);

/* Algorithm 1 to completion for G groups: pvf_state_init, then pvf_round until every group
 * is done.  Synchronises the stream once per round to read 5*G status words (one copy).
 *   out_tokens dev int32 [G, T]; stats host (may be NULL). */
pvf_status pvf_decode(pvf_ctx *ctx, void *stream, const int32_t *prompt, int32_t G,
                      const uint32_t *plan_bitmap, const pvf_decode_cfg *cfg,
                      const pvf_state *state, int32_t *out_tokens, pvf_stats *stats);

/* ---- building blocks, exported so that each kernel can be checked and timed alone ------- */

/* Stage 1 of the epilogue alone (Sec. 3: y-hat and p per position): for each of n_rows
 * rows of `logits` [n_rows, vocab], over all ids except mask_id,
 *   tok = lowest id attaining max_w x_w,  conf = 1 / sum_w exp(x_w - max x),
 *   x_w = logit_scale * logit_w.   conf dev float32 [n_rows], tok dev int32 [n_rows]. */
pvf_status pvf_stage1(void *stream, const void *logits, int32_t logits_dtype, int64_t n_rows,
                      int32_t vocab, int32_t mask_id, float logit_scale, float *conf,
                      int32_t *tok);

/* Entropy of the token distribution per row (Sec. 3, H_i): ent[r] = -sum_w p_w ln p_w with
 * p = softmax(logit_scale * logits[r]) over all ids except mask_id.  ent dev float32 [n_rows]. */
pvf_status pvf_entropy(void *stream, const void *logits, int32_t logits_dtype, int64_t n_rows,
                       int32_t vocab, int32_t mask_id, float logit_scale, float *ent);

/* Filtering rule of App. A.2: bit v of plan_bitmap (ceil(vocab/32) dev words, overwritten) is set
 * iff v != mask_id, n_v >= n_min, m_v >= m_min, a_v / m_v >= rho_ver and vig_v / n_v >= gamma_vig
 * (ratios in float64; a ratio with a zero denominator counts as 0).  Inputs are the accumulators of pvf_state, all dev. */
pvf_status pvf_plan_vocab_select(void *stream, const uint32_t *cal_n, const uint32_t *cal_m,
                                 const uint32_t *cal_a, const double *cal_vig, int32_t vocab,
                                 int32_t mask_id, uint32_t n_min, uint32_t m_min, float rho_ver,
                                 float gamma_vig, uint32_t *plan_bitmap);

/* C[M,N] = A[M,K] * W[N,K]^T (+ residual[M,N]); all dev, dtype PVF_F32 / PVF_BF16.
 * residual may be NULL and may alias C. */
pvf_status pvf_gemm(void *stream, int32_t dtype, const void *A, const void *W, void *C,
                    const void *residual, int32_t M, int32_t N, int32_t K);

/* The same products as a context launches them: with the context's workspace, launches of up to 640 rows
 * (the window forward of a K/V-cached round, the full forward of one short canvas) split K over several
 * workgroups per tile and add the float32 partial tiles in split order.  Operands in the context's dtype.
 * Launches of one context must not overlap (they share that workspace). */
pvf_status pvf_ctx_gemm(pvf_ctx *ctx, void *stream, const void *A, const void *W, void *C,
                        const void *residual, int32_t M, int32_t N, int32_t K);
pvf_status pvf_ctx_gemm_swiglu(pvf_ctx *ctx, void *stream, const void *A, const void *W, void *act,
                               int32_t M, int32_t ff, int32_t K);

/* act[M, ff] = silu(A W_gate^T) * (A W_up^T) with W [2*ff, K] (rows gate | up). */
pvf_status pvf_gemm_swiglu(void *stream, int32_t dtype, const void *A, const void *W, void *act,
                           int32_t M, int32_t ff, int32_t K);

/* out[M, d] = x / sqrt(mean(x^2) + eps) * gain. */
pvf_status pvf_rmsnorm(void *stream, int32_t dtype, const void *x, const void *gain, void *out,
                       int32_t M, int32_t d, float eps);

/* In-place rotary embedding of the q and k thirds of qkv [S*T, 3*d] (row m is canvas
 * position m % T), then out[S*T, d] = softmax(q k^T / sqrt(d_head)) v per canvas and head,
 * over all T keys.
 * Unlike the other calls this one is SYNCHRONOUS and ALLOCATES: it builds the rotary table on the
 * host, allocates the table and (bf16, d_head = 128) a key-contiguous copy of v with hipMalloc,
 * synchronises the stream and frees both before it returns.  It exists to check the kernels alone;
 * a round uses the context's table and workspace. */
pvf_status pvf_rope_attention(void *stream, int32_t dtype, void *qkv, void *out, int32_t S,
                              int32_t T, int32_t n_heads, int32_t d_head, float rope_theta);

/* pvf_rope_attention for callers that cannot allocate (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): same arguments and results, but the rotary table and the
 * key-contiguous copy of v live in a static device array of the library (17 MiB per GPU, held until
 * the process ends), the table is computed by a kernel on `stream`, and the call neither allocates,
 * frees nor synchronises.  Limits: T <= 2048, d_head <= 128, and on the bf16 / d_head = 128 path
 * S*T*n_heads*d_head <= 8 Mi elements; beyond them PVF_ESHAPE.  All calls on one GPU share that
 * array: calls that overlap on one GPU (different streams or threads) race; calls on one stream
 * are ordered and each rewrites everything it reads. */
pvf_status pvf_rope_attention_noalloc(void *stream, int32_t dtype, void *qkv, void *out, int32_t S,
                                      int32_t T, int32_t n_heads, int32_t d_head, float rope_theta);

/* The attention half of a layer as the forward runs it: qkv[S*T, 3*d] = x[S*T, d] * wqkv[3*d, d]^T,
 * rotary embedding of q and k, out[S*T, d] = attention.  On return qkv holds rotated q | rotated k
 * | v.  With bf16, d_head = 128 and T % 64 == 0 the rotation and the key-contiguous copy of v that
 * the attention kernel reads are fused into the projection's epilogue; the results equal
 * pvf_gemm followed by pvf_rope_attention up to the rounding of one fused multiply-add.
 * vt: dev [S, n_heads, 128, T] in dtype, or NULL.  On the fused path (bf16, d_head = 128, T % 64 == 0)
 * it receives the key-contiguous copy of v the attention kernel reads: vt[s][h][c][t'] = v[s*T + t][h*128 + c]
 * with t' = t with bits 2 and 3 exchanged (each 16 keys stored as 0-3, 8-11, 4-7, 12-15); on the other
 * paths it is left untouched.  NULL: the library allocates that copy itself.
 * Like pvf_rope_attention this call allocates its table (and vt if NULL) and synchronises the stream. */
pvf_status pvf_qkv_attention(void *stream, int32_t dtype, const void *x, const void *wqkv, void *qkv,
                             void *vt, void *out, int32_t S, int32_t T, int32_t n_heads, int32_t d_head,
                             float rope_theta);

/* Fills dev buffer with n values ~ N(0, std^2) (+ mean) from a counter-based generator;
 * used to materialise random-init weights of benchmark shapes directly in HBM. */
pvf_status pvf_fill_normal(void *stream, int32_t dtype, void *dst, int64_t n, uint64_t seed,
                           float mean, float std);

#ifdef __cplusplus
}
#endif
#endif /* PVF_H */
