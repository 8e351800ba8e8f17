// Shared declarations of libpvf's translation units (host side + small device helpers).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pvf.h"

namespace pvf {

typedef __bf16 bf16_t;

// ---- error reporting ---------------------------------------------------------------
// Records a printf-style message on the context (or in a thread-local slot if ctx == NULL).
void set_error(pvf_ctx *ctx, const char *fmt, ...);

#define PVF_HIP_CHECK(ctx, call)                                                         \
  do {                                                                                   \
    hipError_t e__ = (call);                                                             \
    if (e__ != hipSuccess) {                                                             \
      ::pvf::set_error(ctx, "%s: %s (%s:%d)", #call, hipGetErrorString(e__), __FILE__,  \
                       __LINE__);                                                        \
      return PVF_EHIP;                                                                   \
    }                                                                                    \
  } while (0)

#define PVF_LAUNCH_CHECK(ctx, what) PVF_HIP_CHECK(ctx, hipGetLastError())

#define PVF_REQUIRE(ctx, cond, code, ...)                                                \
  do {                                                                                   \
    if (!(cond)) {                                                                       \
      ::pvf::set_error(ctx, __VA_ARGS__);                                                \
      return code;                                                                       \
    }                                                                                    \
  } while (0)

// ---- device helpers ------------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) {
  return __uint_as_float(bits16 << 16);
}
__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_float(float x);
template <> __device__ __forceinline__ float from_float<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_float<bf16_t>(float x) { return (bf16_t)x; }

constexpr int kWave = 64;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}

// ---- kernel launchers (each defined in the .hip file holding its kernels) -------------
// Row filter of the epilogue's stage 1: which logits rows exist and where their summary goes.
struct RowFilter {
  const int32_t *n_drafts;  // [G] or NULL (NULL: every row is live, out row = in row)
  const int32_t *done;      // [G]
  const int32_t *k_active;  // [G]
  const int32_t *seq_slot;  // [n_seq] compact sequence -> slot g*(1+K)+j, or NULL (identity)
  int32_t slots_per_group;  // 1+K
  int32_t R, prompt_len, block_len, T;
};

// Where a logits row's summary goes and whether the row exists at all.
__device__ __forceinline__ bool row_target(const RowFilter &rf, int64_t row, int64_t *out_row) {
  *out_row = row;
  if (rf.n_drafts == nullptr) return true;
  const int s = (int)(row / rf.R), r = (int)(row % rf.R);
  const int slot = rf.seq_slot ? rf.seq_slot[s] : s;
  const int g = slot / rf.slots_per_group, j = slot % rf.slots_per_group;
  *out_row = (int64_t)slot * rf.R + r;
  if (rf.done[g] || j > rf.n_drafts[g]) return false;
  return rf.prompt_len + rf.k_active[g] * rf.block_len + r < rf.T;
}

pvf_status launch_stage1(pvf_ctx *ctx, hipStream_t s, const void *logits, int dtype,
                         int64_t n_rows, int vocab, int mask_id, float scale,
                         const RowFilter &rf, float *conf, int32_t *tok);

// rows of the decision window: min(c * block_len, gen_len), c = 2, or 4 with n_sparse > 0
int window_rows(const pvf_decode_cfg &c);

// entropy per logits row (calibration only); rows are filtered like stage 1
pvf_status launch_entropy(pvf_ctx *ctx, hipStream_t s, const void *logits, int dtype,
                          int64_t n_rows, int vocab, int mask_id, float scale,
                          const RowFilter &rf, float *ent);

pvf_status launch_plan_vocab_select(pvf_ctx *ctx, hipStream_t s, const uint32_t *cal_n,
                                    const uint32_t *cal_m, const uint32_t *cal_a,
                                    const double *cal_vig, int vocab, int mask_id, uint32_t n_min,
                                    uint32_t m_min, float rho_ver, float gamma_vig,
                                    uint32_t *plan_bitmap);

pvf_status launch_stage2(pvf_ctx *ctx, hipStream_t s, int G, int vocab, int mask_id,
                         const uint32_t *plan_bitmap, const pvf_decode_cfg &cfg,
                         const pvf_state &st);

pvf_status launch_state_init(pvf_ctx *ctx, hipStream_t s, const int32_t *prompt, int G,
                             int mask_id, const pvf_decode_cfg &cfg, const pvf_state &st);

// builds seq_slot[] and row_pos[] for a round; n_seq entries are written (padding repeats slot 0)
pvf_status launch_build_batch(pvf_ctx *ctx, hipStream_t s, int G, int n_seq,
                              const pvf_decode_cfg &cfg, const pvf_state &st,
                              int32_t *seq_slot, int32_t *row_pos);

// block-level K/V cache (kvcache.hip)
pvf_status launch_fill_row_pos(pvf_ctx *ctx, hipStream_t s, const pvf_decode_cfg &cfg, const pvf_state &st,
                               const int32_t *seq_slot, int n_seq, int32_t *row_pos);
pvf_status launch_kv_store(pvf_ctx *ctx, hipStream_t s, int dtype, const void *qkv, const void *vt,
                           const int32_t *seq_slot, int slots_per_group, int S, int T, int d,
                           void *kc, void *vc, void *vtc, int64_t group_stride);
pvf_status launch_embed_rows(pvf_ctx *ctx, hipStream_t s, int dtype, const void *embed, const int32_t *canvas,
                             const int32_t *seq_slot, const int32_t *row_pos, int n_rows, int R, int T,
                             int d, int vocab, void *out);
pvf_status launch_rope_rows(pvf_ctx *ctx, hipStream_t s, int dtype, void *qkv, const int32_t *row_pos,
                            int n_rows, int T, int n_heads, int d_head, const float2 *cos_sin);
pvf_status launch_attention_window(pvf_ctx *ctx, hipStream_t s, int dtype, const void *qkv_w, const void *kc,
                                   const void *vc, int64_t group_stride, const pvf_decode_cfg &cfg,
                                   const pvf_state &st, const int32_t *seq_slot, int n_seq, int n_heads,
                                   int d_head, void *out);

// out[5 g ..] = done, n_drafts, n_commit[0..2] of group g
pvf_status launch_pack_status(pvf_ctx *ctx, hipStream_t s, int G, const pvf_state &st, int32_t *out);

pvf_status launch_copy_out(pvf_ctx *ctx, hipStream_t s, int G, int K, int T,
                           const int32_t *canvas, int32_t *out_tokens);

// forward building blocks
// ss (bf16 only, may be NULL): ss[m] = sum of squares of row m
pvf_status launch_embed(pvf_ctx *ctx, hipStream_t s, int dtype, const void *embed,
                        const int32_t *tokens, const int32_t *seq_slot, int S, int T, int d,
                        int vocab, void *h, float *ss = nullptr);
// out[n, k] = bf16(w[n, k] * gain[k])
pvf_status launch_fold_gain(pvf_ctx *ctx, hipStream_t s, const void *w, const void *gain, void *out, int64_t n, int k);
pvf_status launch_rmsnorm(pvf_ctx *ctx, hipStream_t s, int dtype, const void *x,
                          const void *gain, void *out, int M, int d, float eps);
pvf_status launch_gather_rows(pvf_ctx *ctx, hipStream_t s, int dtype, const void *h,
                              const int32_t *row_pos, int S, int T, int R, int d, void *out);
pvf_status launch_rope(pvf_ctx *ctx, hipStream_t s, int dtype, void *qkv, int M, int T,
                       int n_heads, int d_head, const float2 *cos_sin);
enum GemmEpilogue { kEpiStore = 0, kEpiResidual = 1, kEpiSwiglu = 2, kEpiQkvRope = 3, kEpiPartial = 4 };
// RMSNorm folded into the projections around it (bf16 MFMA GEMMs of launches above the split-K range):
// the projection that writes the residual stream also writes, per output tile column `slot`, the sum of
// squares of each row's (rounded) values, ss[slot * ld + m]; the projection that reads the stream takes h
// itself as its operand, with the gain folded into its weights, and multiplies row m of its accumulators by
// rsqrt(sum over slots of ss / d + eps) in its epilogue.
struct NormArgs {
  float *ss_out = nullptr;        // kEpiResidual: where the row sums of squares of this launch go
  const float *ss_in = nullptr;   // kEpiSwiglu / kEpiQkvRope: row sums of squares of the operand rows
  int32_t n_slots_in = 0, ld = 0; // slots to add up; rows per slot
  float inv_d = 0.f, eps = 0.f;
};
// C[M,N] = A[M,K] W[N,K]^T; kEpiResidual adds residual[M,N]; kEpiSwiglu: W is [2N,K] (gate|up),
// C[M,N] = silu(gate) * up.
pvf_status launch_gemm(pvf_ctx *ctx, hipStream_t s, int dtype, GemmEpilogue epi, const void *A,
                       const void *W, void *C, const void *residual, int M, int N, int K);
// Pieces of the split-K path for launches of few rows.
// out[M, N] = epilogue(sum over splits of partial[z][M][Nw]) in split order (store, + residual, SwiGLU of gate | up halves)
pvf_status launch_splitk_finalize(pvf_ctx *ctx, hipStream_t s, GemmEpilogue epi, const float *partial, int splits,
                                  int M, int N, void *C, const void *residual);
// h[m, :] <- h[m, :] + sum over splits of partial[z][m][:] (rounded once), then out[m, :] = RMSNorm(h[m, :]) * gain
pvf_status launch_reduce_residual_rmsnorm(pvf_ctx *ctx, hipStream_t s, const float *partial, int splits, int M, int d,
                                          void *h, const void *gain, void *out, float eps);
bool reduce_residual_rmsnorm_supported(int dtype, int d);

pvf_status launch_fill_normal(pvf_ctx *ctx, hipStream_t s, int dtype, void *dst, int64_t n,
                              uint64_t seed, float mean, float std);

}  // namespace pvf
