// Block-level K/V cache for PVF decoding (the setting the paper's tokens/s are measured in,
// Sec. 5.1 "under KV cache").  While a block is being decoded the per-layer rotated keys and the
// values of every canvas position are kept from the full forward made when the block was
// entered; a cached round runs only the window rows of each canvas through the layers, and
// their queries attend to all T positions -- window positions through the keys / values just
// computed for this canvas, all others through the cache of the canvas' group.
//
// Kernels here: storing a full forward's K/V into the cache, token embedding / rotary embedding
// of window rows at their own canvas positions, and the window attention (plain version: any
// dtype and head size; float32 rows accumulate in float64 like the plain full attention).
#include "common.h"

#include <type_traits>

namespace pvf {
namespace {

// Window geometry of the canvas behind compact sequence s.
struct WinInfo {
  const int32_t *seq_slot;   // [n_seq] -> slot g*(1+K)+j
  const int32_t *k_active;   // [G]
  int32_t slots_per_group, prompt_len, block_len, T, R;
  __device__ __forceinline__ void get(int s, int *g, int *w0, int *n_valid) const {
    const int slot = seq_slot[s];
    *g = slot / slots_per_group;
    *w0 = prompt_len + k_active[*g] * block_len;
    *n_valid = min(R, T - *w0);
  }
};

// ---- cache store: K and V thirds of the backbone rows of a full forward -> cache[g][layer] ----
template <typename T>
__global__ void __launch_bounds__(256)
kv_store_kernel(const T *__restrict__ qkv, const int32_t *__restrict__ seq_slot, int slots_per_group,
                int T_len, int d, T *__restrict__ kc, T *__restrict__ vc, int64_t group_stride) {
  const int t = blockIdx.x, s = blockIdx.y;
  const int slot = seq_slot[s];
  if (slot % slots_per_group != 0) return;                 // drafts are not cached
  const int g = slot / slots_per_group;
  const T *row = qkv + ((int64_t)s * T_len + t) * 3 * d;
  T *kd = kc + g * group_stride + (int64_t)t * d;
  T *vd = vc ? vc + g * group_stride + (int64_t)t * d : nullptr;
  for (int i = threadIdx.x; i < d; i += 256) {
    kd[i] = row[d + i];
    if (vd) vd[i] = row[2 * d + i];
  }
}

// key-contiguous V copy [H*dh*T] of each backbone canvas (MFMA attention layout)
template <typename T>
__global__ void __launch_bounds__(256)
vt_store_kernel(const T *__restrict__ vt, const int32_t *__restrict__ seq_slot, int slots_per_group,
                int64_t n_per_seq, T *__restrict__ vtc, int64_t group_stride) {
  const int s = blockIdx.y;
  const int slot = seq_slot[s];
  if (slot % slots_per_group != 0) return;
  const int g = slot / slots_per_group;
  const uint4 *src = reinterpret_cast<const uint4 *>(vt + (int64_t)s * n_per_seq);
  uint4 *dst = reinterpret_cast<uint4 *>(vtc + g * group_stride);
  const int64_t nv = n_per_seq * sizeof(T) / 16;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nv; i += (int64_t)gridDim.x * 256) dst[i] = src[i];
}

// ---- window rows: embedding and rotary embedding at explicit canvas positions ----------------
template <typename T>
__global__ void __launch_bounds__(256)
embed_rows_kernel(const T *__restrict__ embed, const int32_t *__restrict__ canvas, const int32_t *__restrict__ seq_slot,
                  const int32_t *__restrict__ row_pos, int R, int T_len, int d, int vocab, T *__restrict__ out) {
  const int64_t m = blockIdx.x;                           // s*R + r
  const int s = (int)(m / R);
  int pos = row_pos[m];
  if (pos < 0) pos = T_len - 1;                           // padding row of a window cut by the canvas end
  int tok = canvas[(int64_t)seq_slot[s] * T_len + pos];
  tok = min(max(tok, 0), vocab - 1);
  const T *src = embed + (int64_t)tok * d;
  for (int i = threadIdx.x; i < d; i += 256) out[m * d + i] = src[i];
}

template <typename T>
__global__ void __launch_bounds__(256)
rope_rows_kernel(T *__restrict__ qkv, const int32_t *__restrict__ row_pos, int T_len, int n_heads, int dh,
                 const float2 *__restrict__ cos_sin) {
  const int64_t m = blockIdx.x;
  int pos = row_pos[m];
  if (pos < 0) pos = T_len - 1;
  const int half = dh / 2, d = n_heads * dh;
  T *row = qkv + m * 3 * (int64_t)d;
  for (int idx = threadIdx.x; idx < 2 * n_heads * half; idx += blockDim.x) {
    const int i = idx % half, hh = idx / half;            // q heads then k heads
    T *p = row + (int64_t)hh * dh;
    const float2 cs = cos_sin[(int64_t)pos * half + i];
    const float a = to_float(p[i]), b = to_float(p[i + half]);
    p[i] = from_float<T>(a * cs.x - b * cs.y);
    p[i + half] = from_float<T>(b * cs.x + a * cs.y);
  }
}

// ---- window attention, plain version -----------------------------------------------------------
// One block = 8 window rows (queries) of one (sequence, head); scores over all T keys in LDS.
constexpr int TQW = 8;

template <typename T>
__global__ void __launch_bounds__(256)
attention_window_kernel(const T *__restrict__ qkv_w, const T *__restrict__ kc, const T *__restrict__ vc,
                        int64_t group_stride, WinInfo wi, int n_heads, int dh, float inv_sqrt_dh,
                        T *__restrict__ out) {
  using Acc = typename std::conditional<std::is_same<T, float>::value, double, float>::type;
  constexpr bool kPrecise = std::is_same<T, float>::value;
  extern __shared__ float smem[];
  float *s_q = smem;                       // [TQW][dh]
  float *s_p = smem + TQW * dh;            // [TQW][T]
  const int tid = threadIdx.x;
  const int q0 = blockIdx.x * TQW, head = blockIdx.y, seq = blockIdx.z;
  const int T_len = wi.T, R = wi.R, d = n_heads * dh;
  int g, w0, n_valid;
  wi.get(seq, &g, &w0, &n_valid);
  const int nq = min(TQW, R - q0);
  const T *fresh = qkv_w + (int64_t)seq * R * 3 * d + (int64_t)head * dh;      // row r: + r*3d; k at +d, v at +2d
  const T *kcg = kc + g * group_stride + (int64_t)head * dh;                   // row t: + t*d
  const T *vcg = vc + g * group_stride + (int64_t)head * dh;

  for (int i = tid; i < nq * dh; i += 256) {
    const int q = i / dh, c = i % dh;
    s_q[q * dh + c] = to_float(fresh[(int64_t)(q0 + q) * 3 * d + c]);
  }
  __syncthreads();
  for (int i = tid; i < nq * T_len; i += 256) {
    const int k = i / nq, q = i % nq;
    const bool in_win = k >= w0 && k < w0 + n_valid;
    const T *kr = in_win ? fresh + (int64_t)(k - w0) * 3 * d + d : kcg + (int64_t)k * d;
    Acc acc = 0;
    for (int c = 0; c < dh; ++c) acc += (Acc)s_q[q * dh + c] * (Acc)to_float(kr[c]);
    s_p[q * T_len + k] = (float)(acc * (Acc)inv_sqrt_dh);
  }
  __syncthreads();
  const int lane = tid % kWave, wid = tid / kWave;
  for (int q = wid; q < nq; q += 256 / kWave) {
    float *pr = s_p + q * T_len;
    float m = -INFINITY;
    for (int k = lane; k < T_len; k += kWave) m = fmaxf(m, pr[k]);
    m = wave_max(m);
    float z = 0.f;
    for (int k = lane; k < T_len; k += kWave) {
      const float e = kPrecise ? expf(pr[k] - m) : __expf(pr[k] - m);
      pr[k] = e; z += e;
    }
    z = wave_sum(z);
    const float inv = 1.0f / z;
    for (int k = lane; k < T_len; k += kWave) pr[k] *= inv;
  }
  __syncthreads();
  for (int i = tid; i < nq * dh; i += 256) {
    const int q = i / dh, c = i % dh;
    const float *pr = s_p + q * T_len;
    Acc acc = 0;
    for (int k = 0; k < T_len; ++k) {
      const bool in_win = k >= w0 && k < w0 + n_valid;
      const T *vr = in_win ? fresh + (int64_t)(k - w0) * 3 * d + 2 * d : vcg + (int64_t)k * d;
      acc += (Acc)pr[k] * (Acc)to_float(vr[c]);
    }
    out[((int64_t)seq * R + q0 + q) * d + (int64_t)head * dh + c] = from_float<T>((float)acc);
  }
}

// row_pos[s*R + r] = canvas position of window row r of compact sequence s, or -1 past the end
__global__ void fill_row_pos_kernel(WinInfo wi, int n_seq, int32_t *__restrict__ row_pos) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_seq * wi.R) return;
  int g, w0, n_valid;
  wi.get(idx / wi.R, &g, &w0, &n_valid);
  const int r = idx % wi.R;
  row_pos[idx] = r < n_valid ? w0 + r : -1;
}

}  // namespace

static WinInfo make_win(const pvf_decode_cfg &cfg, const pvf_state &st, const int32_t *seq_slot) {
  WinInfo wi;
  wi.seq_slot = seq_slot; wi.k_active = st.k_active; wi.slots_per_group = 1 + cfg.K;
  wi.prompt_len = cfg.prompt_len; wi.block_len = cfg.block_len; wi.T = cfg.prompt_len + cfg.gen_len;
  wi.R = window_rows(cfg);
  return wi;
}

pvf_status launch_fill_row_pos(pvf_ctx *ctx, hipStream_t s, const pvf_decode_cfg &cfg, const pvf_state &st,
                               const int32_t *seq_slot, int n_seq, int32_t *row_pos) {
  if (n_seq == 0) return PVF_OK;
  const WinInfo wi = make_win(cfg, st, seq_slot);
  fill_row_pos_kernel<<<(n_seq * wi.R + 255) / 256, 256, 0, s>>>(wi, n_seq, row_pos);
  PVF_LAUNCH_CHECK(ctx, "fill_row_pos");
  return PVF_OK;
}

pvf_status launch_kv_store(pvf_ctx *ctx, hipStream_t s, int dtype, const void *qkv, const void *vt,
                           const int32_t *seq_slot, int slots_per_group, int S, int T, int d,
                           void *kc, void *vc, void *vtc, int64_t group_stride) {
  if (S == 0) return PVF_OK;
  const dim3 grid(T, S);
  if (dtype == PVF_BF16) {
    kv_store_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t *)qkv, seq_slot, slots_per_group, T, d,
                                                 (bf16_t *)kc, (bf16_t *)vc, group_stride);
    if (vtc) {
      PVF_LAUNCH_CHECK(ctx, "kv_store");
      vt_store_kernel<bf16_t><<<dim3(64, S), 256, 0, s>>>((const bf16_t *)vt, seq_slot, slots_per_group,
                                                          (int64_t)T * d, (bf16_t *)vtc, group_stride);
    }
  } else {
    kv_store_kernel<float><<<grid, 256, 0, s>>>((const float *)qkv, seq_slot, slots_per_group, T, d,
                                                (float *)kc, (float *)vc, group_stride);
  }
  PVF_LAUNCH_CHECK(ctx, "kv_store");
  return PVF_OK;
}

pvf_status launch_embed_rows(pvf_ctx *ctx, hipStream_t s, int dtype, const void *embed, const int32_t *canvas,
                             const int32_t *seq_slot, const int32_t *row_pos, int n_rows, int R, int T,
                             int d, int vocab, void *out) {
  if (n_rows == 0) return PVF_OK;
  if (dtype == PVF_BF16)
    embed_rows_kernel<bf16_t><<<n_rows, 256, 0, s>>>((const bf16_t *)embed, canvas, seq_slot, row_pos, R, T, d, vocab, (bf16_t *)out);
  else
    embed_rows_kernel<float><<<n_rows, 256, 0, s>>>((const float *)embed, canvas, seq_slot, row_pos, R, T, d, vocab, (float *)out);
  PVF_LAUNCH_CHECK(ctx, "embed_rows");
  return PVF_OK;
}

pvf_status launch_rope_rows(pvf_ctx *ctx, hipStream_t s, int dtype, void *qkv, const int32_t *row_pos,
                            int n_rows, int T, int n_heads, int d_head, const float2 *cos_sin) {
  if (n_rows == 0) return PVF_OK;
  if (dtype == PVF_BF16)
    rope_rows_kernel<bf16_t><<<n_rows, 256, 0, s>>>((bf16_t *)qkv, row_pos, T, n_heads, d_head, cos_sin);
  else
    rope_rows_kernel<float><<<n_rows, 256, 0, s>>>((float *)qkv, row_pos, T, n_heads, d_head, cos_sin);
  PVF_LAUNCH_CHECK(ctx, "rope_rows");
  return PVF_OK;
}

pvf_status launch_attention_window(pvf_ctx *ctx, hipStream_t s, int dtype, const void *qkv_w, const void *kc,
                                   const void *vc, int64_t group_stride, const pvf_decode_cfg &cfg,
                                   const pvf_state &st, const int32_t *seq_slot, int n_seq, int n_heads,
                                   int d_head, void *out) {
  if (n_seq == 0) return PVF_OK;
  const WinInfo wi = make_win(cfg, st, seq_slot);
  const size_t lds = (size_t)TQW * (d_head + wi.T) * sizeof(float);
  PVF_REQUIRE(ctx, lds <= 64 * 1024, PVF_ESHAPE, "window attention: T=%d d_head=%d needs %zu bytes of LDS", wi.T, d_head, lds);
  const dim3 grid((wi.R + TQW - 1) / TQW, n_heads, n_seq);
  const float isd = 1.0f / sqrtf((float)d_head);
  if (dtype == PVF_BF16)
    attention_window_kernel<bf16_t><<<grid, 256, lds, s>>>((const bf16_t *)qkv_w, (const bf16_t *)kc, (const bf16_t *)vc,
                                                           group_stride, wi, n_heads, d_head, isd, (bf16_t *)out);
  else
    attention_window_kernel<float><<<grid, 256, lds, s>>>((const float *)qkv_w, (const float *)kc, (const float *)vc,
                                                          group_stride, wi, n_heads, d_head, isd, (float *)out);
  PVF_LAUNCH_CHECK(ctx, "attention_window");
  return PVF_OK;
}

}  // namespace pvf
