// Offline side of PVF: the two kernels that the construction of the planning-token vocabulary
// needs beyond the decoding path (Sec. 3 "Verified information gain", App. A.2).
//
// entropy   H = -sum_w p_w ln p_w of softmax(logit_scale * logits) per row, the [MASK] column
//           excluded.  With t_w = x_w - max x:  H = ln S - U / S,  S = sum e^t,  U = sum t e^t.
//           One workgroup per row, two passes over the row (max, then the sums; the second
//           pass comes from L2: a full-width bf16 row is 253 KB).  The sums run in float64:
//           this kernel serves calibration runs, not the decoding loop, and is sized for
//           accuracy.  x_w is rounded to float32 once (fl32(scale * logit)) like in stage 1.
// select    the filtering rule: one thread per 32 vocabulary ids builds one bitmap word.
#include "common.h"

#include <math.h>

namespace pvf {
namespace {

constexpr int kEntBlock = 512;

template <typename T>
__global__ void __launch_bounds__(kEntBlock)
entropy_kernel(const T *__restrict__ logits, int vocab, int mask_id, float scale, RowFilter rf,
               float *__restrict__ ent) {
#pragma clang fp contract(off)   // x_w = fl32(scale * logit) is rounded before the max is subtracted
  const int tid = threadIdx.x;
  int64_t out_row;
  if (!row_target(rf, blockIdx.x, &out_row)) {
    if (tid == 0) ent[out_row] = 0.f;
    return;
  }
  const T *__restrict__ p = logits + (int64_t)blockIdx.x * vocab;
  __shared__ float s_m[kEntBlock / kWave];
  __shared__ double s_s[kEntBlock / kWave], s_u[kEntBlock / kWave];
  const int lane = tid % kWave, wid = tid / kWave;

  float m = -INFINITY;
  for (int w = tid; w < vocab; w += kEntBlock)
    if (w != mask_id) m = fmaxf(m, scale * to_float(p[w]));
  m = wave_max(m);
  if (lane == 0) s_m[wid] = m;
  __syncthreads();
  m = s_m[0];
#pragma unroll
  for (int i = 1; i < kEntBlock / kWave; ++i) m = fmaxf(m, s_m[i]);

  double S = 0.0, U = 0.0;
  for (int w = tid; w < vocab; w += kEntBlock) {
    if (w == mask_id) continue;
    const float t = scale * to_float(p[w]) - m;            // <= 0, exact for nearby values
    const double e = exp((double)t);
    S += e;
    if (t > -INFINITY) U += (double)t * e;                  // 0 * ln 0 = 0
  }
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) {
    S += __shfl_xor(S, o, kWave);
    U += __shfl_xor(U, o, kWave);
  }
  if (lane == 0) { s_s[wid] = S; s_u[wid] = U; }
  __syncthreads();
  if (tid == 0) {
    double St = 0.0, Ut = 0.0;
#pragma unroll
    for (int i = 0; i < kEntBlock / kWave; ++i) { St += s_s[i]; Ut += s_u[i]; }
    ent[out_row] = (float)(log(St) - Ut / St);
  }
}

__global__ void plan_vocab_select_kernel(const uint32_t *__restrict__ cal_n, const uint32_t *__restrict__ cal_m,
                                         const uint32_t *__restrict__ cal_a, const double *__restrict__ cal_vig,
                                         int vocab, int mask_id, uint32_t n_min, uint32_t m_min,
                                         float rho_ver, float gamma_vig, uint32_t *__restrict__ bitmap) {
  const int word = blockIdx.x * blockDim.x + threadIdx.x;
  if (word >= (vocab + 31) / 32) return;
  uint32_t bits = 0;
  for (int b = 0; b < 32; ++b) {
    const int v = word * 32 + b;
    if (v >= vocab || v == mask_id) continue;
    const uint32_t n = cal_n[v], m = cal_m[v];
    if (n < n_min || m < m_min) continue;
    const double r = m ? (double)cal_a[v] / (double)m : 0.0;   // r_ver = 0 when there was no opportunity
    const double g = n ? cal_vig[v] / (double)n : 0.0;
    if (r >= (double)rho_ver && g >= (double)gamma_vig) bits |= 1u << b;
  }
  bitmap[word] = bits;
}

}  // namespace

pvf_status launch_entropy(pvf_ctx *ctx, hipStream_t s, const void *logits, int dtype,
                          int64_t n_rows, int vocab, int mask_id, float scale,
                          const RowFilter &rf, float *ent) {
  if (n_rows == 0) return PVF_OK;
  PVF_REQUIRE(ctx, n_rows > 0 && n_rows < (1ll << 31), PVF_EINVAL, "entropy: n_rows=%lld out of range", (long long)n_rows);
  const dim3 grid((unsigned)n_rows);
  if (dtype == PVF_BF16)
    entropy_kernel<bf16_t><<<grid, kEntBlock, 0, s>>>(static_cast<const bf16_t *>(logits), vocab, mask_id, scale, rf, ent);
  else
    entropy_kernel<float><<<grid, kEntBlock, 0, s>>>(static_cast<const float *>(logits), vocab, mask_id, scale, rf, ent);
  PVF_LAUNCH_CHECK(ctx, "entropy");
  return PVF_OK;
}

pvf_status launch_plan_vocab_select(pvf_ctx *ctx, hipStream_t s, const uint32_t *cal_n,
                                    const uint32_t *cal_m, const uint32_t *cal_a,
                                    const double *cal_vig, int vocab, int mask_id, uint32_t n_min,
                                    uint32_t m_min, float rho_ver, float gamma_vig,
                                    uint32_t *plan_bitmap) {
  const int words = (vocab + 31) / 32;
  plan_vocab_select_kernel<<<(words + 255) / 256, 256, 0, s>>>(cal_n, cal_m, cal_a, cal_vig, vocab, mask_id,
                                                               n_min, m_min, rho_ver, gamma_vig, plan_bitmap);
  PVF_LAUNCH_CHECK(ctx, "plan_vocab_select");
  return PVF_OK;
}

}  // namespace pvf
