// Non-causal multi-head attention, plain version: out = softmax(q k^T / sqrt(dh)) v over all
// T keys of the same canvas, no mask of any kind (the denoiser sees the whole canvas, Sec. 2).
// One block = 8 queries of one (canvas, head); the full score rows live in LDS.  Any d_head,
// any dtype; this is the float32 path (dot products and sums in float64) and the fallback of
// the MFMA kernel (float32 accumulation).
#include "common.h"

#include <type_traits>

namespace pvf {
namespace {

constexpr int TQ = 8;

template <typename T>
__global__ void __launch_bounds__(256)
attention_simple_kernel(const T *__restrict__ qkv, T *__restrict__ out, int T_len, int n_heads,
                        int dh, float inv_sqrt_dh) {
  using Acc = typename std::conditional<std::is_same<T, float>::value, double, float>::type;
  constexpr bool kPrecise = std::is_same<T, float>::value;
  extern __shared__ float smem[];
  float *s_q = smem;                 // [TQ][dh]
  float *s_p = smem + TQ * dh;       // [TQ][T_len]
  const int tid = threadIdx.x;
  const int q0 = blockIdx.x * TQ, head = blockIdx.y, seq = blockIdx.z;
  const int d = n_heads * dh;
  const int64_t row0 = (int64_t)seq * T_len;
  const T *qb = qkv + row0 * 3 * d + (int64_t)head * dh;
  const T *kb = qb + d, *vb = qb + 2 * d;
  const int nq = min(TQ, T_len - q0);

  for (int i = tid; i < nq * dh; i += 256) {
    const int q = i / dh, c = i % dh;
    s_q[q * dh + c] = to_float(qb[(int64_t)(q0 + q) * 3 * d + c]);
  }
  __syncthreads();
  for (int i = tid; i < nq * T_len; i += 256) {
    const int k = i / nq, q = i % nq;
    const T *kr = kb + (int64_t)k * 3 * d;
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
    for (int k = 0; k < T_len; ++k) acc += (Acc)pr[k] * (Acc)to_float(vb[(int64_t)k * 3 * d + c]);
    out[(row0 + q0 + q) * d + (int64_t)head * dh + c] = from_float<T>((float)acc);
  }
}

}  // namespace

pvf_status launch_attention_simple(pvf_ctx *ctx, hipStream_t s, int dtype, const void *qkv,
                                   void *out, int S, int T, int n_heads, int d_head) {
  if (S == 0 || T == 0) return PVF_OK;
  const size_t lds = (size_t)TQ * (d_head + T) * sizeof(float);
  PVF_REQUIRE(ctx, lds <= 64 * 1024, PVF_ESHAPE, "attention: T=%d d_head=%d needs %zu bytes of LDS", T, d_head, lds);
  const dim3 grid((T + TQ - 1) / TQ, n_heads, S);
  const float isd = 1.0f / sqrtf((float)d_head);
  if (dtype == PVF_BF16)
    attention_simple_kernel<bf16_t><<<grid, 256, lds, s>>>((const bf16_t *)qkv, (bf16_t *)out, T, n_heads, d_head, isd);
  else
    attention_simple_kernel<float><<<grid, 256, lds, s>>>((const float *)qkv, (float *)out, T, n_heads, d_head, isd);
  PVF_LAUNCH_CHECK(ctx, "attention_simple");
  return PVF_OK;
}

}  // namespace pvf
