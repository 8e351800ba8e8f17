// Memory-bound pieces of the denoiser forward: embedding gather, RMSNorm, window-row gather,
// rotary embedding, and a counter-based normal generator for random-init weights.
// The paper treats P_theta as a black box (Sec. 2); the architecture is this library's.
#include "common.h"

namespace pvf {
namespace {

// 16-byte vector of T
template <typename T> struct Pack { static constexpr int N = 16 / sizeof(T); };

// ---- embedding: h[s*T + t, :] = E[tokens[slot(s)*T + t], :] ----------------------------
template <typename T>
__global__ void __launch_bounds__(256)
embed_kernel(const T *__restrict__ embed, const int32_t *__restrict__ tokens,
             const int32_t *__restrict__ seq_slot, int T_len, int d, int vocab, T *__restrict__ h,
             float *__restrict__ ss_out) {
  const int64_t m = blockIdx.x;
  const int s = (int)(m / T_len), t = (int)(m % T_len);
  const int slot = seq_slot ? seq_slot[s] : s;
  int id = tokens[(int64_t)slot * T_len + t];
  id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);   // ids are validated on the host; stay in bounds regardless
  constexpr int N = Pack<T>::N;
  const uint4 *src = reinterpret_cast<const uint4 *>(embed + (int64_t)id * d);
  uint4 *dst = reinterpret_cast<uint4 *>(h + m * d);
  float ss = 0.f;
  for (int i = threadIdx.x; i < d / N; i += blockDim.x) {
    const uint4 v = src[i];
    dst[i] = v;
    if (sizeof(T) == 2 && ss_out) {                     // row sum of squares for the norm folded into the first projection
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float a = __uint_as_float(w[q] << 16), b = __uint_as_float(w[q] & 0xffff0000u);
        ss += a * a + b * b;
      }
    }
  }
  if (sizeof(T) == 2 && ss_out) {                       // uniform branch
    __shared__ float s_part[4];
    ss = wave_sum(ss);
    if (threadIdx.x % kWave == 0) s_part[threadIdx.x / kWave] = ss;
    __syncthreads();
    if (threadIdx.x == 0) ss_out[m] = s_part[0] + s_part[1] + s_part[2] + s_part[3];
  }
}

// out[n][k] = bf16(w[n][k] * gain[k]); one thread = 8 consecutive k
__global__ void __launch_bounds__(256)
fold_gain_kernel(const bf16_t *__restrict__ w, const bf16_t *__restrict__ gain, bf16_t *__restrict__ out, int64_t nvec, int kvec) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= nvec) return;
  const uint4 a = reinterpret_cast<const uint4 *>(w)[i], g = reinterpret_cast<const uint4 *>(gain)[i % kvec];
  const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, gw[4] = {g.x, g.y, g.z, g.w};
  uint32_t o[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const bf16_t lo = (bf16_t)(__uint_as_float(aw[q] << 16) * __uint_as_float(gw[q] << 16));
    const bf16_t hi = (bf16_t)(__uint_as_float(aw[q] & 0xffff0000u) * __uint_as_float(gw[q] & 0xffff0000u));
    o[q] = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
  }
  reinterpret_cast<uint4 *>(out)[i] = make_uint4(o[0], o[1], o[2], o[3]);
}

// ---- RMSNorm: out = x * rsqrt(mean(x^2) + eps) * gain, one row per block ---------------
template <typename T>
__global__ void __launch_bounds__(256)
rmsnorm_kernel(const T *__restrict__ x, const T *__restrict__ gain, T *__restrict__ out, int d,
               float eps) {
  const int64_t m = blockIdx.x;
  const T *xr = x + m * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += blockDim.x) { const float v = to_float(xr[i]); ss += v * v; }
  __shared__ float s_part[4];
  ss = wave_sum(ss);
  if (threadIdx.x % kWave == 0) s_part[threadIdx.x / kWave] = ss;
  __syncthreads();
  const float tot = s_part[0] + s_part[1] + s_part[2] + s_part[3];
  const float r = 1.0f / sqrtf(tot / (float)d + eps);
  for (int i = threadIdx.x; i < d; i += blockDim.x)
    out[m * d + i] = from_float<T>(to_float(xr[i]) * r * to_float(gain[i]));
}

// vectorised bf16 variant (d % 8 == 0): 16-byte loads, values kept in registers between passes
template <int MAXV>
__global__ void __launch_bounds__(256)
rmsnorm_bf16_vec_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ gain,
                        bf16_t *__restrict__ out, int d, float eps) {
  const int64_t m = blockIdx.x;
  const uint4 *xr = reinterpret_cast<const uint4 *>(x + m * d);
  const uint4 *gr = reinterpret_cast<const uint4 *>(gain);
  uint4 *orow = reinterpret_cast<uint4 *>(out + m * d);
  const int nvec = d / 8;
  uint4 v[MAXV];
  float ss = 0.f;
#pragma unroll
  for (int k = 0; k < MAXV; ++k) {
    const int i = threadIdx.x + k * 256;
    if (i < nvec) {
      v[k] = xr[i];
      const uint32_t w[4] = {v[k].x, v[k].y, v[k].z, v[k].w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float a = __uint_as_float(w[q] << 16), b = __uint_as_float(w[q] & 0xffff0000u);
        ss += a * a + b * b;
      }
    }
  }
  __shared__ float s_part[4];
  ss = wave_sum(ss);
  if (threadIdx.x % kWave == 0) s_part[threadIdx.x / kWave] = ss;
  __syncthreads();
  const float r = rsqrtf((s_part[0] + s_part[1] + s_part[2] + s_part[3]) / (float)d + eps);
#pragma unroll
  for (int k = 0; k < MAXV; ++k) {
    const int i = threadIdx.x + k * 256;
    if (i < nvec) {
      const uint4 g4 = gr[i];
      const uint32_t w[4] = {v[k].x, v[k].y, v[k].z, v[k].w};
      const uint32_t gw[4] = {g4.x, g4.y, g4.z, g4.w};
      uint32_t o[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float a = __uint_as_float(w[q] << 16) * r * __uint_as_float(gw[q] << 16);
        const float b = __uint_as_float(w[q] & 0xffff0000u) * r * __uint_as_float(gw[q] & 0xffff0000u);
        const bf16_t ab = (bf16_t)a, bb = (bf16_t)b;
        o[q] = (uint32_t)__builtin_bit_cast(uint16_t, ab) | ((uint32_t)__builtin_bit_cast(uint16_t, bb) << 16);
      }
      orow[i] = make_uint4(o[0], o[1], o[2], o[3]);
    }
  }
}

// ---- window-row gather: out[s*R + r, :] = h[s*T + row_pos[s*R + r], :] (zeros if < 0) ---
template <typename T>
__global__ void __launch_bounds__(256)
gather_rows_kernel(const T *__restrict__ h, const int32_t *__restrict__ row_pos, int T_len, int R,
                   int d, T *__restrict__ out) {
  const int64_t row = blockIdx.x;
  const int s = (int)(row / R);
  const int pos = row_pos[row];
  constexpr int N = Pack<T>::N;
  uint4 *dst = reinterpret_cast<uint4 *>(out + row * d);
  if (pos < 0 || pos >= T_len) {
    for (int i = threadIdx.x; i < d / N; i += blockDim.x) dst[i] = make_uint4(0, 0, 0, 0);
    return;
  }
  const uint4 *src = reinterpret_cast<const uint4 *>(h + ((int64_t)s * T_len + pos) * d);
  for (int i = threadIdx.x; i < d / N; i += blockDim.x) dst[i] = src[i];
}

// ---- rotary embedding, in place on the q and k thirds of qkv [M, 3d] --------------------
// pair (i, i + dh/2) of each head at canvas position m % T is rotated by cos_sin[pos][i].
template <typename T>
__global__ void __launch_bounds__(256)
rope_kernel(T *__restrict__ qkv, int T_len, int n_heads, int dh, const float2 *__restrict__ cos_sin) {
  const int64_t m = blockIdx.x;
  const int pos = (int)(m % T_len);
  const int half = dh / 2, d = n_heads * dh;
  T *row = qkv + m * 3 * (int64_t)d;
  for (int idx = threadIdx.x; idx < 2 * n_heads * half; idx += blockDim.x) {
    const int i = idx % half, hh = idx / half;        // hh in [0, 2*n_heads): q heads then k heads
    T *p = row + (int64_t)hh * dh;                    // k third starts right after the q third
    const float2 cs = cos_sin[(int64_t)pos * half + i];
    const float a = to_float(p[i]), b = to_float(p[i + half]);
    p[i] = from_float<T>(a * cs.x - b * cs.y);
    p[i + half] = from_float<T>(b * cs.x + a * cs.y);
  }
}

// ---- N(mean, std^2) fill from a counter-based generator ---------------------------------
__device__ __forceinline__ uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
template <typename T>
__global__ void fill_normal_kernel(T *__restrict__ dst, int64_t n, uint64_t seed, float mean, float std) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; 2 * p < n; p += stride) {
    const uint64_t r = mix64(mix64(seed) ^ (uint64_t)p);
    const float u1 = ((float)(uint32_t)(r >> 40) + 0.5f) * (1.0f / 16777216.0f);     // (0,1)
    const float u2 = (float)(uint32_t)((r >> 8) & 0xffffffu) * (1.0f / 16777216.0f);
    const float rad = sqrtf(-2.0f * __logf(u1));
    float sn, cs;
    __sincosf(6.283185307179586f * u2, &sn, &cs);
    dst[2 * p] = from_float<T>(mean + std * rad * cs);
    if (2 * p + 1 < n) dst[2 * p + 1] = from_float<T>(mean + std * rad * sn);
  }
}

}  // namespace

pvf_status launch_embed(pvf_ctx *ctx, hipStream_t s, int dtype, const void *embed,
                        const int32_t *tokens, const int32_t *seq_slot, int S, int T, int d,
                        int vocab, void *h, float *ss) {
  const unsigned M = (unsigned)(S * (int64_t)T);
  if (M == 0) return PVF_OK;
  if (dtype == PVF_BF16)
    embed_kernel<bf16_t><<<M, 256, 0, s>>>((const bf16_t *)embed, tokens, seq_slot, T, d, vocab, (bf16_t *)h, ss);
  else
    embed_kernel<float><<<M, 256, 0, s>>>((const float *)embed, tokens, seq_slot, T, d, vocab, (float *)h, nullptr);
  PVF_LAUNCH_CHECK(ctx, "embed");
  return PVF_OK;
}

pvf_status launch_fold_gain(pvf_ctx *ctx, hipStream_t s, const void *w, const void *gain, void *out, int64_t n, int k) {
  PVF_REQUIRE(ctx, k % 8 == 0 && n > 0, PVF_ESHAPE, "fold_gain: n=%lld k=%d", (long long)n, k);
  const int64_t nvec = n * (k / 8);
  fold_gain_kernel<<<(unsigned)((nvec + 255) / 256), 256, 0, s>>>((const bf16_t *)w, (const bf16_t *)gain, (bf16_t *)out, nvec, k / 8);
  PVF_LAUNCH_CHECK(ctx, "fold_gain");
  return PVF_OK;
}

pvf_status launch_rmsnorm(pvf_ctx *ctx, hipStream_t s, int dtype, const void *x, const void *gain,
                          void *out, int M, int d, float eps) {
  if (M == 0) return PVF_OK;
  if (dtype == PVF_BF16) {
    if (d % 8 == 0 && d / 8 <= 256 * 2)
      rmsnorm_bf16_vec_kernel<2><<<M, 256, 0, s>>>((const bf16_t *)x, (const bf16_t *)gain, (bf16_t *)out, d, eps);
    else
      rmsnorm_kernel<bf16_t><<<M, 256, 0, s>>>((const bf16_t *)x, (const bf16_t *)gain, (bf16_t *)out, d, eps);
  } else {
    rmsnorm_kernel<float><<<M, 256, 0, s>>>((const float *)x, (const float *)gain, (float *)out, d, eps);
  }
  PVF_LAUNCH_CHECK(ctx, "rmsnorm");
  return PVF_OK;
}

// Finishes a split-K projection that writes into the residual stream and norms the result for the next
// projection, one workgroup per row: h <- bf16(h + sum_z partial[z]) (split order, rounded once), then
// out = bf16(h * rsqrt(mean(h^2) + eps) * gain) on the rounded values -- what the residual epilogue followed
// by rmsnorm_bf16_vec_kernel computes, without writing and re-reading h in between.
template <int MAXV>
__global__ void __launch_bounds__(256)
reduce_residual_rmsnorm_kernel(const float *__restrict__ partial, int splits, int M, bf16_t *__restrict__ h,
                               const bf16_t *__restrict__ gain, bf16_t *__restrict__ out, int d, float eps) {
  const int64_t m = blockIdx.x;
  const int nvec = d / 8;
  uint4 *hr = reinterpret_cast<uint4 *>(h + m * d);
  const uint4 *gr = reinterpret_cast<const uint4 *>(gain);
  uint4 *orow = reinterpret_cast<uint4 *>(out + m * d);
  uint4 v[MAXV];
  float ss = 0.f;
#pragma unroll
  for (int k = 0; k < MAXV; ++k) {
    const int i = threadIdx.x + k * 256;
    if (i < nvec) {
      float a[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) a[e] = 0.f;
      for (int z0 = 0; z0 < splits; z0 += 4) {             // 4 splits in flight at a time, added in split order
        float4 p0[4], p1[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int z = min(z0 + j, splits - 1);
          const float4 *pr = reinterpret_cast<const float4 *>(partial + ((int64_t)z * M + m) * d + (int64_t)i * 8);
          p0[j] = pr[0]; p1[j] = pr[1];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (z0 + j < splits) {
            a[0] += p0[j].x; a[1] += p0[j].y; a[2] += p0[j].z; a[3] += p0[j].w;
            a[4] += p1[j].x; a[5] += p1[j].y; a[6] += p1[j].z; a[7] += p1[j].w;
          }
        }
      }
      const uint4 r4 = hr[i];
      const uint32_t rw[4] = {r4.x, r4.y, r4.z, r4.w};
      uint32_t o[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const bf16_t lo = (bf16_t)(a[2 * q] + __uint_as_float(rw[q] << 16));
        const bf16_t hi = (bf16_t)(a[2 * q + 1] + __uint_as_float(rw[q] & 0xffff0000u));
        o[q] = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
        const float x = __uint_as_float(o[q] << 16), y = __uint_as_float(o[q] & 0xffff0000u);
        ss += x * x + y * y;
      }
      v[k] = make_uint4(o[0], o[1], o[2], o[3]);
      hr[i] = v[k];
    }
  }
  __shared__ float s_part[4];
  ss = wave_sum(ss);
  if (threadIdx.x % kWave == 0) s_part[threadIdx.x / kWave] = ss;
  __syncthreads();
  const float r = rsqrtf((s_part[0] + s_part[1] + s_part[2] + s_part[3]) / (float)d + eps);
#pragma unroll
  for (int k = 0; k < MAXV; ++k) {
    const int i = threadIdx.x + k * 256;
    if (i < nvec) {
      const uint4 g4 = gr[i];
      const uint32_t w[4] = {v[k].x, v[k].y, v[k].z, v[k].w};
      const uint32_t gw[4] = {g4.x, g4.y, g4.z, g4.w};
      uint32_t o[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float a = __uint_as_float(w[q] << 16) * r * __uint_as_float(gw[q] << 16);
        const float b = __uint_as_float(w[q] & 0xffff0000u) * r * __uint_as_float(gw[q] & 0xffff0000u);
        const bf16_t ab = (bf16_t)a, bb = (bf16_t)b;
        o[q] = (uint32_t)__builtin_bit_cast(uint16_t, ab) | ((uint32_t)__builtin_bit_cast(uint16_t, bb) << 16);
      }
      orow[i] = make_uint4(o[0], o[1], o[2], o[3]);
    }
  }
}

bool reduce_residual_rmsnorm_supported(int dtype, int d) { return dtype == PVF_BF16 && d % 8 == 0 && d / 8 <= 256 * 2; }

pvf_status launch_reduce_residual_rmsnorm(pvf_ctx *ctx, hipStream_t s, const float *partial, int splits, int M, int d,
                                          void *h, const void *gain, void *out, float eps) {
  if (M == 0) return PVF_OK;
  PVF_REQUIRE(ctx, d % 8 == 0 && d / 8 <= 256 * 2 && splits >= 1, PVF_ESHAPE, "reduce_residual_rmsnorm: d=%d splits=%d", d, splits);
  reduce_residual_rmsnorm_kernel<2><<<M, 256, 0, s>>>(partial, splits, M, (bf16_t *)h, (const bf16_t *)gain, (bf16_t *)out, d, eps);
  PVF_LAUNCH_CHECK(ctx, "reduce_residual_rmsnorm");
  return PVF_OK;
}

pvf_status launch_gather_rows(pvf_ctx *ctx, hipStream_t s, int dtype, const void *h,
                              const int32_t *row_pos, int S, int T, int R, int d, void *out) {
  const unsigned rows = (unsigned)(S * (int64_t)R);
  if (rows == 0) return PVF_OK;
  if (dtype == PVF_BF16)
    gather_rows_kernel<bf16_t><<<rows, 256, 0, s>>>((const bf16_t *)h, row_pos, T, R, d, (bf16_t *)out);
  else
    gather_rows_kernel<float><<<rows, 256, 0, s>>>((const float *)h, row_pos, T, R, d, (float *)out);
  PVF_LAUNCH_CHECK(ctx, "gather_rows");
  return PVF_OK;
}

pvf_status launch_rope(pvf_ctx *ctx, hipStream_t s, int dtype, void *qkv, int M, int T,
                       int n_heads, int d_head, const float2 *cos_sin) {
  if (M == 0) return PVF_OK;
  if (dtype == PVF_BF16)
    rope_kernel<bf16_t><<<M, 256, 0, s>>>((bf16_t *)qkv, T, n_heads, d_head, cos_sin);
  else
    rope_kernel<float><<<M, 256, 0, s>>>((float *)qkv, T, n_heads, d_head, cos_sin);
  PVF_LAUNCH_CHECK(ctx, "rope");
  return PVF_OK;
}

pvf_status launch_fill_normal(pvf_ctx *ctx, hipStream_t s, int dtype, void *dst, int64_t n,
                              uint64_t seed, float mean, float std) {
  if (n <= 0) return PVF_OK;
  const int blocks = (int)((n / 2 + 255) / 256 < 65536 ? (n / 2 + 255) / 256 + 1 : 65536);
  if (dtype == PVF_BF16)
    fill_normal_kernel<bf16_t><<<blocks, 256, 0, s>>>((bf16_t *)dst, n, seed, mean, std);
  else
    fill_normal_kernel<float><<<blocks, 256, 0, s>>>((float *)dst, n, seed, mean, std);
  PVF_LAUNCH_CHECK(ctx, "fill_normal");
  return PVF_OK;
}

}  // namespace pvf
