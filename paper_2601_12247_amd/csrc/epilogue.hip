// Decision epilogue of a PVF round.
//
// stage 1  one pass over every live logits row: top-1 token (lowest id on ties, the [MASK]
//          column excluded) and its softmax probability (Sec. 3, definitions of y-hat and p).
//          The row is streamed once from HBM with 16-byte loads; the softmax itself is never
//          written anywhere.
// stage 2 (the decisions on those summaries) lives in decision.hip.
#include "common.h"

#include <math.h>

#include <type_traits>

namespace pvf {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegInf = -INFINITY;

// 2^x by the hardware instruction (no denormal fix-up: results below 2^-126 flush to 0).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ------------------------------------------------------------------------------------
// stage 1
// ------------------------------------------------------------------------------------
template <typename T> struct Vec16;  // how a 16-byte load splits into elements
template <> struct Vec16<bf16_t> {
  static constexpr int N = 8;
  static constexpr uint32_t kFill = 0xff80ff80u;  // two bf16 -inf
  __device__ static __forceinline__ void unpack(const uint4 &w, float *f) {
    f[0] = __uint_as_float(w.x << 16); f[1] = __uint_as_float(w.x & 0xffff0000u);
    f[2] = __uint_as_float(w.y << 16); f[3] = __uint_as_float(w.y & 0xffff0000u);
    f[4] = __uint_as_float(w.z << 16); f[5] = __uint_as_float(w.z & 0xffff0000u);
    f[6] = __uint_as_float(w.w << 16); f[7] = __uint_as_float(w.w & 0xffff0000u);
  }
};
template <> struct Vec16<float> {
  static constexpr int N = 4;
  static constexpr uint32_t kFill = 0xff800000u;  // -inf
  __device__ static __forceinline__ void unpack(const uint4 &w, float *f) {
    f[0] = __uint_as_float(w.x); f[1] = __uint_as_float(w.y);
    f[2] = __uint_as_float(w.z); f[3] = __uint_as_float(w.w);
  }
};

// 16-byte load with the non-temporal hint: a logits row is read exactly once, so it should not
// displace anything in the caches (measured: 6.5 instead of 5.9 TB/s on 2048 full-width rows).
__device__ __forceinline__ uint4 load_stream(const uint4 *p) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
  return make_uint4(t.x, t.y, t.z, t.w);
}

// Running (max, scaled sum) of one thread.  Values v live in the "compare domain": the raw
// logit for bf16 rows (scaling by a positive factor keeps order and ties of bf16 values), or
// logit_scale * logit for float rows.  Terms are 2^(v*c + nmc) with nmc = -fl(m*c); every
// term of the thread is therefore off by the same factor 2^delta, delta = m*c - fl(m*c),
// which is known exactly and divided out when the thread's sum is handed on.
struct Running {
  float m = kNegInf, z = 0.f, nmc = 0.f, delta = 0.f;
  int first = 0, cnt = 0;      // vectors first, first+BLOCK, .. (cnt of them) held the value that raised m
  __device__ __forceinline__ void raise(float gm, float c, int first_vec, int n_vec) {
    const float nmc2 = -(gm * c);
    const float d2 = fmaf(gm, c, nmc2);
    z *= fast_exp2((m - gm) * c - delta + d2);   // m = -inf on first use: z stays 0
    m = gm; nmc = nmc2; delta = d2; first = first_vec; cnt = n_vec;
  }
  __device__ __forceinline__ float true_sum() const { return z * fast_exp2(-delta); }
};

template <typename T, int BLOCK, int U>
__global__ void __launch_bounds__(BLOCK)
stage1_vec_kernel(const T *__restrict__ logits, int vocab, int mask_id, float scale,
                  RowFilter rf, float *__restrict__ conf, int32_t *__restrict__ tok) {
  constexpr int N = Vec16<T>::N;
  constexpr bool kRaw = (sizeof(T) == 2);
  const int tid = threadIdx.x;
  int64_t out_row;
  if (!row_target(rf, blockIdx.x, &out_row)) {
    if (tid == 0) { conf[out_row] = 0.f; tok[out_row] = -1; }
    return;
  }
  const uint4 *__restrict__ p =
      reinterpret_cast<const uint4 *>(logits + (int64_t)blockIdx.x * vocab);
  const int nvec = vocab / N;
  const int mask_vec = mask_id / N, mask_lane = mask_id % N;
  const float c = kRaw ? scale * kLog2e : kLog2e;
  constexpr int kStride = BLOCK * U;

  // Main loop: groups of U vectors per thread, no bounds checks; then a one-vector-at-a-time
  // tail.  A thread visits vector indices in increasing order, so the group in which its
  // running max was first raised to its final value holds the lowest id attaining it.
  Running run;
  const int nfull = nvec / kStride;
  // The [MASK] column lies in exactly one group iteration of the whole block; only that
  // iteration pays for the per-vector check (the others would otherwise spend one predicated
  // select per element on it).
  const int it_mask = mask_vec / kStride;
  auto group = [&](int it, auto check_mask) {
    const int base = it * kStride + tid;
    uint4 w[U];
#pragma unroll
    for (int u = 0; u < U; ++u) w[u] = load_stream(p + base + u * BLOCK);
    __builtin_amdgcn_sched_barrier(0);           // issue all U loads before touching any result
    float f[U][N];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      Vec16<T>::unpack(w[u], f[u]);
      if (!kRaw) {
#pragma unroll
        for (int i = 0; i < N; ++i) f[u][i] *= scale;
      }
      if (decltype(check_mask)::value && base + u * BLOCK == mask_vec) {
#pragma unroll
        for (int i = 0; i < N; ++i) if (i == mask_lane) f[u][i] = kNegInf;
      }
    }
    float gm = kNegInf;
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int i = 0; i < N; ++i) gm = fmaxf(gm, f[u][i]);
    if (gm > run.m) run.raise(gm, c, base, U);
    float acc = 0.f;
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int i = 0; i < N; ++i) acc += fast_exp2(fmaf(f[u][i], c, run.nmc));
    run.z += acc;
  };
  const int split = it_mask < nfull ? it_mask : nfull;
  for (int it = 0; it < split; ++it) group(it, std::false_type{});
  if (it_mask < nfull) group(it_mask, std::true_type{});
  for (int it = split + 1; it < nfull; ++it) group(it, std::false_type{});
  for (int idx = nfull * kStride + tid; idx < nvec; idx += BLOCK) {
    float f[N];
    Vec16<T>::unpack(load_stream(p + idx), f);
    if (!kRaw) {
#pragma unroll
      for (int i = 0; i < N; ++i) f[i] *= scale;
    }
    if (idx == mask_vec) {
#pragma unroll
      for (int i = 0; i < N; ++i) if (i == mask_lane) f[i] = kNegInf;
    }
    float gm = kNegInf;
#pragma unroll
    for (int i = 0; i < N; ++i) gm = fmaxf(gm, f[i]);
    if (gm > run.m) run.raise(gm, c, idx, 1);
    if (run.m > kNegInf) {                       // a vector holding only the mask column has no live value
#pragma unroll
      for (int i = 0; i < N; ++i) run.z += fast_exp2(fmaf(f[i], c, run.nmc));
    }
  }

  // ---- block reduction: max, then sum rescaled to the block max ----
  __shared__ float s_f[BLOCK / kWave];
  __shared__ int s_i[BLOCK / kWave];
  const int lane = tid % kWave, wid = tid / kWave;
  float M = wave_max(run.m);
  if (lane == 0) s_f[wid] = M;
  __syncthreads();
  M = s_f[0];
#pragma unroll
  for (int i = 1; i < BLOCK / kWave; ++i) M = fmaxf(M, s_f[i]);
  __syncthreads();
  float zt = (run.m > kNegInf) ? run.true_sum() * fast_exp2((run.m - M) * c) : 0.f;
  zt = wave_sum(zt);
  if (lane == 0) s_f[wid] = zt;

  // ---- arg-max: lowest id attaining M.  Each thread whose own max equals M rescans the
  // (at most U) vectors of the iteration in which it first reached that max. ----
  int cand = INT_MAX;
  if (run.m == M) {
    for (int u = 0; u < run.cnt && cand == INT_MAX; ++u) {
      const int idx = run.first + u * BLOCK;
      float f[N];
      Vec16<T>::unpack(p[idx], f);
#pragma unroll
      for (int i = N - 1; i >= 0; --i) {
        float v = kRaw ? f[i] : f[i] * scale;
        if (idx * N + i != mask_id && v == M) cand = idx * N + i;
      }
    }
  }
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) cand = min(cand, __shfl_xor(cand, o, kWave));
  if (lane == 0) s_i[wid] = cand;
  __syncthreads();
  if (tid == 0) {
    float Z = 0.f;
    int best = INT_MAX;
#pragma unroll
    for (int i = 0; i < BLOCK / kWave; ++i) { Z += s_f[i]; best = min(best, s_i[i]); }
    conf[out_row] = 1.0f / Z;
    tok[out_row] = best;
  }
}

// Any vocab size / alignment: one element per load.  Used for small test shapes only.
template <typename T, int BLOCK>
__global__ void __launch_bounds__(BLOCK)
stage1_scalar_kernel(const T *__restrict__ logits, int vocab, int mask_id, float scale,
                     RowFilter rf, float *__restrict__ conf, int32_t *__restrict__ tok) {
  const int tid = threadIdx.x;
  int64_t out_row;
  if (!row_target(rf, blockIdx.x, &out_row)) {
    if (tid == 0) { conf[out_row] = 0.f; tok[out_row] = -1; }
    return;
  }
  const T *__restrict__ p = logits + (int64_t)blockIdx.x * vocab;
  float m = kNegInf;
  int arg = INT_MAX;
  for (int w = tid; w < vocab; w += BLOCK) {
    if (w == mask_id) continue;
    const float x = scale * to_float(p[w]);
    if (x > m) { m = x; arg = w; }
  }
  __shared__ float s_f[BLOCK / kWave];
  __shared__ int s_i[BLOCK / kWave];
  const int lane = tid % kWave, wid = tid / kWave;
  float M = wave_max(m);
  if (lane == 0) s_f[wid] = M;
  __syncthreads();
  M = s_f[0];
  for (int i = 1; i < BLOCK / kWave; ++i) M = fmaxf(M, s_f[i]);
  __syncthreads();
  float z = 0.f;
  for (int w = tid; w < vocab; w += BLOCK) {
    if (w == mask_id) continue;
    z += fast_exp2((scale * to_float(p[w]) - M) * kLog2e);
  }
  z = wave_sum(z);
  int cand = (m == M) ? arg : INT_MAX;
  for (int o = kWave / 2; o > 0; o >>= 1) cand = min(cand, __shfl_xor(cand, o, kWave));
  if (lane == 0) { s_f[wid] = z; s_i[wid] = cand; }
  __syncthreads();
  if (tid == 0) {
    float Z = 0.f;
    int best = INT_MAX;
    for (int i = 0; i < BLOCK / kWave; ++i) { Z += s_f[i]; best = min(best, s_i[i]); }
    conf[out_row] = 1.0f / Z;
    tok[out_row] = best;
  }
}

}  // namespace

// ------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------
template <typename T>
static pvf_status launch_stage1_t(pvf_ctx *ctx, hipStream_t s, const T *logits, int64_t n_rows,
                                  int vocab, int mask_id, float scale, const RowFilter &rf,
                                  float *conf, int32_t *tok) {
  constexpr int N = Vec16<T>::N;
  const bool vec_ok = (vocab % N == 0) && ((reinterpret_cast<uintptr_t>(logits) & 15u) == 0);
  const dim3 grid((unsigned)n_rows);
  if (vec_ok && vocab / N >= 512) {
    stage1_vec_kernel<T, 1024, 2><<<grid, 1024, 0, s>>>(logits, vocab, mask_id, scale, rf, conf, tok);
  } else {
    stage1_scalar_kernel<T, 256><<<grid, 256, 0, s>>>(logits, vocab, mask_id, scale, rf, conf, tok);
  }
  PVF_LAUNCH_CHECK(ctx, "stage1");
  return PVF_OK;
}

pvf_status launch_stage1(pvf_ctx *ctx, hipStream_t s, const void *logits, int dtype,
                         int64_t n_rows, int vocab, int mask_id, float scale,
                         const RowFilter &rf, float *conf, int32_t *tok) {
  if (n_rows == 0) return PVF_OK;
  PVF_REQUIRE(ctx, n_rows > 0 && n_rows < (1ll << 31), PVF_EINVAL, "stage1: n_rows=%lld out of range", (long long)n_rows);
  if (dtype == PVF_BF16)
    return launch_stage1_t<bf16_t>(ctx, s, static_cast<const bf16_t *>(logits), n_rows, vocab, mask_id, scale, rf, conf, tok);
  return launch_stage1_t<float>(ctx, s, static_cast<const float *>(logits), n_rows, vocab, mask_id, scale, rf, conf, tok);
}

}  // namespace pvf
