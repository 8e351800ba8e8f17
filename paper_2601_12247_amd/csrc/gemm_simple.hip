// Plain LDS-tiled GEMM on the vector ALU:  C[M,N] = A[M,K] * W[N,K]^T, any M/N/K.  It is the
// float32 path of the forward (small parity model; accumulates in float64 so that its logits
// stay within a few float32 ulps of the exact ones) and the fallback for bf16 shapes that
// the MFMA kernel does not cover (float32 accumulation).
#include "common.h"

#include <type_traits>

namespace pvf {
namespace {

constexpr int BM = 64, BN = 64, BK = 16, TM = 4, TN = 4;

__device__ __forceinline__ float silu_acc(float g) { return g / (1.0f + __expf(-g)); }
__device__ __forceinline__ double silu_acc(double g) { return g / (1.0 + exp(-g)); }

template <typename T, int EPI>
__global__ void __launch_bounds__(256)
gemm_simple_kernel(const T *__restrict__ A, const T *__restrict__ W, T *__restrict__ C,
                   const T *__restrict__ residual, int M, int N, int K) {
  __shared__ float As[BK][BM + 4];
  __shared__ float Ws[BK][BN + 4];
  __shared__ float Us[EPI == kEpiSwiglu ? BK : 1][BN + 4];   // "up" rows for SwiGLU
  const int tid = threadIdx.x;
  const int tx = tid % 16, ty = tid / 16;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  using Acc = typename std::conditional<std::is_same<T, float>::value, double, float>::type;
  Acc acc[TM][TN] = {}, accu[TM][TN] = {};

  for (int k0 = 0; k0 < K; k0 += BK) {
    for (int i = tid; i < BM * BK; i += 256) {
      const int r = i / BK, kk = i % BK;
      const int gm = m0 + r, gk = k0 + kk;
      As[kk][r] = (gm < M && gk < K) ? to_float(A[(int64_t)gm * K + gk]) : 0.f;
      const int gn = n0 + r;
      Ws[kk][r] = (gn < N && gk < K) ? to_float(W[(int64_t)gn * K + gk]) : 0.f;
      if (EPI == kEpiSwiglu)
        Us[kk][r] = (gn < N && gk < K) ? to_float(W[((int64_t)N + gn) * K + gk]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[TM], b[TN], u[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) a[i] = As[kk][ty * TM + i];
#pragma unroll
      for (int j = 0; j < TN; ++j) b[j] = Ws[kk][tx * TN + j];
      if (EPI == kEpiSwiglu) {
#pragma unroll
        for (int j = 0; j < TN; ++j) u[j] = Us[kk][tx * TN + j];
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          acc[i][j] += (Acc)a[i] * (Acc)b[j];
          if (EPI == kEpiSwiglu) accu[i][j] += (Acc)a[i] * (Acc)u[j];
        }
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int gm = m0 + ty * TM + i, gn = n0 + tx * TN + j;
      if (gm >= M || gn >= N) continue;
      Acc v = acc[i][j];
      if (EPI == kEpiResidual) v += (Acc)to_float(residual[(int64_t)gm * N + gn]);
      if (EPI == kEpiSwiglu) v = silu_acc(v) * accu[i][j];
      C[(int64_t)gm * N + gn] = from_float<T>((float)v);
    }
}

template <typename T>
pvf_status run(pvf_ctx *ctx, hipStream_t s, GemmEpilogue epi, const T *A, const T *W, T *C,
               const T *res, int M, int N, int K) {
  const dim3 grid((N + BN - 1) / BN, (M + BM - 1) / BM);
  switch (epi) {
    case kEpiStore: gemm_simple_kernel<T, kEpiStore><<<grid, 256, 0, s>>>(A, W, C, res, M, N, K); break;
    case kEpiResidual: gemm_simple_kernel<T, kEpiResidual><<<grid, 256, 0, s>>>(A, W, C, res, M, N, K); break;
    case kEpiSwiglu: gemm_simple_kernel<T, kEpiSwiglu><<<grid, 256, 0, s>>>(A, W, C, res, M, N, K); break;
    default: PVF_REQUIRE(ctx, false, PVF_ENOTIMPL, "gemm_simple: epilogue %d exists only in the MFMA kernel", (int)epi);
  }
  PVF_LAUNCH_CHECK(ctx, "gemm_simple");
  return PVF_OK;
}

}  // namespace

pvf_status launch_gemm_simple(pvf_ctx *ctx, hipStream_t s, int dtype, GemmEpilogue epi,
                              const void *A, const void *W, void *C, const void *residual, int M,
                              int N, int K) {
  if (M == 0 || N == 0) return PVF_OK;
  if (dtype == PVF_BF16)
    return run<bf16_t>(ctx, s, epi, (const bf16_t *)A, (const bf16_t *)W, (bf16_t *)C, (const bf16_t *)residual, M, N, K);
  return run<float>(ctx, s, epi, (const float *)A, (const float *)W, (float *)C, (const float *)residual, M, N, K);
}

}  // namespace pvf
