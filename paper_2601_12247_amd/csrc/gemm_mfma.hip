// bf16 GEMM on the CDNA4 matrix cores:  C[M,N] = A[M,K] * W[N,K]^T, float32 accumulation,
// with the forward's fused epilogues (plain store, + residual, SwiGLU).  These GEMMs are
// >97% of a PVF round's work (the batched forward over backbone + drafts, Sec. 4.1).
//
// Shape of the kernel
//   * workgroup tile 256 x 256, K step 64, 4 waves in a 2 x 2 grid, each wave 128 x 128 as
//     4 x 4 v_mfma_f32_32x32x16_bf16 tiles (256 accumulator registers per lane);
//   * both operands are K-contiguous in memory, so a 16-byte chunk is 8 consecutive k of one
//     row.  Tiles go from global memory straight into LDS (global_load_lds_dwordx4, no
//     register staging); the k-chunk position inside a 128-byte LDS row is XOR-swizzled with
//     (row >> 1) & 7 so that the ds_read_b128 of an MFMA operand (32 consecutive rows, one
//     chunk) touches every bank once.  The swizzle is applied by choosing which global chunk a
//     lane fetches, because the LDS slot of a direct load is fixed by the lane id;
//   * LDS double buffer (2 x 64 KB): the loads of tile k+1 are in flight while tile k is
//     multiplied; one barrier per K step;
//   * the W tile is fed as the MFMA "A" operand and the activation tile as "B", so a lane ends
//     up with 4 consecutive output columns per accumulator group and stores 8 bytes at a time;
//   * workgroup ids are remapped so that the 32 workgroups resident on one XCD (ids congruent
//     mod 8) cover an 8 x 4 patch of output tiles and share operand tiles through that XCD's L2.
#include "common.h"

namespace pvf {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kThreads = 256;
constexpr int kTileBytes = BM * BK * 2;            // 32 KB per operand tile
constexpr int kStageBytes = 2 * kTileBytes;        // A tile + W tile
constexpr int kLdsBytes = 2 * kStageBytes;         // double buffer
constexpr int kGroupM = 8;

typedef __attribute__((address_space(1))) const void gptr_t;
typedef __attribute__((address_space(3))) void lptr_t;

__device__ __forceinline__ float silu_f(float g) { return g / (1.0f + __expf(-g)); }

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  const bf16_t x = (bf16_t)a, y = (bf16_t)b;
  return (uint32_t)__builtin_bit_cast(uint16_t, x) | ((uint32_t)__builtin_bit_cast(uint16_t, y) << 16);
}

// Row of W that feeds row r (0..255) of the workgroup's W tile.
//  plain:   consecutive rows n0 + r.
//  SwiGLU:  the tile covers 128 output columns f0..f0+127; inside each wave's 128 tile rows the
//           32-row MFMA sub-tiles alternate gate / up for the same 32 columns, so silu(g)*u
//           pairs accumulators of one lane.
template <int EPI>
__device__ __forceinline__ int w_row(int r, int tile_n, int ff) {
  if (EPI != kEpiSwiglu) return tile_n * BN + r;
  const int wn = r >> 7, t = (r >> 5) & 3, e = r & 31;
  const int col = tile_n * 128 + wn * 64 + (t >> 1) * 32 + e;
  return (t & 1) ? ff + col : col;
}

template <int EPI>
__global__ void __launch_bounds__(kThreads, 1)
gemm_bf16_mfma_kernel(const bf16_t *__restrict__ A, const bf16_t *__restrict__ W,
                      bf16_t *__restrict__ C, const bf16_t *__restrict__ Res, int M, int N_out,
                      int K, int tiles_m, int tiles_n) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // ---- XCD-aware tile assignment ----
  const int total = tiles_m * tiles_n;
  const int chunk = (total + 7) >> 3;
  const int L = (blockIdx.x & 7) * chunk + (blockIdx.x >> 3);
  if (L >= total) return;
  const int band = L / (kGroupM * tiles_n);
  const int within = L - band * (kGroupM * tiles_n);
  const int band_rows = min(kGroupM, tiles_m - band * kGroupM);
  const int tile_n = within / band_rows;
  const int tile_m = band * kGroupM + (within - tile_n * band_rows);
  const int m0 = tile_m * BM;

  // ---- global -> LDS: thread tid fills 16-byte slot (i*256 + tid) of each operand tile,
  //      i = 0..7: tile row i*32 + tid/8, slot position tid%8, k-chunk (tid%8) ^ swizzle ----
  const int ld_row = tid >> 3;
  const int ld_chunk = (tid & 7) ^ ((ld_row >> 1) & 7);
  const bf16_t *a_src[8], *w_src[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = i * 32 + ld_row;
    const int am = min(m0 + r, M - 1);                       // ragged last tile: re-read a valid row
    a_src[i] = A + (int64_t)am * K + ld_chunk * 8;
    w_src[i] = W + (int64_t)w_row<EPI>(r, tile_n, N_out) * K + ld_chunk * 8;
  }
  auto issue_loads = [&](int kt, int buf) {
    unsigned char *dst = lds + buf * kStageBytes + wave * 1024;
    const int koff = kt * BK;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_global_load_lds((gptr_t *)(a_src[i] + koff), (lptr_t *)(dst + i * 4096), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((gptr_t *)(w_src[i] + koff), (lptr_t *)(dst + kTileBytes + i * 4096), 16, 0, 0);
    }
  };

  // ---- LDS -> MFMA operands: lane reads row (base + lane%32), chunk (2*kk + lane/32) ----
  const int fr = lane & 31, fh = lane >> 5;
  const int swz = (fr >> 1) & 7;
  int frag_off[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) frag_off[kk] = fr * 128 + (((kk * 2 + fh) ^ swz) << 4);
  const int a_base = wm * 128 * 128;                         // byte offset of the wave's rows in the A tile
  const int w_base = kTileBytes + wn * 128 * 128;

  floatx16 acc[4][4];                                        // [n sub-tile][m sub-tile]
#pragma unroll
  for (int nt = 0; nt < 4; ++nt)
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[nt][mt][e] = 0.f;

  const int nk = K / BK;
  issue_loads(0, 0);
  for (int kt = 0; kt < nk; ++kt) {
    __builtin_amdgcn_s_waitcnt(0x0f70);                      // vmcnt(0): this wave's tile kt has landed
    __syncthreads();                                         // ... and everyone's; buffer (kt+1)&1 is free
    if (kt + 1 < nk) issue_loads(kt + 1, (kt + 1) & 1);
    const unsigned char *stage = lds + (kt & 1) * kStageBytes;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      bf16x8 af[4], wf[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        af[t] = *reinterpret_cast<const bf16x8 *>(stage + a_base + t * 4096 + frag_off[kk]);
        wf[t] = *reinterpret_cast<const bf16x8 *>(stage + w_base + t * 4096 + frag_off[kk]);
      }
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
          acc[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[nt], af[mt], acc[nt][mt], 0, 0, 0);
    }
  }

  // ---- epilogue: lane holds, for sub-tile (nt, mt) and group i, the 4 consecutive columns
  //      nt*32 + 8*i + 4*(lane/32) + {0..3} of row mt*32 + lane%32 ----
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) {
    const int m = m0 + wm * 128 + mt * 32 + fr;
    if (m >= M) continue;
    if (EPI == kEpiSwiglu) {
      bf16_t *crow = C + (int64_t)m * N_out + tile_n * 128 + wn * 64;
#pragma unroll
      for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float v[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] = silu_f(acc[2 * p][mt][4 * i + j]) * acc[2 * p + 1][mt][4 * i + j];
          uint2 o = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
          *reinterpret_cast<uint2 *>(crow + p * 32 + 8 * i + 4 * fh) = o;
        }
    } else {
      const int64_t off = (int64_t)m * N_out + tile_n * BN + wn * 128;
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int64_t o = off + nt * 32 + 8 * i + 4 * fh;
          float v[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] = acc[nt][mt][4 * i + j];
          if (EPI == kEpiResidual) {
            const uint2 r = *reinterpret_cast<const uint2 *>(Res + o);
            v[0] += __uint_as_float(r.x << 16); v[1] += __uint_as_float(r.x & 0xffff0000u);
            v[2] += __uint_as_float(r.y << 16); v[3] += __uint_as_float(r.y & 0xffff0000u);
          }
          *reinterpret_cast<uint2 *>(C + o) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
        }
    }
  }
}

template <int EPI>
pvf_status run(pvf_ctx *ctx, hipStream_t s, const void *A, const void *W, void *C, const void *Res,
               int M, int N_out, int K) {
  static bool configured = false;
  if (!configured) {
    PVF_HIP_CHECK(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_bf16_mfma_kernel<EPI>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes));
    configured = true;
  }
  const int tiles_m = (M + BM - 1) / BM;
  const int tiles_n = (EPI == kEpiSwiglu) ? N_out / 128 : N_out / BN;
  const int total = tiles_m * tiles_n;
  const int grid = 8 * ((total + 7) / 8);
  gemm_bf16_mfma_kernel<EPI><<<grid, kThreads, kLdsBytes, s>>>(
      (const bf16_t *)A, (const bf16_t *)W, (bf16_t *)C, (const bf16_t *)Res, M, N_out, K, tiles_m, tiles_n);
  PVF_LAUNCH_CHECK(ctx, "gemm_mfma");
  return PVF_OK;
}

}  // namespace

bool gemm_mfma_supported(int dtype, GemmEpilogue epi, int M, int N, int K) {
  if (dtype != PVF_BF16 || M < 1 || K < BK || K % BK != 0) return false;
  if (epi == kEpiSwiglu) return N % 128 == 0;
  return N % BN == 0;
}

pvf_status launch_gemm_mfma(pvf_ctx *ctx, hipStream_t s, GemmEpilogue epi, const void *A,
                            const void *W, void *C, const void *residual, int M, int N, int K) {
  const uintptr_t al = (uintptr_t)A | (uintptr_t)W | (uintptr_t)C | (uintptr_t)residual;
  PVF_REQUIRE(ctx, (al & 15u) == 0, PVF_EINVAL, "gemm_mfma: operands must be 16-byte aligned");
  switch (epi) {
    case kEpiStore: return run<kEpiStore>(ctx, s, A, W, C, residual, M, N, K);
    case kEpiResidual: return run<kEpiResidual>(ctx, s, A, W, C, residual, M, N, K);
    case kEpiSwiglu: return run<kEpiSwiglu>(ctx, s, A, W, C, residual, M, N, K);
  }
  return PVF_EINVAL;
}

}  // namespace pvf
