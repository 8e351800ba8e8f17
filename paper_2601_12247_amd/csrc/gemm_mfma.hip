// bf16 GEMM on the CDNA4 matrix cores:  C[M,N] = A[M,K] * W[N,K]^T, float32 accumulation,
// with the forward's fused epilogues (plain store, + residual, SwiGLU).  These GEMMs are
// >90% of a PVF round's time (the batched forward over backbone + drafts, Sec. 4.1).
//
// Shape of the kernel
//   * workgroup tile BM x BN (256 or 128 each), 4 waves in a 2 x 2 grid, each wave
//     (BM/2) x (BN/2) as v_mfma_f32_32x32x16_bf16 tiles (256 accumulator registers per lane at
//     256 x 256);
//   * both operands are K-contiguous in memory, so a 16-byte chunk is 8 consecutive k of one
//     row.  K advances in stages of BK (64 or 32) through a ring of LDS buffers; tiles go from
//     global memory straight into LDS (global_load_lds_dwordx4, no register staging) ahead of
//     the MFMAs; one raw s_barrier per stage, preceded by an explicit s_waitcnt vmcnt(n) that
//     lets the loads of later stages stay in flight;
//   * an LDS row is 2*BK bytes (8 or 4 chunks); the chunk position is XOR-swizzled with
//     (row >> 1) & 7 resp. (row >> 2) & 3 so that the ds_read_b128 of an MFMA operand
//     (consecutive rows, one chunk) touches every bank once.  The swizzle is applied by choosing
//     which global chunk a lane fetches, because the LDS slot of a direct load is fixed by the
//     lane id;
//   * the W tile is fed as the MFMA "A" operand and the activation tile as "B", so a lane ends
//     up with 4 consecutive output columns per accumulator group and stores 8 bytes at a time;
//   * workgroup ids are remapped so that the 32 workgroups resident on one XCD (ids congruent
//     mod 8) cover a patch of 8 x 4 output tiles and share operand tiles through that XCD's L2.
#include "common.h"

#include <cstdlib>
#include <type_traits>

namespace pvf {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kGroupM = 8;

typedef __attribute__((address_space(1))) const void gptr_t;
typedef __attribute__((address_space(3))) void lptr_t;

__device__ __forceinline__ float silu_f(float g) { return g / (1.0f + __expf(-g)); }

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  const bf16_t x = (bf16_t)a, y = (bf16_t)b;
  return (uint32_t)__builtin_bit_cast(uint16_t, x) | ((uint32_t)__builtin_bit_cast(uint16_t, y) << 16);
}

// s_waitcnt vmcnt(n) only (expcnt / lgkmcnt left at "no wait"); n is a 6-bit field split 4 + 2
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

// Row of W that feeds row r (0..BN-1) of the workgroup's W tile.
//  plain:   consecutive rows tile_n*BN + r.
//  SwiGLU:  the tile covers BN/2 output columns; inside each wave's BN/2 tile rows the 32-row
//           MFMA sub-tiles alternate gate / up for the same 32 columns, so silu(g)*u pairs
//           accumulators of one lane.
template <int EPI, int BN>
__device__ __forceinline__ int w_row(int r, int tile_n, int ff) {
  if (EPI != kEpiSwiglu) return tile_n * BN + r;
  const int wn = r / (BN / 2), t = (r % (BN / 2)) >> 5, e = r & 31;
  const int col = tile_n * (BN / 2) + wn * (BN / 4) + (t >> 1) * 32 + e;
  return (t & 1) ? ff + col : col;
}

template <int EPI, int BM, int BN, int BK, int kStages>
__global__ void __launch_bounds__(kThreads, (kStages * (BM + BN) * BK * 2 <= 80 * 1024) ? 2 : 1)
gemm_bf16_mfma_kernel(const bf16_t *__restrict__ A, const bf16_t *__restrict__ W,
                      bf16_t *__restrict__ C, const bf16_t *__restrict__ Res, int M, int N_out,
                      int K, int tiles_m, int tiles_n) {
  constexpr int MT = BM / 64, NT = BN / 64;          // MFMA tiles per wave in each direction
  constexpr int kATile = BM * BK * 2, kWTile = BN * BK * 2, kStage = kATile + kWTile;
  constexpr int CPR = BK / 8;                        // 16-byte chunks per LDS row
  constexpr int RPI = 256 / CPR;                     // tile rows covered by one load instruction of the block
  constexpr int LA = BM / RPI, LW = BN / RPI;        // direct loads per thread per stage
  constexpr int KS = BK / 16;                        // MFMA k-steps per stage
  constexpr int kRowBytes = BK * 2;
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

  // ---- global -> LDS: thread tid fills 16-byte slot (i*256 + tid) of an operand tile:
  //      tile row i*RPI + tid/CPR, slot position tid%CPR, k-chunk position ^ swizzle(row) ----
  const int ld_row = tid / CPR;
  const int ld_chunk = (tid % CPR) ^ (CPR == 8 ? (ld_row >> 1) & 7 : (ld_row >> 2) & 3);
  const bf16_t *a_src[LA], *w_src[LW];
#pragma unroll
  for (int i = 0; i < LA; ++i) {
    const int am = min(m0 + i * RPI + ld_row, M - 1);         // ragged last tile: re-read a valid row
    a_src[i] = A + (int64_t)am * K + ld_chunk * 8;
  }
#pragma unroll
  for (int i = 0; i < LW; ++i)
    w_src[i] = W + (int64_t)w_row<EPI, BN>(i * RPI + ld_row, tile_n, N_out) * K + ld_chunk * 8;
  auto issue_loads = [&](int kt) {
    unsigned char *dst = lds + (kt % kStages) * kStage + wave * 1024;
    const int koff = kt * BK;
#pragma unroll
    for (int i = 0; i < LA; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t *)(a_src[i] + koff), (lptr_t *)(dst + i * 4096), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < LW; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t *)(w_src[i] + koff), (lptr_t *)(dst + kATile + i * 4096), 16, 0, 0);
  };
  constexpr int kLoadsPerStage = LA + LW;
  auto issue_one = [&](int kt, int i) {                      // load i (A loads first, then W) of stage kt
    unsigned char *dst = lds + (kt % kStages) * kStage + wave * 1024;
    const int koff = kt * BK;
    if (i < LA)
      __builtin_amdgcn_global_load_lds((gptr_t *)(a_src[i] + koff), (lptr_t *)(dst + i * 4096), 16, 0, 0);
    else
      __builtin_amdgcn_global_load_lds((gptr_t *)(w_src[i - LA] + koff), (lptr_t *)(dst + kATile + (i - LA) * 4096), 16, 0, 0);
  };

  // ---- LDS -> MFMA operands: lane reads row (base + lane%32), chunk (2*kk + lane/32) ----
  const int fr = lane & 31, fh = lane >> 5;
  const int swz = CPR == 8 ? (fr >> 1) & 7 : (fr >> 2) & 3;
  int frag_off[KS];
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) frag_off[kk] = fr * kRowBytes + (((kk * 2 + fh) ^ swz) << 4);
  const int a_base = wm * (BM / 2) * kRowBytes;              // byte offset of the wave's rows in the A tile
  const int w_base = kATile + wn * (BN / 2) * kRowBytes;

  floatx16 acc[NT][MT];                                      // [n sub-tile][m sub-tile]
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[nt][mt][e] = 0.f;

  const int nk = K / BK;
#pragma unroll
  for (int s = 0; s < kStages - 1; ++s)
    if (s < nk) issue_loads(s);

  // Waits until at most n whole stages of this wave's direct loads are still in flight.
  auto wait_stages = [&](int n) {
    if (kStages >= 4 && n >= 2) wait_vmcnt<2 * kLoadsPerStage>();
    else if (kStages >= 3 && n >= 1) wait_vmcnt<kLoadsPerStage>();
    else wait_vmcnt<0>();
  };
  auto read_frags = [&](const unsigned char *stage, int kk, bf16x8 (&af)[MT], bf16x8 (&wf)[NT]) {
#pragma unroll
    for (int t = 0; t < MT; ++t)
      af[t] = *reinterpret_cast<const bf16x8 *>(stage + a_base + t * 32 * kRowBytes + frag_off[kk]);
#pragma unroll
    for (int t = 0; t < NT; ++t)
      wf[t] = *reinterpret_cast<const bf16x8 *>(stage + w_base + t * 32 * kRowBytes + frag_off[kk]);
  };

  // Software pipeline over k-steps (16 k each).  Invariant at the top of a stage: its first
  // fragments are already in registers.
  //  * fragments of k-step kk+1 are read while the MFMAs of k-step kk run; in the LAST k-step of
  //    stage kt the wave first waits for its own direct loads of stage kt+1, passes the block's
  //    one barrier per stage, and reads the first fragments of stage kt+1 -- so neither the
  //    barrier nor the LDS latency after it leaves the MFMA pipe empty;
  //  * that barrier also frees ring slot kt % kStages; the direct loads that refill it (stage
  //    kt + kStages) are issued during the first KS-1 k-steps of stage kt+1, a few per group of
  //    MT MFMAs rather than in one burst: a wave issues in order, and sixteen back-to-back
  //    vector-memory instructions from each of four waves stall the MFMAs queued behind them.
  constexpr int kGroups = (KS - 1) * NT;
  constexpr int kPerGroup = (kLoadsPerStage + kGroups - 1) / kGroups;
  bf16x8 af[2][MT], wf[2][NT];
  wait_stages(min(kStages - 2, nk - 1));
  __builtin_amdgcn_s_barrier();
  read_frags(lds, 0, af[0], wf[0]);
  auto run_stage = [&](int kt, auto with_loads) {
    const unsigned char *stage = lds + (kt % kStages) * kStage;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      const int cur = kk & 1, nxt = cur ^ 1;
      if (kk + 1 < KS) {
        read_frags(stage, kk + 1, af[nxt], wf[nxt]);
      } else if (kt + 1 < nk) {
        wait_stages(min(kStages - 2, nk - 2 - kt));          // stage kt+1 has landed (my part of it)
        __builtin_amdgcn_s_waitcnt(0xc07f);                  // lgkmcnt(0): my reads of stage kt are done
        // Raw barrier (no fence): every wave has waited for its own direct loads and LDS reads.
        __builtin_amdgcn_s_barrier();
        read_frags(lds + ((kt + 1) % kStages) * kStage, 0, af[nxt], wf[nxt]);
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        if (decltype(with_loads)::value && kk + 1 < KS) {
#pragma unroll
          for (int q = 0; q < kPerGroup; ++q) {
            const int i = (kk * NT + nt) * kPerGroup + q;
            if (i < kLoadsPerStage) issue_one(kt + kStages - 1, i);
          }
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          acc[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[cur][nt], af[cur][mt], acc[nt][mt], 0, 0, 0);
      }
    }
  };
  const int n_loading = nk - (kStages - 1);                  // stages that still have a stage to prefetch
  int kt = 0;
  for (; kt < n_loading; ++kt) run_stage(kt, std::true_type{});
  for (; kt < nk; ++kt) run_stage(kt, std::false_type{});

  // ---- epilogue: lane holds, for sub-tile (nt, mt) and group i, the 4 consecutive columns
  //      nt*32 + 8*i + 4*(lane/32) + {0..3} of row mt*32 + lane%32 ----
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = m0 + wm * (BM / 2) + mt * 32 + fr;
    if (m >= M) continue;
    if (EPI == kEpiSwiglu) {
      bf16_t *crow = C + (int64_t)m * N_out + tile_n * (BN / 2) + wn * (BN / 4);
#pragma unroll
      for (int p = 0; p < NT / 2; ++p)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float v[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] = silu_f(acc[2 * p][mt][4 * i + j]) * acc[2 * p + 1][mt][4 * i + j];
          uint2 o = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
          *reinterpret_cast<uint2 *>(crow + p * 32 + 8 * i + 4 * fh) = o;
        }
    } else {
      const int64_t off = (int64_t)m * N_out + tile_n * BN + wn * (BN / 2);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
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

template <int EPI, int BM, int BN, int BK, int ST>
pvf_status run(pvf_ctx *ctx, hipStream_t s, const void *A, const void *W, void *C, const void *Res,
               int M, int N_out, int K) {
  constexpr int kLdsBytes = ST * (BM + BN) * BK * 2;
  static_assert(kLdsBytes <= 160 * 1024, "LDS ring exceeds the 160 KB of a CU");
  static bool configured = false;
  if (!configured) {
    PVF_HIP_CHECK(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_bf16_mfma_kernel<EPI, BM, BN, BK, ST>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes));
    configured = true;
  }
  const int tiles_m = (M + BM - 1) / BM;
  const int tiles_n = (EPI == kEpiSwiglu) ? N_out / (BN / 2) : N_out / BN;
  const int total = tiles_m * tiles_n;
  const int grid = 8 * ((total + 7) / 8);
  gemm_bf16_mfma_kernel<EPI, BM, BN, BK, ST><<<grid, kThreads, kLdsBytes, s>>>(
      (const bf16_t *)A, (const bf16_t *)W, (bf16_t *)C, (const bf16_t *)Res, M, N_out, K, tiles_m, tiles_n);
  PVF_LAUNCH_CHECK(ctx, "gemm_mfma");
  return PVF_OK;
}

struct TileCfg { int bm, bn, bk, stages; double eff; };
constexpr int kNumCfg = 4;
constexpr TileCfg kCfg[kNumCfg] = {
    {256, 256, 32, 4, 1.00}, {128, 256, 64, 3, 0.85}, {256, 128, 64, 3, 0.85}, {128, 128, 64, 4, 0.80}};

template <int EPI>
pvf_status run_cfg(pvf_ctx *ctx, hipStream_t s, int cfg, const void *A, const void *W, void *C,
                   const void *Res, int M, int N, int K) {
  switch (cfg) {
    case 0: return run<EPI, 256, 256, 32, 4>(ctx, s, A, W, C, Res, M, N, K);
    case 1: return run<EPI, 128, 256, 64, 3>(ctx, s, A, W, C, Res, M, N, K);
    case 2: return run<EPI, 256, 128, 64, 3>(ctx, s, A, W, C, Res, M, N, K);
    default: return run<EPI, 128, 128, 64, 4>(ctx, s, A, W, C, Res, M, N, K);
  }
}

// Tile shape: the one with the least estimated time = rounds of workgroups over the 256 CUs
// x tile area / relative efficiency of the shape (measured on the forward's GEMM shapes: the
// smaller tiles re-read operands more often but quantise better when there are few tiles).
// PVF_GEMM_TILE=<n> in the environment forces shape n (for tuning runs).
int pick_config(GemmEpilogue epi, int M, int N, int K) {
  static const int forced = [] { const char *e = getenv("PVF_GEMM_TILE"); return e ? atoi(e) : -1; }();
  int best = -1;
  double best_t = 0;
  for (int c = 0; c < kNumCfg; ++c) {
    const int ncols = (epi == kEpiSwiglu) ? kCfg[c].bn / 2 : kCfg[c].bn;
    if (N % ncols != 0 || K % kCfg[c].bk != 0) continue;
    if (forced == c) return c;
    const int64_t tiles = (int64_t)((M + kCfg[c].bm - 1) / kCfg[c].bm) * (N / ncols);
    const double t = (double)((tiles + 255) / 256) * kCfg[c].bm * kCfg[c].bn / kCfg[c].eff;
    if (best < 0 || t < best_t) { best = c; best_t = t; }
  }
  return best;
}

}  // namespace

bool gemm_mfma_supported(int dtype, GemmEpilogue epi, int M, int N, int K) {
  if (dtype != PVF_BF16 || M < 1 || K < 64 || K % 64 != 0) return false;
  return N % (epi == kEpiSwiglu ? 64 : 128) == 0;
}

pvf_status launch_gemm_mfma(pvf_ctx *ctx, hipStream_t s, GemmEpilogue epi, const void *A,
                            const void *W, void *C, const void *residual, int M, int N, int K) {
  const uintptr_t al = (uintptr_t)A | (uintptr_t)W | (uintptr_t)C | (uintptr_t)residual;
  PVF_REQUIRE(ctx, (al & 15u) == 0, PVF_EINVAL, "gemm_mfma: operands must be 16-byte aligned");
  const int cfg = pick_config(epi, M, N, K);
  PVF_REQUIRE(ctx, cfg >= 0, PVF_ESHAPE, "gemm_mfma: no tile shape for N=%d", N);
  switch (epi) {
    case kEpiStore: return run_cfg<kEpiStore>(ctx, s, cfg, A, W, C, residual, M, N, K);
    case kEpiResidual: return run_cfg<kEpiResidual>(ctx, s, cfg, A, W, C, residual, M, N, K);
    case kEpiSwiglu: return run_cfg<kEpiSwiglu>(ctx, s, cfg, A, W, C, residual, M, N, K);
  }
  return PVF_EINVAL;
}

}  // namespace pvf
