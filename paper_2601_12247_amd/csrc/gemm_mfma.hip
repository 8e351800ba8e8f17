// bf16 GEMM on the CDNA4 matrix cores:  C[M,N] = A[M,K] * W[N,K]^T, float32 accumulation,
// with the forward's fused epilogues (plain store, + residual, SwiGLU, and for the QKV projection
// the rotary embedding of q, k plus the key-contiguous copy of v).  These GEMMs are
// >90% of a PVF round's time (the batched forward over backbone + drafts, Sec. 4.1).
//
// Shape of the kernel
//   * workgroup tile BM x BN, WM x WN waves, each wave (BM/WM) x (BN/WN) as
//     v_mfma_f32_16x16x32_bf16 tiles (in a loop that also feeds LDS and direct loads this shape
//     sustains ~14% more than 32x32x16 at two waves per SIMD, although a loop of nothing but
//     MFMAs runs both at the same rate).  The shapes in use: 256 x 256 with 8 waves (2 x 4) for the
//     wide layers; 192 x 256, 128 x 256, 256 x 128, 160 x 256, 320 x 128, 192 x 128 and 128 x 128, also
//     with 8 waves, where they put (nearly) one tile on every CU; 64 x 64 and 64 x 128 with 4 waves for
//     launches with few rows, which stream the weights and want many workgroups with deep rings
//     (pick_config); launches of up to 640 rows may also split K over several workgroups per tile;
//   * both operands are K-contiguous in memory, so a 16-byte chunk is 8 consecutive k of one
//     row.  K advances in stages of BK = 64 (whole 128-byte lines per row: half the L2 requests
//     of 64-byte pieces) through a ring of LDS buffers; tiles go from
//     global memory straight into LDS (global_load_lds_dwordx4, no register staging) ahead of
//     the MFMAs; one raw s_barrier per stage, preceded by an explicit s_waitcnt vmcnt(n) that
//     lets the loads of later stages stay in flight.  The ring is as deep as the 160 KB of LDS
//     allow (two stages of the 256 x 256 tile, three of 160 x 256, five of 128 x 128): where a
//     stage lasts well under a microsecond the second stage of look-ahead is worth 10-15 %;
//   * an LDS row is 128 bytes (8 chunks); the chunk position is XOR-swizzled with
//     (row >> 1) & 7 so that the ds_read_b128 of an MFMA operand (16 consecutive rows, 4 chunk
//     positions) touches every bank once per 16 lanes.  The swizzle is applied by choosing
//     which global chunk a lane fetches, because the LDS slot of a direct load is fixed by the
//     lane id;
//   * the W tile is fed as the MFMA "A" operand and the activation tile as "B", so a lane ends
//     up with 4 consecutive output columns per accumulator group; the epilogue turns 32 rows at
//     a time around through LDS and stores whole 16-byte pieces of 128-byte lines;
//   * workgroup ids are remapped so that the 32 workgroups resident on one XCD (ids congruent
//     mod 8) cover a patch of 8 x 4 output tiles and share operand tiles through that XCD's L2.
#include "common.h"

#include <cstdlib>
#include <type_traits>

namespace pvf {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));


typedef __attribute__((address_space(1))) const void gptr_t;
typedef __attribute__((address_space(3))) void lptr_t;

__device__ __forceinline__ float silu_f(float g) { return g / (1.0f + __expf(-g)); }

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  const bf16_t x = (bf16_t)a, y = (bf16_t)b;
  return (uint32_t)__builtin_bit_cast(uint16_t, x) | ((uint32_t)__builtin_bit_cast(uint16_t, y) << 16);
}

// s_waitcnt vmcnt(n) only (expcnt / lgkmcnt left at "no wait"); n is a 6-bit field split 4 + 2
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

// Row of W that feeds row r (0..BN-1) of the workgroup's W tile.
//  plain:   consecutive rows tile_n*BN + r.
//  SwiGLU:  the tile covers BN/2 output columns; inside each wave's BN/WN tile rows groups of 32
//           rows alternate gate / up for the same 32 columns, so silu(g)*u pairs accumulators
//           of one lane (16-row MFMA sub-tiles 4P, 4P+1 with 4P+2, 4P+3).
//  QKV with rotary embedding (ff = 3 d): in the q and k thirds a wave's 64 tile rows are columns
//           [32g, 32g + 32) of a head followed by their rotation partners [64 + 32g, 64 + 32g + 32)
//           (g = wave % 2), so the pair (i, i + 64) meets in one lane (sub-tiles t and t + 2).
template <int EPI, int BN, int WN>
__device__ __forceinline__ int w_row(int r, int tile_n, int ff) {
  if (EPI == kEpiQkvRope) {
    if (tile_n * BN >= 2 * (ff / 3)) return tile_n * BN + r;           // v third: as it is
    const int wn = r >> 6, t = (r >> 4) & 3, e = r & 15;
    return tile_n * BN + (wn >> 1) * 128 + (t >> 1) * 64 + (wn & 1) * 32 + (t & 1) * 16 + e;
  }
  if (EPI != kEpiSwiglu) return tile_n * BN + r;
  constexpr int WT = BN / WN;
  const int wn = r / WT, t = (r % WT) >> 5, e = r & 31;
  const int col = tile_n * (BN / 2) + wn * (WT / 2) + (t >> 1) * 32 + e;
  return (t & 1) ? ff + col : col;
}

// workgroups per CU (by LDS) x waves per workgroup / 4 SIMDs
constexpr int waves_per_simd(int lds_bytes, int waves) { return (lds_bytes <= 80 * 1024 ? 2 : 1) * waves / 4; }

// kEpiQkvRope: the GEMM is the QKV projection of canvases of T tokens (d_head = 128, N = 3 * H * 128).
// Its epilogue rotates the q and k thirds (rotary embedding, pair (i, i + 64) of each head, angle
// of canvas position row % T from the cos_sin table [T][64]) before storing them, and writes the
// v third a second time key-contiguous, vt[canvas][head][d][t'] with bits 2 and 3 of t swapped in t'
// (each 16 keys stored as {0-3, 8-11 | 4-7, 12-15}), the layout the attention kernel reads its values in.
struct RopeArgs {
  const float2 *cos_sin;
  bf16_t *vt;
  int32_t T, H;
  int32_t store_v;                                   // 0: the v third of C is not written (only vt)
};

// kEpiPartial: the launch is split along K (blockIdx.y = split); every split stores its tile of float32
// partial sums to partial[split][M][N], which splitk_finalize_kernel adds up and finishes.
struct SplitK {
  float *partial;
  int32_t nk_per;                                    // k stages per split
};

template <int EPI, int BM, int BN, int BK, int kStages, int WM, int WN>
__global__ void __launch_bounds__(64 * WM * WN)
__attribute__((amdgpu_waves_per_eu(waves_per_simd(kStages * (BM + BN) * BK * 2, WM * WN),
                                   waves_per_simd(kStages * (BM + BN) * BK * 2, WM * WN))))
gemm_bf16_mfma_kernel(const bf16_t *__restrict__ A, const bf16_t *__restrict__ W,
                      bf16_t *__restrict__ C, const bf16_t *__restrict__ Res, int M, int N_out,
                      int K, int tiles_m, int tiles_n, int group_m, RopeArgs ra, SplitK sk, NormArgs na) {
  constexpr int kThreads = 64 * WM * WN;
  constexpr int MT = (BM / WM + 31) / 32;                  // 32-row passes of the epilogue (the last one may have 16 rows)
  constexpr int MT16 = BM / (16 * WM), NT16 = BN / (16 * WN);   // 16x16 MFMA tiles per wave in each direction
  constexpr int kATile = BM * BK * 2, kWTile = BN * BK * 2, kStage = kATile + kWTile;
  constexpr int CPR = BK / 8;                        // 16-byte chunks per LDS row
  constexpr int RPI = kThreads / CPR;                // tile rows covered by one load instruction of the block
  constexpr int kInstrBytes = kThreads * 16;         // LDS bytes filled by one load instruction of the block
  // A tile of 2.5 x RPI rows (160 x 256): the last A load instruction fills rows only from the lower half of the
  // block; the waves of the upper half repeat their previous load (same bytes to the same slot), so that every wave
  // has the same number of loads in flight and the same wait counts.
  constexpr bool kHalfA = BM % RPI != 0;
  constexpr int LA = (BM + RPI - 1) / RPI, LW = BN / RPI;        // direct loads per thread per stage
  constexpr int KS = BK / 32;                        // MFMA k-steps per stage
  constexpr int kRowBytes = BK * 2;
  // With a ring of only two stages the refill of a slot is issued as soon as the slot is free (right
  // after the barrier in the last k-step of the stage that was read from it), all of it in that one
  // k-step: the loads of stage kt + 2 then have a whole stage to land.  Deeper rings spread the refill
  // of the slot freed one stage ago over the first k-steps of a stage.
  constexpr bool kLate = kStages == 2;
  constexpr int kAhead = kLate ? kStages : kStages - 1;     // stages in flight after the prologue
  static_assert(BM % (RPI / 2) == 0 && (!kHalfA || LA >= 2) && BN % RPI == 0 && BK == 64 && BM % (16 * WM) == 0 && BN % (32 * WN) == 0, "tile shape");
  static_assert((EPI != kEpiQkvRope && EPI != kEpiSwiglu) || BM % (32 * WM) == 0, "the rotary and SwiGLU epilogues take whole 32-row passes");
  static_assert(EPI != kEpiSwiglu || NT16 % 4 == 0, "SwiGLU pairs 32-column gate/up groups inside a wave");
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: LDS targets become scalar arithmetic
  const int wm = wave / WN, wn = wave % WN;

  // ---- XCD-aware tile assignment ----
  const int total = tiles_m * tiles_n;
  const int chunk = (total + 7) >> 3;
  const int L = (blockIdx.x & 7) * chunk + (blockIdx.x >> 3);
  if (L >= total) return;
  const int band = L / (group_m * tiles_n);
  const int within = L - band * (group_m * tiles_n);
  const int band_rows = min(group_m, tiles_m - band * group_m);
  const int tile_n = within / band_rows;
  const int tile_m = band * group_m + (within - tile_n * band_rows);
  const int m0 = tile_m * BM;

  // ---- global -> LDS: thread tid fills 16-byte slot (i*kThreads + tid) of an operand tile:
  //      tile row i*RPI + tid/CPR, slot position tid%CPR, k-chunk position ^ swizzle(row) ----
  const int ld_row = tid / CPR;
  const int ld_chunk = (tid % CPR) ^ (CPR == 8 ? (ld_row >> 1) & 7 : (ld_row >> 2) & 3);
  // Per-lane byte offsets (32 bit) from the operand base; the k advance goes into the uniform
  // base pointer, so a load needs no per-lane address arithmetic.
  uint32_t a_off[LA], w_off[LW];
#pragma unroll
  for (int i = 0; i < LA; ++i) {
    const int am = min(m0 + i * RPI + ld_row, M - 1);         // ragged last tile: re-read a valid row
    a_off[i] = ((uint32_t)am * (uint32_t)K + ld_chunk * 8) * 2u;
  }
#pragma unroll
  for (int i = 0; i < LW; ++i)
    w_off[i] = ((uint32_t)w_row<EPI, BN, WN>(i * RPI + ld_row, tile_n, N_out) * (uint32_t)K + ld_chunk * 8) * 2u;
  const char *Ab = reinterpret_cast<const char *>(A), *Wb = reinterpret_cast<const char *>(W);
  if (EPI == kEpiPartial) {                                  // this split's range of k
    Ab += (size_t)blockIdx.y * sk.nk_per * (BK * 2);
    Wb += (size_t)blockIdx.y * sk.nk_per * (BK * 2);
  }
  constexpr int kLoadsPerStage = LA + LW;
  auto issue_one = [&](int kt, int i) {                      // load i (A loads first, then W) of stage kt
    unsigned char *dst = lds + (kt % kStages) * kStage + wave * 1024;
    const size_t koff = (size_t)kt * (BK * 2);
    if (i < LA) {
      const int ia = (kHalfA && i == LA - 1 && wave >= WM * WN / 2) ? i - 1 : i;      // uniform
      __builtin_amdgcn_global_load_lds((gptr_t *)(Ab + koff + a_off[ia]), (lptr_t *)(dst + ia * kInstrBytes), 16, 0, 0);
    } else
      __builtin_amdgcn_global_load_lds((gptr_t *)(Wb + koff + w_off[i - LA]), (lptr_t *)(dst + kATile + (i - LA) * kInstrBytes), 16, 0, 0);
  };

  // ---- LDS -> MFMA operands: lane reads row (base + lane%16), chunk (4*kk + lane/16) ----
  const int fr = lane & 15, fq = lane >> 4;
  const int swz = (fr >> 1) & 7;
  int frag_off[KS];
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) frag_off[kk] = fr * kRowBytes + (((kk * 4 + fq) ^ swz) << 4);
  const int a_base = wm * (BM / WM) * kRowBytes;             // byte offset of the wave's rows in the A tile
  const int w_base = kATile + wn * (BN / WN) * kRowBytes;

  floatx4 acc[NT16][MT16];                                   // [n sub-tile][m sub-tile]
#pragma unroll
  for (int nt = 0; nt < NT16; ++nt)
#pragma unroll
    for (int mt = 0; mt < MT16; ++mt)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[nt][mt][e] = 0.f;

  const int nk = EPI == kEpiPartial ? sk.nk_per : K / BK;
#pragma unroll
  for (int s = 0; s < kAhead; ++s)
    if (s < nk) {
#pragma unroll
      for (int i = 0; i < kLoadsPerStage; ++i) issue_one(s, i);
    }

  // Folded RMSNorm on the operand side: thread t < BM adds up the sums of squares of operand row m0 + t now,
  // while the first stages are in flight (8 loads at a time, slot order), and keeps 1 / rms for the epilogue.
  static_assert(BM <= kThreads, "one thread per tile row");
  float my_rnorm = 1.f;
  if ((EPI == kEpiSwiglu || EPI == kEpiQkvRope) && na.ss_in != nullptr && tid < BM) {
    const float *src = na.ss_in + min(m0 + tid, M - 1);
    float t = 0.f;
    for (int s0 = 0; s0 < na.n_slots_in; s0 += 8) {
      float v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = s0 + j < na.n_slots_in ? src[(int64_t)(s0 + j) * na.ld] : 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) t += v[j];
    }
    my_rnorm = rsqrtf(t * na.inv_d + na.eps);
  }

  // Waits until at most n whole stages of this wave's direct loads are still in flight.
  auto wait_stages = [&](int n) {
    if (kStages >= 4 && n >= 2) wait_vmcnt<2 * kLoadsPerStage>();
    else if ((kStages >= 3 || kLate) && n >= 1) wait_vmcnt<kLoadsPerStage>();
    else wait_vmcnt<0>();
  };
  // Operand fragments of a k-step (32 k).  The A fragments and the W fragment of the last pass
  // are double-buffered in registers; the other W fragments are single register sets that are
  // re-read for the next k-step right after the pass that used them.
  static_assert(KS % 2 == 0, "the register double buffer alternates with the k-step inside a stage");
  bf16x8 af[2][MT16], wf[NT16 - 1], wl[2];
  auto read_a = [&](const unsigned char *stage, int kk, int buf, int mt) {
    af[buf][mt] = *reinterpret_cast<const bf16x8 *>(stage + a_base + mt * 16 * kRowBytes + frag_off[kk]);
  };
  auto read_w = [&](const unsigned char *stage, int kk, int buf, int nt) {
    const bf16x8 v = *reinterpret_cast<const bf16x8 *>(stage + w_base + nt * 16 * kRowBytes + frag_off[kk]);
    if (nt == NT16 - 1) wl[buf] = v; else wf[nt] = v;
  };

  // Software pipeline over k-steps, written out in issue order and pinned with sched_barrier
  // after every MFMA: a wave issues in order, so whatever stands between two MFMAs must fit into
  // the cycles the first one keeps the matrix pipe busy.  A k-step runs its MFMAs n sub-tile by
  // n sub-tile (a "pass" = one W fragment against all A fragments).  The LDS reads for the NEXT
  // k-step follow single MFMAs and are all issued before the last pass starts, so a k-step never
  // begins by waiting for LDS.  The direct loads that fall to a k-step follow one MFMA each.
  // In the LAST k-step of stage kt the wave, kBarrierAt MFMAs in, waits for its own direct loads
  // of stage kt+1 and passes the block's one barrier per stage (its LDS reads of stage kt were
  // issued a pass or more ago); the fragments it reads after that are the first ones of stage kt+1.
  // A steady stage (one that still prefetches) has compile-time wait counts and no branches.
  constexpr int kMfmaPerStep = MT16 * NT16;
  constexpr int kVmPerStep = KS > 1 ? (kLoadsPerStage + KS - 2) / (KS - 1) : kLoadsPerStage;
  constexpr int kLateStride = (MT16 * NT16 - 4) / (LA + LW) >= 2 ? 2 : 1;   // every second MFMA where the k-step is long enough
  constexpr int kBarrierAt = MT16 - 1 < 4 ? MT16 - 1 : 4;   // MFMAs of the last k-step issued before the barrier
  // the A reads are spread over MFMAs (kBarrierAt, kReadEnd): up to the start of the last pass
  constexpr int kReadEnd = (NT16 - 1) * MT16 > kBarrierAt + 2 ? (NT16 - 1) * MT16 : kBarrierAt + 2;
  static_assert(!kLate || kLoadsPerStage * kLateStride <= kMfmaPerStep - kBarrierAt + kLateStride - 1, "the refill loads fit into the last k-step");
  static_assert(kReadEnd <= kMfmaPerStep, "the A reads fit into the k-step");
  wait_stages(min(kAhead - 1, nk - 1));
  __builtin_amdgcn_s_barrier();
#pragma unroll
  for (int nt = 0; nt < NT16; ++nt) read_w(lds, 0, 0, nt);
#pragma unroll
  for (int mt = 0; mt < MT16; ++mt) read_a(lds, 0, 0, mt);
  auto run_stage = [&](int kt, auto steady) {
    constexpr bool kSteady = decltype(steady)::value;
    const unsigned char *stage = lds + (kt % kStages) * kStage;
    const unsigned char *next = lds + ((kt + 1) % kStages) * kStage;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      const int cur = kk & 1, nxt = cur ^ 1;
      const bool last = kk + 1 == KS;
      const bool more = !last || kSteady || kt + 1 < nk;     // is there a next k-step to read for
      const unsigned char *src = last ? next : stage;
      const int skk = last ? 0 : kk + 1;
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < kMfmaPerStep; ++i) {
        const int nt = i / MT16, mt = i % MT16;
        if (last && more && i == kBarrierAt) {
          if (kSteady) wait_vmcnt<(kStages - 2) * kLoadsPerStage>();   // stage kt+1 has landed (my part of it)
          else wait_stages(min(kStages - 2, nk - 2 - kt));
          __builtin_amdgcn_s_waitcnt(0xc07f);                // lgkmcnt(0): my reads of stage kt are done
          // Raw barrier (no fence): every wave has waited for its own direct loads and LDS reads.
          __builtin_amdgcn_s_barrier();
          __builtin_amdgcn_sched_barrier(0);
        }
        acc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(nt == NT16 - 1 ? wl[cur] : wf[nt], af[cur][mt], acc[nt][mt], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (more) {
          if (i == kBarrierAt) read_w(src, skk, nxt, NT16 - 1);
#pragma unroll
          for (int m2 = 0; m2 < MT16; ++m2)
            if (i == kBarrierAt + 1 + (m2 * (kReadEnd - kBarrierAt - 1)) / MT16) read_a(src, skk, nxt, m2);
          if (mt == MT16 - 1 && nt < NT16 - 1) read_w(src, skk, nxt, nt);
        }
        if (!kLate && kSteady && !last) {
#pragma unroll
          for (int q = 0; q < kVmPerStep; ++q)
            if ((q * kMfmaPerStep) / kVmPerStep == i && kk * kVmPerStep + q < kLoadsPerStage)
              issue_one(kt + kStages - 1, kk * kVmPerStep + q);
        }
        // slot kt % kStages was freed by the barrier above: one refill load after every kLateStride-th MFMA
        if (kLate && kSteady && last && i >= kBarrierAt && (i - kBarrierAt) % kLateStride == 0 &&
            (i - kBarrierAt) / kLateStride < kLoadsPerStage)
          issue_one(kt + kStages, (i - kBarrierAt) / kLateStride);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  const int n_loading = nk - kAhead;                         // stages that still have a stage to prefetch
  int kt = 0;
  for (; kt < n_loading; ++kt) run_stage(kt, std::true_type{});
  for (; kt < nk; ++kt) run_stage(kt, std::false_type{});

  // ---- epilogue ----
  // A lane holds, for sub-tile (nt, mt), the 4 consecutive columns nt*16 + 4*(lane/16) + {0..3}
  // of row mt*16 + lane%16, so a direct store would write 8-byte pieces.  Instead each wave turns 32 rows at a time
  // around through its own piece of the (now free) LDS ring and stores 16 bytes per lane with
  // consecutive lanes along a row (whole 128-byte lines).  Staging is bf16 except for the
  // residual epilogue, which stages float32 so that acc + residual is rounded once.
  constexpr int WTM = BM / WM, WTN = BN / WN;
  constexpr int OC = (EPI == kEpiSwiglu) ? WTN / 2 : WTN;            // output columns of this wave
  constexpr bool kStageF32 = EPI == kEpiResidual || EPI == kEpiPartial;
  constexpr int kElem = kStageF32 ? 4 : 2;
  constexpr int kStride = OC * kElem + 16;                           // padded row of the staging area
  constexpr int LPR = OC / 8;                                        // lanes per output row (8 columns each)
  constexpr int kRowsPerInstr = 64 / LPR;
  static_assert(WM * WN * 32 * kStride <= kStages * kStage, "staging area exceeds the LDS ring");
  const int out_col0 = (EPI == kEpiSwiglu ? tile_n * (BN / 2) : tile_n * BN) + wn * OC;
  const int rd_row = lane / LPR, rd_col = (lane % LPR) * 8;
  // The residual rows of the whole wave tile are requested at once, before the staging starts:
  // fetched 32 rows at a time where they are added, each piece cost a full memory latency.
  constexpr int kRowIters = 32 / kRowsPerInstr;
  uint4 rs[EPI == kEpiResidual ? MT : 1][kRowIters];
  if (EPI == kEpiResidual) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int j = 0; j < kRowIters; ++j) {
        if (mt * 32 + j * kRowsPerInstr >= WTM) continue;            // beyond a last pass of 16 rows
        const int m = m0 + wm * WTM + mt * 32 + j * kRowsPerInstr + rd_row;
        rs[mt][j] = make_uint4(0, 0, 0, 0);
        if (m < M) rs[mt][j] = *reinterpret_cast<const uint4 *>(Res + (int64_t)m * N_out + out_col0 + rd_col);
      }
  }
  __syncthreads();                                                   // every wave is done with the ring
  // Folded RMSNorm: kNormOff bytes into the (free) ring lie above every staging area.  A reading projection
  // puts 1 / rms of its BM operand rows there; a writing one collects the row sums of squares of its output.
  // (The small tiles of the few-row launches have no room for it and never take part.)
  constexpr int kNormOff = 80 * 1024;
  constexpr bool kNormRoom = kNormOff + WN * BM * 4 <= kStages * kStage;
  float *norm_x = reinterpret_cast<float *>(lds + kNormOff);
  const bool norm_in = kNormRoom && (EPI == kEpiSwiglu || EPI == kEpiQkvRope) && na.ss_in != nullptr;     // uniform
  const bool norm_out = kNormRoom && EPI == kEpiResidual && na.ss_out != nullptr;                         // uniform
  if (norm_in) {
    if (tid < BM) norm_x[tid] = my_rnorm;
    __syncthreads();
  }
  const int rope_third = EPI == kEpiQkvRope ? (tile_n * BN) / (N_out / 3) : 2;   // 0 = q, 1 = k, 2 = v (uniform per workgroup)
  // v third of the QKV projection: a wave keeps two passes (64 keys) in its staging area, so that the
  // key-contiguous copy is written in whole 128-byte lines; columns are XOR-swizzled by the 16-key block
  // of the row, which makes the transposing 2-byte reads free of bank conflicts.
  constexpr int kVPasses = (EPI == kEpiQkvRope && WTM % 64 == 0) ? 2 : 1;
  static_assert(WM * WN * kVPasses * 32 * kStride <= kStages * kStage, "v staging area exceeds the LDS ring");
  static_assert(!kNormRoom || WM * WN * kVPasses * 32 * kStride <= kNormOff, "staging area reaches into the norm exchange area");
  const bool v_tile = EPI == kEpiQkvRope && rope_third == 2;
  unsigned char *my = lds + wave * ((v_tile ? kVPasses : 1) * 32 * kStride);
  // rotary epilogue: cos / sin of the lane's rows (2 halves of 16) and columns (2 sub-tiles x 4 pairs) of a
  // pass, requested one pass ahead
  const int rope_g = wn & 1;
  float4 csr[EPI == kEpiQkvRope ? 2 : 1][2][2][2];
  auto load_cs = [&](int mt) {
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
        const int m = m0 + wm * WTM + mt * 32 + h * 16 + fr;
        const float4 *cs4 = reinterpret_cast<const float4 *>(ra.cos_sin + (int64_t)(min(m, M - 1) % ra.T) * 64 + rope_g * 32 + nt * 16 + 4 * fq);
        csr[EPI == kEpiQkvRope ? mt & 1 : 0][h][nt][0] = cs4[0];
        csr[EPI == kEpiQkvRope ? mt & 1 : 0][h][nt][1] = cs4[1];
      }
  };
  if (EPI == kEpiQkvRope && rope_third < 2) load_cs(0);
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    if (EPI == kEpiQkvRope && rope_third < 2 && mt + 1 < MT) load_cs(mt + 1);
    // lane: row h*16 + lane%16 of the pass (h = 16-row half), 4 consecutive columns per n sub-tile
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      if (2 * mt + h >= MT16) continue;                                 // a last pass of 16 rows
      const int vp = v_tile ? mt % kVPasses : 0;                        // pass inside the v staging group
      unsigned char *wrow = my + (vp * 32 + h * 16 + fr) * kStride;
      const int xs = v_tile ? (2 * vp + h) << 3 : 0;                    // column swizzle of this 16-row block
      const int m16 = 2 * mt + h;
      if (norm_in) {                                                     // row m16 * 16 + fr of the wave tile
        const float rs = norm_x[wm * WTM + m16 * 16 + fr];
#pragma unroll
        for (int nt = 0; nt < NT16; ++nt)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[nt][m16][e] *= rs;
      }
      if (EPI == kEpiQkvRope && rope_third < 2) {
        // a = column i of the head (sub-tile nt), b = column i + 64 (sub-tile nt + 2), both rounded to bf16 first
        // (the values a separate rotary pass would read): i <- a cos - b sin, i + 64 <- b cos + a sin
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
          constexpr int kHalf = NT16 / 2;                     // 2 here; keeps the index valid in the other instances
          const int nb = nt % kHalf + kHalf;
          const uint32_t aw[2] = {pack_bf16x2(acc[nt % kHalf][m16][0], acc[nt % kHalf][m16][1]), pack_bf16x2(acc[nt % kHalf][m16][2], acc[nt % kHalf][m16][3])};
          const uint32_t bw[2] = {pack_bf16x2(acc[nb][m16][0], acc[nb][m16][1]), pack_bf16x2(acc[nb][m16][2], acc[nb][m16][3])};
          uint32_t lo[2], up[2];
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            const float4 c4 = csr[EPI == kEpiQkvRope ? mt & 1 : 0][h][nt][e];
            const float a0 = __uint_as_float(aw[e] << 16), a1 = __uint_as_float(aw[e] & 0xffff0000u);
            const float b0 = __uint_as_float(bw[e] << 16), b1 = __uint_as_float(bw[e] & 0xffff0000u);
            lo[e] = pack_bf16x2(a0 * c4.x - b0 * c4.y, a1 * c4.z - b1 * c4.w);
            up[e] = pack_bf16x2(b0 * c4.x + a0 * c4.y, b1 * c4.z + a1 * c4.w);
          }
          *reinterpret_cast<uint2 *>(wrow + (nt * 16 + 4 * fq) * 2) = make_uint2(lo[0], lo[1]);
          *reinterpret_cast<uint2 *>(wrow + (32 + nt * 16 + 4 * fq) * 2) = make_uint2(up[0], up[1]);
        }
      } else if (EPI == kEpiSwiglu) {
#pragma unroll
        for (int P = 0; P < NT16 / 4; ++P)
#pragma unroll
          for (int c = 0; c < 2; ++c) {                     // gate sub-tiles 4P, 4P+1; up sub-tiles 4P+2, 4P+3
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = silu_f(acc[4 * P + c][m16][j]) * acc[4 * P + 2 + c][m16][j];
            *reinterpret_cast<uint2 *>(wrow + (P * 32 + c * 16 + 4 * fq) * 2) =
                make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
          }
      } else {
#pragma unroll
        for (int nt = 0; nt < NT16; ++nt) {
          const int col = (nt * 16 + 4 * fq) ^ xs;
          if (kStageF32)
            *reinterpret_cast<float4 *>(wrow + col * 4) = make_float4(acc[nt][m16][0], acc[nt][m16][1], acc[nt][m16][2], acc[nt][m16][3]);
          else
            *reinterpret_cast<uint2 *>(wrow + col * 2) = make_uint2(pack_bf16x2(acc[nt][m16][0], acc[nt][m16][1]),
                                                                   pack_bf16x2(acc[nt][m16][2], acc[nt][m16][3]));
        }
      }
    }
    if (EPI == kEpiQkvRope) {
      static_assert(EPI != kEpiQkvRope || (WTN == 64 && WN % 2 == 0), "a head is two wave tiles wide");
      const int d_model = N_out / 3;
      const int m_base = m0 + wm * WTM + mt * 32;
      if (rope_third < 2) {
        // staged row: 32 columns from 32g of the head, then the 32 from 64 + 32g
        const int col = tile_n * BN + (wn >> 1) * 128 + rope_g * 32 + (rd_col < 32 ? rd_col : rd_col + 32);
#pragma unroll
        for (int j = 0; j < 32 / kRowsPerInstr; ++j) {
          const int r = j * kRowsPerInstr + rd_row;
          const int m = m_base + r;
          if (m < M) *reinterpret_cast<uint4 *>(C + (int64_t)m * N_out + col) =
                         *reinterpret_cast<const uint4 *>(my + r * kStride + rd_col * 2);
        }
      } else {
        const int vp = mt % kVPasses;
        if (ra.store_v)
#pragma unroll
        for (int j = 0; j < 32 / kRowsPerInstr; ++j) {               // v as it is ...
          const int r = j * kRowsPerInstr + rd_row;
          const int rl = vp * 32 + r;                                // row inside the staging group
          const int m = m_base + r;
          if (m < M) *reinterpret_cast<uint4 *>(C + (int64_t)m * N_out + out_col0 + rd_col) =
                         *reinterpret_cast<const uint4 *>(my + rl * kStride + ((rd_col ^ ((rl >> 4) << 3)) * 2));
        }
        // ... and key-contiguous, once the group's passes are staged: a lane gathers the 8 keys of one 16-byte
        // chunk of one d column (each 16 keys are stored as {0-3, 8-11 | 4-7, 12-15}); the lanes of a store
        // cover all chunks of 64 / chunks neighbouring columns
        const int key0 = m_base - vp * 32;
        if ((vp == kVPasses - 1 || mt == MT - 1) && key0 < M) {
          const int chunks = 4 * (vp + 1);                           // 16-byte chunks per column: 4 or 8
          const int seq = key0 / ra.T, t0 = key0 % ra.T;
          const int vcol0 = out_col0 - 2 * d_model;                  // column inside the v third
          const int g = lane % chunks, blk = g >> 1;
          const unsigned char *src = my + (16 * blk + 4 * (g & 1)) * kStride;
#pragma unroll
          for (int it = 0; it < chunks; ++it) {
            const int c = it * (64 / chunks) + lane / chunks;
            const unsigned char *sc = src + ((c ^ (blk << 3)) * 2);
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {                            // key pairs (0,1) (2,3) (8,9) (10,11) of the chunk's half
              const int kr = (e & 1) * 2 + (e >> 1) * 8;
              const uint32_t lo = *reinterpret_cast<const uint16_t *>(sc + kr * kStride);
              const uint32_t hi = *reinterpret_cast<const uint16_t *>(sc + (kr + 1) * kStride);
              w[e] = lo | (hi << 16);
            }
            const int head = (vcol0 + c) >> 7, dcol = (vcol0 + c) & 127;
            *reinterpret_cast<uint4 *>(ra.vt + (((int64_t)seq * ra.H + head) * 128 + dcol) * ra.T + t0 + g * 8) =
                make_uint4(w[0], w[1], w[2], w[3]);
          }
        }
      }
      continue;
    }
#pragma unroll
    for (int j = 0; j < 32 / kRowsPerInstr; ++j) {
      if (mt * 32 + j * kRowsPerInstr >= WTM) continue;              // beyond a last pass of 16 rows
      const int r = j * kRowsPerInstr + rd_row;
      const int m = m0 + wm * WTM + mt * 32 + r;
      const int64_t o = (int64_t)m * N_out + out_col0 + rd_col;
      if (EPI == kEpiPartial) {
        if (m < M) {
          float4 *dst = reinterpret_cast<float4 *>(sk.partial + (int64_t)blockIdx.y * M * N_out + o);
          dst[0] = *reinterpret_cast<const float4 *>(my + r * kStride + rd_col * 4);
          dst[1] = *reinterpret_cast<const float4 *>(my + r * kStride + rd_col * 4 + 16);
        }
        continue;
      }
      uint4 out;
      if (EPI == kEpiResidual) {
        const float4 x0 = *reinterpret_cast<const float4 *>(my + r * kStride + rd_col * 4);
        const float4 x1 = *reinterpret_cast<const float4 *>(my + r * kStride + rd_col * 4 + 16);
        const uint4 r4 = rs[EPI == kEpiResidual ? mt : 0][j];
        out.x = pack_bf16x2(x0.x + __uint_as_float(r4.x << 16), x0.y + __uint_as_float(r4.x & 0xffff0000u));
        out.y = pack_bf16x2(x0.z + __uint_as_float(r4.y << 16), x0.w + __uint_as_float(r4.y & 0xffff0000u));
        out.z = pack_bf16x2(x1.x + __uint_as_float(r4.z << 16), x1.y + __uint_as_float(r4.z & 0xffff0000u));
        out.w = pack_bf16x2(x1.z + __uint_as_float(r4.w << 16), x1.w + __uint_as_float(r4.w & 0xffff0000u));
      } else {
        out = *reinterpret_cast<const uint4 *>(my + r * kStride + rd_col * 2);
      }
      if (m < M) *reinterpret_cast<uint4 *>(C + o) = out;
      if (norm_out) {                                                    // sum of squares of the row's rounded values
        const uint32_t ow[4] = {out.x, out.y, out.z, out.w};
        float q = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float a = __uint_as_float(ow[e] << 16), b = __uint_as_float(ow[e] & 0xffff0000u);
          q += a * a + b * b;
        }
#pragma unroll
        for (int off = 1; off < LPR; off <<= 1) q += __shfl_xor(q, off, 64);   // the LPR lanes that share the row
        if (rd_col == 0) norm_x[wn * BM + wm * WTM + mt * 32 + r] = q;
      }
    }
  }
  if (norm_out) {                                                        // add the WN column parts in a fixed order
    __syncthreads();
    for (int row = tid; row < BM; row += kThreads) {
      float t = 0.f;
#pragma unroll
      for (int w = 0; w < WN; ++w) t += norm_x[w * BM + row];
      if (m0 + row < M) na.ss_out[(int64_t)tile_n * na.ld + m0 + row] = t;
    }
  }
}

template <int EPI, int BM, int BN, int BK, int ST, int WM, int WN>
pvf_status run(pvf_ctx *ctx, hipStream_t s, const void *A, const void *W, void *C, const void *Res,
               int M, int N_out, int K, const RopeArgs &ra, const SplitK &sk = SplitK{nullptr, 0}, int splits = 1,
               const NormArgs &na = NormArgs{}) {
  constexpr int kLdsBytes = ST * (BM + BN) * BK * 2;
  static_assert(kLdsBytes <= 160 * 1024, "LDS ring exceeds the 160 KB of a CU");
  // once per kernel instance; a function-local static is initialised exactly once even with concurrent callers
  static const hipError_t configured = hipFuncSetAttribute(
      reinterpret_cast<const void *>(gemm_bf16_mfma_kernel<EPI, BM, BN, BK, ST, WM, WN>),
      hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
  PVF_HIP_CHECK(ctx, configured);
  const int tiles_m = (M + BM - 1) / BM;
  const int tiles_n = (EPI == kEpiSwiglu) ? N_out / (BN / 2) : N_out / BN;
  const int total = tiles_m * tiles_n;
  const int grid = 8 * ((total + 7) / 8);
  // bands of at most kBand tile rows, all of (nearly) the same height: the 32 workgroups that run
  // together on an XCD then cover a patch of kBand x 32/kBand tiles in every band, whose operand rows
  // that XCD's L2 fetches once.  The patch that fetches least has rows : columns = BN : BM.
  constexpr int kBand = BM > BN ? 4 : 8;
  const int n_bands = (tiles_m + kBand - 1) / kBand;
  const int group_m = (tiles_m + n_bands - 1) / n_bands;
  gemm_bf16_mfma_kernel<EPI, BM, BN, BK, ST, WM, WN><<<dim3(grid, splits), 64 * WM * WN, kLdsBytes, s>>>(
      (const bf16_t *)A, (const bf16_t *)W, (bf16_t *)C, (const bf16_t *)Res, M, N_out, K, tiles_m, tiles_n, group_m, ra, sk, na);
  PVF_LAUNCH_CHECK(ctx, "gemm_mfma");
  return PVF_OK;
}

struct TileCfg { int bm, bn, bk, stages; double eff; bool plain_only; };
constexpr int kNumCfg = 10;
// Every shape for many rows runs 8 waves, two per SIMD (the two small ones 4 waves, two workgroups per CU):
// with one wave per SIMD the 256 x 256 tile (wave tiles of 128 x 128, a third fewer LDS reads) measured 2-4 %
// slower, smaller wave tiles far slower.
// plain_only: wave tiles 32 columns wide, which the SwiGLU and rotary epilogues cannot pair up, or 80 rows high
// (a last epilogue pass of 16 rows, which only the plain epilogues handle).
constexpr TileCfg kCfg[kNumCfg] = {
    {256, 256, 64, 2, 1.00, false},   // the wide layers
    {128, 256, 64, 3, 0.89, false}, {256, 128, 64, 3, 0.885, false},
    {128, 128, 64, 5, 0.70, false},   // launches of a single round of tiles: the smallest area finishes first
    {192, 256, 64, 2, 0.93, false},   // fills the chip when M / 256 leaves many CUs idle
    {320, 128, 64, 2, 0.78, true},    // 2560 rows = 8 tile rows: with N = 4096 exactly one tile per CU (wave tiles 80 x 64)
    {64, 64, 64, 5, 0.0, true},       // few rows (window forward of the K/V-cached rounds): the GEMM streams the weights,
    {64, 128, 64, 3, 0.0, false},     // so many small workgroups with deep rings; chosen by pick_config for M <= 384
    {192, 128, 64, 3, 0.86, true},    // 1536 rows = 8 tile rows: with N = 4096 one tile per CU
    {160, 256, 64, 3, 0.85, true}};   // 2560 rows = 16 tile rows: one tile per CU like 320 x 128, with room for a third stage

template <int EPI>
pvf_status run_cfg(pvf_ctx *ctx, hipStream_t s, int cfg, const void *A, const void *W, void *C,
                   const void *Res, int M, int N, int K, const RopeArgs &ra = RopeArgs{}, const NormArgs &na = NormArgs{}) {
  constexpr bool kPlain = EPI != kEpiSwiglu && EPI != kEpiQkvRope;
  switch (cfg) {
    case 0: return run<EPI, 256, 256, 64, 2, 2, 4>(ctx, s, A, W, C, Res, M, N, K, ra, SplitK{nullptr, 0}, 1, na);
    case 1: return run<EPI, 128, 256, 64, 3, 2, 4>(ctx, s, A, W, C, Res, M, N, K, ra, SplitK{nullptr, 0}, 1, na);
    case 2: return run<EPI, 256, 128, 64, 3, 4, 2>(ctx, s, A, W, C, Res, M, N, K, ra, SplitK{nullptr, 0}, 1, na);
    case 4: return run<EPI, 192, 256, 64, 2, 2, 4>(ctx, s, A, W, C, Res, M, N, K, ra, SplitK{nullptr, 0}, 1, na);
    case 5: if constexpr (kPlain) return run<EPI, 320, 128, 64, 2, 4, 2>(ctx, s, A, W, C, Res, M, N, K, ra, SplitK{nullptr, 0}, 1, na); break;
    case 6: if constexpr (kPlain) return run<EPI, 64, 64, 64, 5, 2, 2>(ctx, s, A, W, C, Res, M, N, K, ra, SplitK{nullptr, 0}, 1, na); break;
    case 7: return run<EPI, 64, 128, 64, 3, 2, 2>(ctx, s, A, W, C, Res, M, N, K, ra, SplitK{nullptr, 0}, 1, na);
    case 8: if constexpr (kPlain) return run<EPI, 192, 128, 64, 3, 2, 4>(ctx, s, A, W, C, Res, M, N, K, ra, SplitK{nullptr, 0}, 1, na); break;
    case 9: if constexpr (kPlain) return run<EPI, 160, 256, 64, 3, 2, 4>(ctx, s, A, W, C, Res, M, N, K, ra, SplitK{nullptr, 0}, 1, na); break;
    default: break;
  }
  return run<EPI, 128, 128, 64, 5, 4, 2>(ctx, s, A, W, C, Res, M, N, K, ra, SplitK{nullptr, 0}, 1, na);
}

// Tile shape: the one with the least estimated time = rounds of workgroups over the 256 CUs
// x tile area / relative efficiency of the shape (measured on the forward's GEMM shapes: the
// smaller tiles re-read operands more often but quantise better when there are few tiles).
// PVF_GEMM_TILE=<n> in the environment forces shape n (for tuning runs).
int pick_config(GemmEpilogue epi, int M, int N, int K) {
  static const int forced = [] { const char *e = getenv("PVF_GEMM_TILE"); return (e && e[0]) ? atoi(e) : -1; }();
  const bool plain = epi != kEpiSwiglu && epi != kEpiQkvRope;
  // Few rows: the launch streams the weight matrix once and is bound by HBM, not by the MFMAs.
  // Many small workgroups with deep LDS rings keep more bytes in flight (measured on the layer
  // shapes: 3.2x faster than the large tiles at M = 64, 2x at M = 320).
  // The output head (N = vocabulary) has enough tiles to fill the chip at any M > 64 and goes by the
  // cost model below.
  if (forced < 0 && M <= 384 && (M <= 64 || N <= 32768)) {
    if (plain && M <= 128 && N % 64 == 0) return 6;
    if (N % (epi == kEpiSwiglu ? 64 : 128) == 0) return 7;
  }
  int best = -1;
  double best_t = 0;
  for (int c = 0; c < kNumCfg; ++c) {
    const int ncols = (epi == kEpiSwiglu) ? kCfg[c].bn / 2 : kCfg[c].bn;
    if (N % ncols != 0 || K % kCfg[c].bk != 0 || (kCfg[c].plain_only && !plain)) continue;
    if (forced == c) return c;
    if (kCfg[c].eff <= 0.0) continue;
    const int64_t tiles = (int64_t)((M + kCfg[c].bm - 1) / kCfg[c].bm) * (N / ncols);
    const double t = (double)((tiles + 255) / 256) * kCfg[c].bm * kCfg[c].bn / kCfg[c].eff;
    if (best < 0 || t < best_t) { best = c; best_t = t; }
  }
  return best;
}

// Adds the partial sums of a split-K launch in split order (deterministic) and finishes like the
// fused epilogues: store, + residual (rounded once), or SwiGLU of the gate | up halves of a partial row.
// One thread = 8 consecutive output columns of one row.  Nw = length of a partial row.
template <int EPI>
__global__ void __launch_bounds__(256)
splitk_finalize_kernel(const float *__restrict__ partial, int splits, int M, int Nw, int N_out,
                       bf16_t *__restrict__ out, const bf16_t *__restrict__ res) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int per_row = N_out / 8;
  if (idx >= (int64_t)M * per_row) return;
  const int m = (int)(idx / per_row), c = (int)(idx % per_row) * 8;
  float v[8], u[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = u[e] = 0.f;
  for (int z = 0; z < splits; ++z) {
    const float *row = partial + ((int64_t)z * M + m) * Nw + c;
    const float4 a0 = *reinterpret_cast<const float4 *>(row), a1 = *reinterpret_cast<const float4 *>(row + 4);
    v[0] += a0.x; v[1] += a0.y; v[2] += a0.z; v[3] += a0.w; v[4] += a1.x; v[5] += a1.y; v[6] += a1.z; v[7] += a1.w;
    if (EPI == kEpiSwiglu) {
      const float4 b0 = *reinterpret_cast<const float4 *>(row + N_out), b1 = *reinterpret_cast<const float4 *>(row + N_out + 4);
      u[0] += b0.x; u[1] += b0.y; u[2] += b0.z; u[3] += b0.w; u[4] += b1.x; u[5] += b1.y; u[6] += b1.z; u[7] += b1.w;
    }
  }
  if (EPI == kEpiSwiglu) {
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = silu_f(v[e]) * u[e];
  }
  const int64_t o = (int64_t)m * N_out + c;
  if (EPI == kEpiResidual) {
    const uint4 rs = *reinterpret_cast<const uint4 *>(res + o);
    const uint32_t rw[4] = {rs.x, rs.y, rs.z, rs.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      v[2 * e] += __uint_as_float(rw[e] << 16);
      v[2 * e + 1] += __uint_as_float(rw[e] & 0xffff0000u);
    }
  }
  *reinterpret_cast<uint4 *>(out + o) = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]),
                                                   pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
}

constexpr int kSplitMaxRows = 640;   // launches with more rows have enough tiles without splitting K

// Tile shape and number of splits of a split-K launch; splits = 0: not possible.  The estimate is rounds of
// workgroups over the chip x (k stages per workgroup + ~8 stages' worth of prologue and epilogue).
// Up to 384 rows the tiles are as tall as the launch (64x128, 192x128, 320x128: all rows in one or two row
// tiles).  From there to 640 rows (one 512-token canvas) 128x128 tiles, and only where they would leave half
// the chip idle (the O and down projections: 128 tiles).
void splitk_plan(int M, int Nw, int K, size_t ws_floats, int *tile, int *splits) {
  *tile = M <= 64 ? 7 : M <= 192 ? 8 : M <= 384 ? 5 : 3;
  const int bm = M <= 64 ? 64 : M <= 192 ? 192 : M <= 384 ? 320 : 128;
  const int slots = M <= 64 ? 512 : 256;                     // the 4-wave shape runs two workgroups per CU
  const int tiles = ((M + bm - 1) / bm) * (Nw / 128), nk = K / 64;
  *splits = 0;
  if (M > 384 && tiles > 128) return;
  int best = 0;
  for (int sp = 1; sp <= 8; sp <<= 1) {
    if (nk % sp != 0 || nk / sp < 8 || (size_t)sp * M * Nw > ws_floats) continue;
    // 64-row tiles do little arithmetic per stage and are bound by the bytes in flight: as many workgroups as fit twice
    const int cost = M <= 64 ? (tiles * sp <= 2 * slots ? -sp : 1) : ((tiles * sp + slots - 1) / slots) * (nk / sp + 8);
    if (*splits == 0 || cost < best) { *splits = sp; best = cost; }
  }
}

}  // namespace

bool gemm_mfma_supported(int dtype, GemmEpilogue epi, int M, int N, int K);
bool gemm_mfma_norm_capable(int cfg);

// Few rows (window forward of the K/V-cached rounds, full forward of one short canvas): tiles as tall as
// the launch up to 384 rows, so that every weight row goes from L2 to a CU once, and K split over 2-8
// workgroups per tile to fill the chip and to shorten the serial k loop; a second small kernel adds the
// partial sums.  ws: float32 scratch.
bool gemm_mfma_splitk_supported(int dtype, GemmEpilogue epi, int M, int N, int K, size_t ws_floats) {
  if (epi == kEpiQkvRope || epi == kEpiPartial || !gemm_mfma_supported(dtype, epi, M, N, K)) return false;
  const int Nw = epi == kEpiSwiglu ? 2 * N : N;
  if (M > kSplitMaxRows || Nw % 128 != 0 || N % 8 != 0 || Nw > 32768) return false;
  int tile, splits;
  splitk_plan(M, Nw, K, ws_floats, &tile, &splits);
  // one split only for SwiGLU, whose fused epilogue the tall tiles (wave tiles 32 columns wide) do not have
  return splits >= 2 || (splits == 1 && epi == kEpiSwiglu && M > 128 && M <= 384);
}

// The split-K launch alone: float32 partial tiles ws[split][M][Nw] (Nw = weight rows: 2 N for SwiGLU); *splits_out
// = number of splits written.
pvf_status launch_gemm_mfma_splitk_partial(pvf_ctx *ctx, hipStream_t s, const void *A, const void *W, int M, int Nw, int K,
                                           float *ws, size_t ws_floats, int *splits_out) {
  const uintptr_t al = (uintptr_t)A | (uintptr_t)W | (uintptr_t)ws;
  PVF_REQUIRE(ctx, (al & 15u) == 0, PVF_EINVAL, "gemm_mfma: operands must be 16-byte aligned");
  int tile, splits;
  splitk_plan(M, Nw, K, ws_floats, &tile, &splits);
  PVF_REQUIRE(ctx, splits >= 1 && ws != nullptr, PVF_ESHAPE, "gemm_mfma: no split-K plan for M=%d N=%d K=%d", M, Nw, K);
  const SplitK sk{ws, K / 64 / splits};
  *splits_out = splits;
  // 193-384 rows: two (three) tile rows of 160 x 256 where the width allows it -- as many tiles as 320 x 128 and room for
  // a third stage, which these latency-bound launches want more than they mind fetching each weight tile twice from L2
  if (tile == 5 && Nw % 256 == 0) return run<kEpiPartial, 160, 256, 64, 3, 2, 4>(ctx, s, A, W, nullptr, nullptr, M, Nw, K, RopeArgs{}, sk, splits);
  if (tile == 3) return run<kEpiPartial, 128, 128, 64, 5, 4, 2>(ctx, s, A, W, nullptr, nullptr, M, Nw, K, RopeArgs{}, sk, splits);
  if (tile == 7) return run<kEpiPartial, 64, 128, 64, 3, 2, 2>(ctx, s, A, W, nullptr, nullptr, M, Nw, K, RopeArgs{}, sk, splits);
  if (tile == 8) return run<kEpiPartial, 192, 128, 64, 3, 2, 4>(ctx, s, A, W, nullptr, nullptr, M, Nw, K, RopeArgs{}, sk, splits);
  return run<kEpiPartial, 320, 128, 64, 2, 4, 2>(ctx, s, A, W, nullptr, nullptr, M, Nw, K, RopeArgs{}, sk, splits);
}

pvf_status launch_splitk_finalize(pvf_ctx *ctx, hipStream_t s, GemmEpilogue epi, const float *partial, int splits,
                                  int M, int N, void *C, const void *residual) {
  const int Nw = epi == kEpiSwiglu ? 2 * N : N;
  const int blocks = (int)(((int64_t)M * (N / 8) + 255) / 256);
  if (blocks == 0) return PVF_OK;
  if (epi == kEpiSwiglu) splitk_finalize_kernel<kEpiSwiglu><<<blocks, 256, 0, s>>>(partial, splits, M, Nw, N, (bf16_t *)C, nullptr);
  else if (epi == kEpiResidual) splitk_finalize_kernel<kEpiResidual><<<blocks, 256, 0, s>>>(partial, splits, M, Nw, N, (bf16_t *)C, (const bf16_t *)residual);
  else splitk_finalize_kernel<kEpiStore><<<blocks, 256, 0, s>>>(partial, splits, M, Nw, N, (bf16_t *)C, nullptr);
  PVF_LAUNCH_CHECK(ctx, "splitk_finalize");
  return PVF_OK;
}

pvf_status launch_gemm_mfma_splitk(pvf_ctx *ctx, hipStream_t s, GemmEpilogue epi, const void *A, const void *W,
                                   void *C, const void *residual, int M, int N, int K, float *ws, size_t ws_floats) {
  const uintptr_t al = (uintptr_t)C | (uintptr_t)residual;
  PVF_REQUIRE(ctx, (al & 15u) == 0, PVF_EINVAL, "gemm_mfma: operands must be 16-byte aligned");
  int splits = 0;
  pvf_status st = launch_gemm_mfma_splitk_partial(ctx, s, A, W, M, epi == kEpiSwiglu ? 2 * N : N, K, ws, ws_floats, &splits);
  if (st != PVF_OK) return st;
  return launch_splitk_finalize(ctx, s, epi, ws, splits, M, N, C, residual);
}


// QKV projection with the rotary embedding and the key-contiguous copy of v fused into the
// epilogue (see RopeArgs).  qkv [M, 3*H*128], vt [M/T, H, 128, T], cos_sin [T, 64].
bool gemm_mfma_qkv_rope_supported(int dtype, int M, int N, int K, int T, int H) {
  if (!gemm_mfma_supported(dtype, kEpiStore, M, N, K)) return false;
  if (N != 3 * H * 128 || H % 2 != 0 || T % 32 != 0 || M % T != 0) return false;
  return pick_config(kEpiQkvRope, M, N, K) >= 0;
}

pvf_status launch_gemm_mfma_qkv_rope(pvf_ctx *ctx, hipStream_t s, const void *A, const void *W, void *qkv,
                                     void *vt, const float2 *cos_sin, int M, int N, int K, int T, int H, bool store_v,
                                     const NormArgs *na) {
  const uintptr_t al = (uintptr_t)A | (uintptr_t)W | (uintptr_t)qkv | (uintptr_t)vt;
  PVF_REQUIRE(ctx, (al & 15u) == 0, PVF_EINVAL, "gemm_mfma: operands must be 16-byte aligned");
  const int cfg = pick_config(kEpiQkvRope, M, N, K);
  PVF_REQUIRE(ctx, cfg >= 0, PVF_ESHAPE, "gemm_mfma: no tile shape with a rotary epilogue for N=%d", N);
  RopeArgs ra;
  ra.cos_sin = cos_sin; ra.vt = (bf16_t *)vt; ra.T = T; ra.H = H; ra.store_v = store_v;
  PVF_REQUIRE(ctx, !na || !na->ss_in || gemm_mfma_norm_capable(cfg), PVF_ESHAPE, "gemm_mfma: tile shape %d cannot fold the norm", cfg);
  return run_cfg<kEpiQkvRope>(ctx, s, cfg, A, W, qkv, nullptr, M, N, K, ra, na ? *na : NormArgs{});
}

bool gemm_mfma_supported(int dtype, GemmEpilogue epi, int M, int N, int K) {
  if (dtype != PVF_BF16 || M < 1 || K < 64 || K % 64 != 0) return false;
  const int64_t w_rows = (epi == kEpiSwiglu) ? 2 * (int64_t)N : N;
  if ((int64_t)M * K * 2 >= (1ll << 32) || w_rows * K * 2 >= (1ll << 32)) return false;   // 32-bit lane offsets
  return N % (epi == kEpiSwiglu ? 64 : 128) == 0;
}

// Tile shapes with room for the folded-norm exchange (every 8-wave shape).
bool gemm_mfma_norm_capable(int cfg) { return cfg >= 0 && cfg != 6 && cfg != 7; }

// Output tile columns (= slots of row sums of squares a kEpiResidual launch writes); 0: no folded norm for this launch.
int gemm_mfma_norm_slots(GemmEpilogue epi, int M, int N, int K) {
  if (!gemm_mfma_supported(PVF_BF16, epi, M, N, K)) return 0;
  const int cfg = pick_config(epi, M, N, K);
  if (!gemm_mfma_norm_capable(cfg)) return 0;
  const int c = cfg == 3 || cfg >= kNumCfg ? 3 : cfg;
  return N / (epi == kEpiSwiglu ? kCfg[c].bn / 2 : kCfg[c].bn);
}

pvf_status launch_gemm_mfma(pvf_ctx *ctx, hipStream_t s, GemmEpilogue epi, const void *A,
                            const void *W, void *C, const void *residual, int M, int N, int K, const NormArgs *na) {
  const uintptr_t al = (uintptr_t)A | (uintptr_t)W | (uintptr_t)C | (uintptr_t)residual;
  PVF_REQUIRE(ctx, (al & 15u) == 0, PVF_EINVAL, "gemm_mfma: operands must be 16-byte aligned");
  const int cfg = pick_config(epi, M, N, K);
  PVF_REQUIRE(ctx, cfg >= 0, PVF_ESHAPE, "gemm_mfma: no tile shape for N=%d", N);
  const NormArgs nrm = na ? *na : NormArgs{};
  PVF_REQUIRE(ctx, !(nrm.ss_in || nrm.ss_out) || gemm_mfma_norm_capable(cfg), PVF_ESHAPE, "gemm_mfma: tile shape %d cannot fold the norm", cfg);
  switch (epi) {
    case kEpiStore: return run_cfg<kEpiStore>(ctx, s, cfg, A, W, C, residual, M, N, K);
    case kEpiResidual: return run_cfg<kEpiResidual>(ctx, s, cfg, A, W, C, residual, M, N, K, RopeArgs{}, nrm);
    case kEpiSwiglu: return run_cfg<kEpiSwiglu>(ctx, s, cfg, A, W, C, residual, M, N, K, RopeArgs{}, nrm);
    case kEpiQkvRope: break;                     // has its own entry (launch_gemm_mfma_qkv_rope)
    case kEpiPartial: break;                     // launch_gemm_mfma_splitk
  }
  return PVF_EINVAL;
}

}  // namespace pvf
