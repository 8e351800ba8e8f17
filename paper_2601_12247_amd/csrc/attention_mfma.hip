// Non-causal attention on the CDNA4 matrix cores (bf16, d_head = 128): every query of a
// canvas attends to all T positions of the same canvas, masked or not -- the denoiser sees
// the whole canvas at once (Sec. 2).  Flash-style: K / V tiles of 64 keys are staged in LDS,
// the softmax is kept online in registers and the T x T score matrix is never materialised.
//
// Layout choices
//   * one workgroup = 128 queries of one (canvas, head); 4 waves x 32 queries;
//   * scores are computed transposed, S^T = K Q^T (MFMA "A" = K rows, "B" = Q rows), so a lane
//     owns ONE query (column lane%32) and 32 of the tile's 64 keys in registers: the softmax
//     max / sum are register loops plus one exchange with lane^32;
//   * O^T = V^T P^T: the probabilities a lane just produced are already the "B" operand of
//     the second product (the contraction index is permuted identically on both operands), and
//     every O^T accumulator of a lane belongs to that lane's query, so rescaling is lane-local;
//   * V is read key-contiguous, from a [canvas, head, d_head, T] copy written by the rotary
//     kernel; K and V^T tiles go global -> LDS directly, XOR-swizzled against bank conflicts,
//     double-buffered.
#include "common.h"

#include <type_traits>

namespace pvf {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(1))) const void gptr_t;
typedef __attribute__((address_space(3))) void lptr_t;

constexpr int DH = 128, TQ = 128, TK = 64;
constexpr int kKTile = TK * DH * 2;          // 16 KB, [key][d] rows of 256 B
constexpr int kVTile = DH * TK * 2;          // 16 KB, [d][key] rows of 128 B
constexpr int kStage = kKTile + kVTile;
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Window mode (K/V-cached rounds): the queries are the R window rows of a canvas (qkv holds only
// those rows, vt their key-contiguous values [seq][head][d][R]); a key inside the window
// [w0, w0 + n_valid) is read from there, every other key from the cache of the canvas' group
// (kc: rotated keys [T][d] row-major, vtc: values [head][d][T]).
struct WinArgs {
  const bf16_t *kc, *vtc;
  int64_t group_stride;
  const int32_t *seq_slot, *k_active;
  int32_t slots_per_group, prompt_len, block_len, R;
};

// SPLIT (window mode with at most 64 query rows per canvas): the 64 queries need only two of the four waves, and
// the loop over the key tiles is a chain of dependent steps of ~2 us each, so the waves work as two pairs: pair
// 0 takes the even key tiles, pair 1 the odd ones (two tiles are staged per step), and at the end pair 0 merges
// pair 1's running maximum, sum and O into its own.  Half as many steps for the same work.
template <bool WIN, bool SPLIT>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
attention_mfma_kernel(const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ vt,
                      bf16_t *__restrict__ out, int T, int H, WinArgs wa) {
  static_assert(!SPLIT || WIN, "the key split exists in window mode only");
  __shared__ __attribute__((aligned(1024))) unsigned char lds[(SPLIT ? 4 : 2) * kStage];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int pair = SPLIT ? wave >> 1 : 0;                    // which half of the key tiles this wave takes
  const int qwave = SPLIT ? wave & 1 : wave;                 // which 32 queries
  const int fr = lane & 31, fh = lane >> 5;
  const int q0 = blockIdx.x * TQ, head = blockIdx.y, seq = blockIdx.z;
  const int d = H * DH;
  const int TQrows = WIN ? wa.R : T;                       // query rows per canvas in qkv / out
  const int64_t row0 = (int64_t)seq * TQrows;
  const bf16_t *qb = qkv + row0 * 3 * d + (int64_t)head * DH;
  const bf16_t *kb = qb + d;
  const bf16_t *vtb = vt + ((int64_t)seq * H + head) * DH * TQrows;
  int w0 = 0, w1 = 0;                                      // window = keys [w0, w1)
  const bf16_t *kcb = nullptr, *vtcb = nullptr;
  if (WIN) {
    const int g = wa.seq_slot[seq] / wa.slots_per_group;
    w0 = wa.prompt_len + wa.k_active[g] * wa.block_len;
    w1 = w0 + min(wa.R, T - w0);
    kcb = wa.kc + g * wa.group_stride + (int64_t)head * DH;
    vtcb = wa.vtc + g * wa.group_stride + (int64_t)head * DH * T;
  }

  // ---- Q fragments: "B" operand, column = query, k-chunk = 8 consecutive d ----
  const int qrow = min(q0 + qwave * 32 + fr, TQrows - 1);
  bf16x8 qf[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks)
    qf[ks] = *reinterpret_cast<const bf16x8 *>(qb + (int64_t)qrow * 3 * d + ks * 16 + fh * 8);

  // ---- global -> LDS addressing (see file header) ----
  // K tile: slot s = i*256 + tid -> key s/16, position s%16, chunk = position ^ (key & 15)
  // V^T tile: slot s -> d-row s/8, position s%8, chunk = position ^ ((row >> 1) & 7)
  const bf16_t *k_src[4], *v_src[4];
  int k_key[4], k_col[4], v_row[4], v_key[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int s = i * 256 + tid;
    const int key = s >> 4, kc = (s & 15) ^ (key & 15);
    k_src[i] = kb + (int64_t)key * 3 * d + kc * 8;
    k_key[i] = key; k_col[i] = kc * 8;
    const int vr = s >> 3, vc = (s & 7) ^ ((vr >> 1) & 7);
    v_src[i] = vtb + (int64_t)vr * T + vc * 8;
    v_row[i] = vr; v_key[i] = vc * 8;
  }
  auto issue_loads = [&](int kt, int slot) {                 // key tile kt -> LDS tile slot `slot`
    unsigned char *dst = lds + slot * kStage + wave * 1024;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bf16_t *ks, *vs;
      if (WIN) {
        const int key = kt * TK + k_key[i];                // canvas position of this K row
        ks = (key >= w0 && key < w1) ? kb + (int64_t)(key - w0) * 3 * d + k_col[i]
                                     : kcb + (int64_t)key * d + k_col[i];
        const int vk = kt * TK + v_key[i];                 // first of the 8 keys of this V^T chunk
        vs = (vk >= w0 && vk < w1) ? vtb + (int64_t)v_row[i] * wa.R + (vk - w0)
                                   : vtcb + (int64_t)v_row[i] * T + vk;
      } else {
        ks = k_src[i] + (int64_t)kt * TK * 3 * d;
        vs = v_src[i] + kt * TK;
      }
      __builtin_amdgcn_global_load_lds((gptr_t *)ks, (lptr_t *)(dst + i * 4096), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((gptr_t *)vs, (lptr_t *)(dst + kKTile + i * 4096), 16, 0, 0);
    }
  };

  floatx16 o[4];                      // O^T: [d tile][..], column = this lane's query
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[t][e] = 0.f;
  float m_run = -INFINITY;
  floatx16 ol;                                               // ol[0] in lanes 0..31: running sum of P for query lane
#pragma unroll
  for (int e = 0; e < 16; ++e) ol[e] = 0.f;
  const floatx16 kZero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  bf16x8 ones;                                               // "A" operand with row 0 = 1, rows 1..31 = 0
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (bf16_t)(fr == 0 ? 1.0f : 0.0f);
  const float c = kLog2e / sqrtf((float)DH);

  // per-lane LDS offsets of the operand reads; the buffer, the key sub-tile and the d tile are
  // compile-time offsets on top (the loop below is unrolled over the two buffers)
  int k_rd[8], v_rd[4];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) k_rd[ks] = fr * 256 + (((ks * 2 + fh) ^ (fr & 15)) << 4);
#pragma unroll
  for (int ks2 = 0; ks2 < 4; ++ks2) v_rd[ks2] = fr * 128 + (((2 * ks2 + fh) ^ ((fr >> 1) & 7)) << 4);

  const int nk = T / TK;
  // step = one key tile (SPLIT: two, one per pair); kBuf = which half of the double buffer holds it
  const int n_steps = SPLIT ? (nk + 1) / 2 : nk;
  auto stage_step = [&](int st, int buf) {
    if (SPLIT) {
      issue_loads(2 * st, 2 * buf);
      if (2 * st + 1 < nk) issue_loads(2 * st + 1, 2 * buf + 1);
    } else {
      issue_loads(st, buf);
    }
  };
  stage_step(0, 0);
  auto tile = [&](int st, auto buf_c) {
    constexpr int kBuf = decltype(buf_c)::value;
    __builtin_amdgcn_s_waitcnt(0x0f70);          // vmcnt(0)
    __syncthreads();
    if (st + 1 < n_steps) stage_step(st + 1, kBuf ^ 1);
    if (SPLIT && 2 * st + pair >= nk) return;    // an odd number of key tiles: pair 1 has none in the last step
    const unsigned char *ks_ = lds + (SPLIT ? 2 * kBuf + pair : kBuf) * kStage;
    const unsigned char *vs_ = ks_ + kKTile;

    // ---- S^T = K Q^T : 2 key sub-tiles x 8 k-steps ----
    floatx16 s[2];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(ks_ + t * 32 * 256 + k_rd[ks]);   // key t*32 + fr
        // the first k-step starts from a constant zero accumulator: no registers to clear per tile
        s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], ks == 0 ? kZero16 : s[t], 0, 0, 0);
      }
    }
    // ---- online softmax for this lane's query ----
    float mx = s[0][0];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[t][e]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    // The running maximum moves only when the tile's maximum exceeds it by more than 8 in the exponent
    // (p then stays below 2^8, no overflow anywhere): the accumulators are rescaled in the first
    // tiles and almost never afterwards, instead of whenever one of the 32 queries sees a new maximum.
    const bool upd = (mx - m_run) * c > 8.0f;                // first tile: m_run = -inf
    const float m_new = upd ? mx : m_run;
    const float alpha = upd ? fast_exp2((m_run - m_new) * c) : 1.0f;   // first tile: exp2(-inf) = 0
    const float nmc = -m_new * c;
    bf16x8 pf[4];                                            // "B" operand of the 4 key k-steps
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int u = 0; u < 2; ++u)                            // k-step u of sub-tile t: register groups 2u, 2u+1
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          pf[2 * t + u][e] = (bf16_t)fast_exp2(fmaf(s[t][8 * u + e], c, nmc));
        }
    m_run = m_new;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[t][e] *= alpha;
      ol[0] *= alpha;
    }
    // ---- O^T += V^T P^T : 4 d tiles x 4 key k-steps.  k slot (fh, e) of k-step ks2 is key
    //      16*ks2 + 4*fh + e (e < 4) or 16*ks2 + 8 + 4*fh + (e - 4): the order P came out in ----
#pragma unroll
    for (int ks2 = 0; ks2 < 4; ++ks2) {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        // d row t*32 + fr; vt stores each group of 16 keys as {0-3, 8-11 | 4-7, 12-15}: chunk 2*ks2 + fh is this lane's 8 keys
        const bf16x8 vf = *reinterpret_cast<const bf16x8 *>(vs_ + t * 32 * 128 + v_rd[ks2]);
        o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[ks2], o[t], 0, 0, 0);
      }
      // row sums of P on the matrix pipe (a "V^T" row of ones): the vector ALU is the busier unit here
      ol = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, pf[ks2], ol, 0, 0, 0);
    }
  };
  for (int st = 0; st + 1 < n_steps; st += 2) {
    tile(st, std::integral_constant<int, 0>{});
    tile(st + 1, std::integral_constant<int, 1>{});
  }
  if (n_steps & 1) tile(n_steps - 1, std::integral_constant<int, 0>{});
  float l_run = __shfl(ol[0], fr, 64);                       // row 0 of that product: lane q % 32, register 0

  if (SPLIT) {
    // pair 1 hands (O, running maximum, running sum) of its key tiles to the wave of pair 0 with the same queries;
    // both are sums of 2^((s - m_pair) c) terms, so they meet after rescaling to the larger maximum
    __syncthreads();                                         // every wave is done with the tiles
    float *x = reinterpret_cast<float *>(lds) + qwave * 66 * 64 + lane;
    if (pair == 1) {
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) x[(t * 16 + e) * 64] = o[t][e];
      x[64 * 64] = m_run;
      x[65 * 64] = l_run;
    }
    __syncthreads();
    if (pair == 1) return;
    const float m1 = x[64 * 64], l1 = x[65 * 64];
    const float mm = fmaxf(m_run, m1);
    const float a0 = fast_exp2((m_run - mm) * c), a1 = fast_exp2((m1 - mm) * c);   // a pair without tiles: m = -inf, factor 0
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[t][e] = o[t][e] * a0 + x[(t * 16 + e) * 64] * a1;
    l_run = l_run * a0 + l1 * a1;
  }

  // ---- out[q][head*128 + d]: lane holds 4 consecutive d per accumulator group ----
  const int q = q0 + qwave * 32 + fr;
  if (q < TQrows) {
    const float inv = 1.0f / l_run;
    bf16_t *orow = out + (row0 + q) * d + (int64_t)head * DH;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        bf16x4 v;
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = (bf16_t)(o[t][4 * i + j] * inv);
        *reinterpret_cast<bf16x4 *>(orow + t * 32 + 8 * i + 4 * fh) = v;
      }
  }
}

// Position of key t inside a key-contiguous vt row: bits 2 and 3 of t are swapped, so that every
// group of 16 keys is stored as {0-3, 8-11 | 4-7, 12-15}.  The 8 keys that one lane of the
// attention kernel feeds into a k-step of the P V product (the order in which the S^T accumulators
// hold them) are then one 16-byte chunk.
__device__ __forceinline__ int vt_pos(int t) { return (t & ~12) | ((t & 4) << 1) | ((t & 8) >> 1); }

// Rotary embedding of q and k in place (pair (i, i + 64) of each head) and the key-contiguous copy of v for 64
// rows of one (canvas, head), by one 256-thread workgroup with 16-byte accesses throughout.
//   base: the rows' q columns of this head (row stride 3 d);  pos(rr): canvas position of row rr;
//   vb: vt row 0 of this (canvas, head) at the first of the 64 keys, vt_stride: keys per vt row.
//   vb[d][vt_pos(rr)] = v[rr][d]
template <typename PosFn>
__device__ __forceinline__ void rope_vt_64rows(bf16_t *base, int d, const float2 *__restrict__ cos_sin, PosFn pos,
                                               bf16_t *vb, int vt_stride, bf16_t (*tile)[64 + 2]) {
  const int tid = threadIdx.x;
  // rotate q and k: 64 rows x 2 tensors x 8 chunks of 8 pairs
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int idx = it * 256 + tid;
    const int ch = idx & 7, which = (idx >> 3) & 1, rr = idx >> 4;
    bf16_t *p = base + (int64_t)rr * 3 * d + which * d + ch * 8;
    const float4 *cs4 = reinterpret_cast<const float4 *>(cos_sin + (int64_t)pos(rr) * 64 + ch * 8);
    const uint4 lo = *reinterpret_cast<const uint4 *>(p), hi = *reinterpret_cast<const uint4 *>(p + 64);
    const uint32_t lw[4] = {lo.x, lo.y, lo.z, lo.w}, hw[4] = {hi.x, hi.y, hi.z, hi.w};
    uint32_t ol[4], oh[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float4 c4 = cs4[e];                              // (cos, sin) of pairs 2e, 2e + 1 of the chunk
      const float a0 = __uint_as_float(lw[e] << 16), a1 = __uint_as_float(lw[e] & 0xffff0000u);
      const float b0 = __uint_as_float(hw[e] << 16), b1 = __uint_as_float(hw[e] & 0xffff0000u);
      const bf16_t l0 = (bf16_t)(a0 * c4.x - b0 * c4.y), l1 = (bf16_t)(a1 * c4.z - b1 * c4.w);
      const bf16_t h0 = (bf16_t)(b0 * c4.x + a0 * c4.y), h1 = (bf16_t)(b1 * c4.z + a1 * c4.w);
      ol[e] = (uint32_t)__builtin_bit_cast(uint16_t, l0) | ((uint32_t)__builtin_bit_cast(uint16_t, l1) << 16);
      oh[e] = (uint32_t)__builtin_bit_cast(uint16_t, h0) | ((uint32_t)__builtin_bit_cast(uint16_t, h1) << 16);
    }
    *reinterpret_cast<uint4 *>(p) = make_uint4(ol[0], ol[1], ol[2], ol[3]);
    *reinterpret_cast<uint4 *>(p + 64) = make_uint4(oh[0], oh[1], oh[2], oh[3]);
  }
  // transpose v through LDS: a thread reads 8 d of one row, then writes the 8 keys of one 16-byte vt chunk
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int idx = it * 256 + tid;
    const int rr = idx & 63, ch = idx >> 6;                  // consecutive lanes = consecutive rows: no bank conflicts
    const uint4 v8 = *reinterpret_cast<const uint4 *>(base + (int64_t)rr * 3 * d + 2 * d + ch * 8);
    const uint32_t w[4] = {v8.x, v8.y, v8.z, v8.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      tile[ch * 8 + 2 * e][rr] = __builtin_bit_cast(bf16_t, (uint16_t)(w[e] & 0xffffu));
      tile[ch * 8 + 2 * e + 1][rr] = __builtin_bit_cast(bf16_t, (uint16_t)(w[e] >> 16));
    }
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int idx = it * 256 + tid;
    const int g = idx & 7, dd = idx >> 3;                    // chunk g of vt row dd: keys 16 (g / 2) + 4 (g % 2) + {0-3, 8-11}
    const int k0 = 16 * (g >> 1) + 4 * (g & 1);
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int kr = k0 + (e & 1) * 2 + (e >> 1) * 8;
      w[e] = (uint32_t)__builtin_bit_cast(uint16_t, tile[dd][kr]) | ((uint32_t)__builtin_bit_cast(uint16_t, tile[dd][kr + 1]) << 16);
    }
    *reinterpret_cast<uint4 *>(vb + (int64_t)dd * vt_stride + g * 8) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// Full canvases: one block = 64 positions of one (canvas, head); vt[canvas][head][d][vt_pos(t)] = v[canvas*T + t][head*128 + d].
__global__ void __launch_bounds__(256)
rope_vt_kernel(bf16_t *__restrict__ qkv, bf16_t *__restrict__ vt, int T, int H,
               const float2 *__restrict__ cos_sin) {
  __shared__ bf16_t tile[DH][64 + 2];
  const int t0 = blockIdx.x * 64, head = blockIdx.y, seq = blockIdx.z;
  const int d = H * DH;
  bf16_t *base = qkv + ((int64_t)seq * T + t0) * 3 * d + (int64_t)head * DH;
  rope_vt_64rows(base, d, cos_sin, [&](int rr) { return t0 + rr; },
                 vt + ((int64_t)seq * H + head) * DH * T + t0, T, tile);
}

// Window rows: rotary embedding at the rows' own canvas positions (row_pos, -1 = padding row,
// rotated like position T-1) and the key-contiguous copy vt[seq][head][d][r] of their values.
// One block = 64 window rows of one (sequence, head).
__global__ void __launch_bounds__(256)
rope_vt_rows_kernel(bf16_t *__restrict__ qkv, bf16_t *__restrict__ vt, const int32_t *__restrict__ row_pos,
                    int R, int T, int H, const float2 *__restrict__ cos_sin) {
  __shared__ bf16_t tile[DH][64 + 2];
  const int r0 = blockIdx.x * 64, head = blockIdx.y, seq = blockIdx.z;
  const int d = H * DH;
  bf16_t *base = qkv + ((int64_t)seq * R + r0) * 3 * d + (int64_t)head * DH;
  rope_vt_64rows(base, d, cos_sin,
                 [&](int rr) { const int pos = row_pos[(int64_t)seq * R + r0 + rr]; return pos < 0 ? T - 1 : pos; },
                 vt + ((int64_t)seq * H + head) * DH * R + r0, R, tile);
}

}  // namespace

// Window attention on the matrix cores needs whole 64-row blocks of window rows and 16-key
// groups (the unit of the vt key order) that lie entirely inside or outside the window.
bool attention_window_mfma_supported(int dtype, int T, int d_head, int R, int block_len, int prompt_len) {
  return dtype == PVF_BF16 && d_head == DH && T >= TK && T % TK == 0 && R % 64 == 0 && block_len % 16 == 0 &&
         prompt_len % 16 == 0;
}

pvf_status launch_rope_vt_rows(pvf_ctx *ctx, hipStream_t s, void *qkv, void *vt, const int32_t *row_pos,
                               int S, int R, int T, int n_heads, const float2 *cos_sin) {
  if (S == 0) return PVF_OK;
  const dim3 grid(R / 64, n_heads, S);
  rope_vt_rows_kernel<<<grid, 256, 0, s>>>((bf16_t *)qkv, (bf16_t *)vt, row_pos, R, T, n_heads, cos_sin);
  PVF_LAUNCH_CHECK(ctx, "rope_vt_rows");
  return PVF_OK;
}

pvf_status launch_attention_window_mfma(pvf_ctx *ctx, hipStream_t s, const void *qkv_w, const void *vt_w,
                                        const void *kc, const void *vtc, int64_t group_stride,
                                        const int32_t *seq_slot, const int32_t *k_active, int slots_per_group,
                                        int prompt_len, int block_len, int R, int S, int T, int n_heads,
                                        void *out) {
  if (S == 0) return PVF_OK;
  WinArgs wa;
  wa.kc = (const bf16_t *)kc; wa.vtc = (const bf16_t *)vtc; wa.group_stride = group_stride;
  wa.seq_slot = seq_slot; wa.k_active = k_active; wa.slots_per_group = slots_per_group;
  wa.prompt_len = prompt_len; wa.block_len = block_len; wa.R = R;
  const dim3 grid((R + TQ - 1) / TQ, n_heads, S);
  if (R <= 64)
    attention_mfma_kernel<true, true><<<grid, 256, 0, s>>>((const bf16_t *)qkv_w, (const bf16_t *)vt_w, (bf16_t *)out, T, n_heads, wa);
  else
    attention_mfma_kernel<true, false><<<grid, 256, 0, s>>>((const bf16_t *)qkv_w, (const bf16_t *)vt_w, (bf16_t *)out, T, n_heads, wa);
  PVF_LAUNCH_CHECK(ctx, "attention_window_mfma");
  return PVF_OK;
}

bool attention_mfma_supported(int dtype, int T, int d_head) {
  return dtype == PVF_BF16 && d_head == DH && T >= TK && T % TK == 0;
}

// qkv must already be rotated and vt filled (launch_rope_vt).
pvf_status launch_attention_mfma(pvf_ctx *ctx, hipStream_t s, const void *qkv, const void *vt,
                                 void *out, int S, int T, int n_heads) {
  if (S == 0) return PVF_OK;
  const dim3 grid((T + TQ - 1) / TQ, n_heads, S);
  attention_mfma_kernel<false, false><<<grid, 256, 0, s>>>((const bf16_t *)qkv, (const bf16_t *)vt, (bf16_t *)out, T, n_heads, WinArgs{});
  PVF_LAUNCH_CHECK(ctx, "attention_mfma");
  return PVF_OK;
}

pvf_status launch_rope_vt(pvf_ctx *ctx, hipStream_t s, void *qkv, void *vt, int S, int T,
                          int n_heads, const float2 *cos_sin) {
  if (S == 0) return PVF_OK;
  const dim3 grid(T / 64, n_heads, S);
  rope_vt_kernel<<<grid, 256, 0, s>>>((bf16_t *)qkv, (bf16_t *)vt, T, n_heads, cos_sin);
  PVF_LAUNCH_CHECK(ctx, "rope_vt");
  return PVF_OK;
}

}  // namespace pvf
