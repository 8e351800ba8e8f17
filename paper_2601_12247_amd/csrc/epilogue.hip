// Decision epilogue of a PVF round.
//
// stage 1  one pass over every live logits row: top-1 token (lowest id on ties, the [MASK]
//          column excluded) and its softmax probability (Sec. 3, definitions of y-hat and p).
//          The row is streamed once from HBM with 16-byte loads; the softmax itself is never
//          written anywhere.
// stage 2  one workgroup per canvas group: impact set (Eq. impact_set), verified
//          compatibility (Eq. at), Filter 2 (C_total, Sec. 4.2), AR acceptance (Sec. 4.3),
//          commit, confidence-threshold commit of the winner's predictions (Sec. 2),
//          planning candidates + Top-K (Sec. 4.1) or AR candidates (Sec. 4.3), and the next
//          batch of canvases (Eq. plan_branch / AR branches).
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

// Where a logits row's summary goes and whether the row exists at all.
__device__ __forceinline__ bool row_target(const RowFilter &rf, int64_t row, int64_t *out_row) {
  *out_row = row;
  if (rf.n_drafts == nullptr) return true;
  const int s = (int)(row / rf.R), r = (int)(row % rf.R);
  const int slot = rf.seq_slot ? rf.seq_slot[s] : s;
  const int g = slot / rf.slots_per_group, j = slot % rf.slots_per_group;
  *out_row = (int64_t)slot * rf.R + r;
  if (rf.done[g] || j > rf.n_drafts[g]) return false;
  return rf.prompt_len + rf.k_active[g] * rf.block_len + r < rf.T;
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

// ------------------------------------------------------------------------------------
// stage 2
// ------------------------------------------------------------------------------------
struct Stage2Args {
  pvf_state st;
  pvf_decode_cfg cfg;
  const uint32_t *plan_bitmap;
  int32_t vocab, mask_id, R, T, n_blocks;
};

constexpr int kStage2Threads = 256;

// Dynamic LDS layout: conf[(1+K)*R] | tok[(1+K)*R] | x[R] | flag[block_len]
__global__ void __launch_bounds__(kStage2Threads) stage2_kernel(Stage2Args a) {
  extern __shared__ unsigned char smem[];
  const int tid = threadIdx.x, nth = kStage2Threads;
  const int g = blockIdx.x;
  const int K = a.cfg.K, bl = a.cfg.block_len, R = a.R, T = a.T, MASK = a.mask_id;
  const int slots = 1 + K;
  float *s_conf = reinterpret_cast<float *>(smem);
  int32_t *s_tok = reinterpret_cast<int32_t *>(s_conf + slots * R);
  int32_t *s_x = s_tok + slots * R;
  int32_t *s_flag = s_x + R;
  __shared__ int32_t s_fpos[PVF_MAX_K], s_ftok[PVF_MAX_K], s_ok[PVF_MAX_K];
  __shared__ int32_t s_npos[PVF_MAX_K], s_ntok[PVF_MAX_K];
  __shared__ double s_C[PVF_MAX_K];
  __shared__ int32_t s_cnt[5];     // 0: impact size, 1: masks left in old block, 2: base commits, 3: candidates, 4: masks in proposing block
  __shared__ int32_t s_winner, s_knew, s_done;

  uint8_t *accept = a.st.accept + (int64_t)g * K;
  int32_t *ncommit = a.st.n_commit + (int64_t)g * 3;
  const int ka_in = a.st.k_active[g];
  if (a.st.done[g] || ka_in < 0 || ka_in >= a.n_blocks) {   // finished (or invalid) group: report an empty round
    for (int j = tid; j < K; j += nth) accept[j] = 0;
    if (tid == 0) {
      a.st.winner[g] = 0; ncommit[0] = ncommit[1] = ncommit[2] = 0; a.st.n_drafts[g] = 0; a.st.done[g] = 1;
    }
    return;
  }

  int Kt = a.st.n_drafts[g];
  Kt = Kt < 0 ? 0 : (Kt > K ? K : Kt);
  const int route = Kt ? a.st.draft_route[g] : PVF_ROUTE_NONE;
  const int ka = ka_in;
  const int w0 = a.cfg.prompt_len + ka * bl;
  int32_t *canvas0 = a.st.canvas + (int64_t)g * slots * T;

  for (int i = tid; i < (1 + Kt) * R; i += nth) {
    s_conf[i] = a.st.conf[(int64_t)g * slots * R + i];
    s_tok[i] = a.st.tok[(int64_t)g * slots * R + i];
  }
  for (int r = tid; r < R; r += nth) s_x[r] = (w0 + r < T) ? canvas0[w0 + r] : -2;
  if (tid < PVF_MAX_K) {
    int fp = -1, ft = -1;
    if (tid < Kt) {
      fp = a.st.fill_pos[(int64_t)g * K + tid] - w0;     // window-relative
      ft = a.st.fill_tok[(int64_t)g * K + tid];
      if (fp < 0 || fp >= bl) fp = -1;                   // a fill outside the active block voids its draft
    }
    s_fpos[tid] = fp; s_ftok[tid] = ft; s_ok[tid] = 0;
  }
  if (tid < 5) s_cnt[tid] = 0;
  __syncthreads();

  // ---------------- verify ----------------
  if (route == PVF_ROUTE_PLAN) {
    // impact set: masked in the base branch and confident under the base branch
    for (int i = tid; i < bl; i += nth) {
      const int imp = (s_x[i] == MASK) && (s_conf[i] >= a.cfg.tau_high);
      s_flag[i] = imp;
      if (imp) atomicAdd(&s_cnt[0], 1);
    }
    __syncthreads();
    if (tid >= 1 && tid <= Kt) {          // one thread per draft
      const int j = tid, fp = s_fpos[j - 1];
      bool ok = (s_cnt[0] > 0) && (fp >= 0);
      double C = 0.0;
      for (int i = 0; i < bl; ++i) {
        if (s_flag[i] && s_tok[j * R + i] != s_tok[i]) ok = false;
        if (s_x[i] == MASK && i != fp) C += (double)s_conf[j * R + i];
      }
      s_ok[j - 1] = ok;
      s_C[j - 1] = C;
    }
  } else if (route == PVF_ROUTE_AR) {
    if (tid >= 1 && tid <= Kt) {
      const int k = tid;
      bool ok = true;
      for (int r = 0; r < k; ++r) {
        const int fp = s_fpos[r];
        if (fp < 0 || s_tok[k * R + fp] != s_ftok[r]) ok = false;
      }
      s_ok[k - 1] = ok;
    }
  }
  __syncthreads();
  if (tid == 0) {
    int w = 0;
    if (route == PVF_ROUTE_PLAN) {
      double best = 0.0;
      for (int j = 1; j <= Kt; ++j)
        if (s_ok[j - 1] && (w == 0 || s_C[j - 1] > best)) { w = j; best = s_C[j - 1]; }
    } else if (route == PVF_ROUTE_AR) {
      for (int k = 1; k <= Kt; ++k) if (s_ok[k - 1]) w = k;
    }
    s_winner = w;
    // ---------------- commit the winner into the window copy of the backbone ----------------
    int n_plan = 0, n_ar = 0;
    if (w) {
      if (route == PVF_ROUTE_PLAN) { s_x[s_fpos[w - 1]] = s_ftok[w - 1]; n_plan = 1; }
      else { for (int r = 0; r < w; ++r) s_x[s_fpos[r]] = s_ftok[r]; n_ar = w; }
    }
    ncommit[1] = n_plan; ncommit[2] = n_ar;
    a.st.winner[g] = w;
  }
  __syncthreads();
  for (int j = tid; j < K; j += nth) accept[j] = (j < Kt) ? (uint8_t)s_ok[j] : 0;

  // ---------------- active block after the commit ----------------
  for (int i = tid; i < bl; i += nth) if (s_x[i] == MASK) atomicAdd(&s_cnt[1], 1);
  __syncthreads();
  if (tid == 0) {
    int kn = ka, dn = 0;
    if (s_cnt[1] == 0) { kn = ka + 1; if (kn >= a.n_blocks) { kn = ka; dn = 1; } }
    s_knew = kn; s_done = dn;
  }
  __syncthreads();
  const int winner = s_winner, k_new = s_knew;
  const int off = (k_new - ka) * bl;             // window row of the (possibly new) active block
  int K_next = 0, route_next = PVF_ROUTE_NONE;

  if (!s_done) {
    // ---------------- propose from the winner's own predictions ----------------
    const float *cw = s_conf + winner * R + off;
    const int32_t *tw = s_tok + winner * R + off;
    int32_t *xb = s_x + off;
    // flag: 0 known, 1 masked (stays), 2 masked and committed by the threshold
    for (int i = tid; i < bl; i += nth) {
      int f = 0;
      if (xb[i] == MASK) {
        f = (cw[i] >= a.cfg.tau_high) ? 2 : 1;
        atomicAdd(&s_cnt[4], 1);
        if (f == 2) atomicAdd(&s_cnt[2], 1);
      }
      s_flag[i] = f;
    }
    __syncthreads();
    if (tid == 0 && s_cnt[2] == 0) {             // progress rule: the single most confident mask
      int best = -1;
      for (int i = 0; i < bl; ++i)
        if (s_flag[i] == 1 && (best < 0 || cw[i] > cw[best])) best = i;
      if (best >= 0) { s_flag[best] = 2; s_cnt[2] = 1; }
    }
    __syncthreads();
    for (int i = tid; i < bl; i += nth) if (s_flag[i] == 2) xb[i] = tw[i];
    const int n_left = s_cnt[4] - s_cnt[2];
    if (tid == 0) {
      ncommit[0] = s_cnt[2];
      if (n_left == 0 && k_new == a.n_blocks - 1) s_done = 1;
    }
    __syncthreads();

    if (!s_done && K > 0 && n_left > 0) {
      // planning candidates: non-base masks whose top-1 is a planning token, confidence in the band
      int32_t *s_cand = s_flag;                  // reuse: 3 = candidate
      if (a.cfg.routes & PVF_ROUTES_PLAN) {
        for (int i = tid; i < bl; i += nth) {
          if (s_flag[i] == 1) {
            const int t = tw[i];
            const bool in_plan = t >= 0 && t < a.vocab && ((a.plan_bitmap[t >> 5] >> (t & 31)) & 1u);
            if (in_plan && cw[i] >= a.cfg.tau_plan_lo && cw[i] < a.cfg.tau_plan_hi) {
              s_cand[i] = 3; atomicAdd(&s_cnt[3], 1);
            }
          }
        }
        __syncthreads();
        if (s_cnt[3] > 0) {
          route_next = PVF_ROUTE_PLAN;
          K_next = min(K, s_cnt[3]);
          for (int i = tid; i < bl; i += nth) {  // rank by (-confidence, position)
            if (s_cand[i] != 3) continue;
            int rank = 0;
            for (int i2 = 0; i2 < bl; ++i2)
              if (s_cand[i2] == 3 && (cw[i2] > cw[i] || (cw[i2] == cw[i] && i2 < i))) ++rank;
            if (rank < K) { s_npos[rank] = w0 + off + i; s_ntok[rank] = tw[i]; }
          }
        }
      }
      if (route_next == PVF_ROUTE_NONE && (a.cfg.routes & PVF_ROUTES_AR)) {
        for (int i = tid; i < bl; i += nth)
          if (s_flag[i] == 1 && cw[i] >= a.cfg.tau_ar_lo) { s_cand[i] = 4; atomicAdd(&s_cnt[3], 1); }
        __syncthreads();
        if (s_cnt[3] > 0) {
          route_next = PVF_ROUTE_AR;
          K_next = min(K, s_cnt[3]);
          for (int i = tid; i < bl; i += nth) {  // leftmost first
            if (s_cand[i] != 4) continue;
            int rank = 0;
            for (int i2 = 0; i2 < i; ++i2) if (s_cand[i2] == 4) ++rank;
            if (rank < K) { s_npos[rank] = w0 + off + i; s_ntok[rank] = tw[i]; }
          }
        }
      }
    }
  } else if (tid == 0) {
    ncommit[0] = 0;
  }
  __syncthreads();

  // ---------------- next batch of canvases: window positions of every slot ----------------
  for (int idx = tid; idx < slots * R; idx += nth) {
    const int j = idx / R, r = idx % R, pos = w0 + r;
    if (pos >= T) continue;
    int v = s_x[r];
    if (j >= 1 && j <= K_next) {
      if (route_next == PVF_ROUTE_PLAN) { if (s_npos[j - 1] == pos) v = s_ntok[j - 1]; }
      else { for (int q = 0; q < j; ++q) if (s_npos[q] == pos) v = s_ntok[q]; }
    }
    canvas0[(int64_t)j * T + pos] = v;
  }
  for (int j = tid; j < K; j += nth) {
    a.st.fill_pos[(int64_t)g * K + j] = (j < K_next) ? s_npos[j] : -1;
    a.st.fill_tok[(int64_t)g * K + j] = (j < K_next) ? s_ntok[j] : -1;
  }
  if (tid == 0) {
    a.st.n_drafts[g] = s_done ? 0 : K_next;
    a.st.draft_route[g] = s_done ? PVF_ROUTE_NONE : route_next;
    a.st.k_active[g] = k_new;
    a.st.done[g] = s_done;
  }
}

// ------------------------------------------------------------------------------------
// small state kernels
// ------------------------------------------------------------------------------------
__global__ void state_init_kernel(const int32_t *__restrict__ prompt, int G, int K, int prompt_len,
                                  int T, int mask_id, pvf_state st) {
  const int g = blockIdx.x;
  for (int idx = threadIdx.x; idx < (1 + K) * T; idx += blockDim.x) {
    const int t = idx % T;
    st.canvas[(int64_t)g * (1 + K) * T + idx] = (t < prompt_len) ? prompt[(int64_t)g * prompt_len + t] : mask_id;
  }
  for (int j = threadIdx.x; j < K; j += blockDim.x) {
    st.fill_pos[(int64_t)g * K + j] = -1; st.fill_tok[(int64_t)g * K + j] = -1; st.accept[(int64_t)g * K + j] = 0;
  }
  if (threadIdx.x == 0) {
    st.n_drafts[g] = 0; st.draft_route[g] = PVF_ROUTE_NONE; st.k_active[g] = 0; st.winner[g] = 0;
    st.n_commit[g * 3 + 0] = st.n_commit[g * 3 + 1] = st.n_commit[g * 3 + 2] = 0;
    st.done[g] = (T == prompt_len);
  }
}

// One block.  Lists the live slots (group-major, slot-minor) and the window positions of each.
__global__ void build_batch_kernel(int G, int K, int n_seq, int R, int T, int prompt_len, int bl,
                                   pvf_state st, int32_t *__restrict__ seq_slot,
                                   int32_t *__restrict__ row_pos) {
  if (threadIdx.x == 0) {
    int n = 0;
    for (int g = 0; g < G; ++g) {
      if (st.done[g]) continue;
      int kt = st.n_drafts[g]; kt = kt < 0 ? 0 : (kt > K ? K : kt);
      for (int j = 0; j <= kt && n < n_seq; ++j) seq_slot[n++] = g * (1 + K) + j;
    }
    const int first = n ? seq_slot[0] : 0;
    while (n < n_seq) seq_slot[n++] = first;       // padding: repeats a live canvas
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < n_seq * R; idx += blockDim.x) {
    const int s = idx / R, r = idx % R;
    const int g = seq_slot[s] / (1 + K);
    const int pos = prompt_len + st.k_active[g] * bl + r;
    row_pos[idx] = pos < T ? pos : -1;
  }
}

__global__ void copy_out_kernel(int K, int T, const int32_t *__restrict__ canvas,
                                int32_t *__restrict__ out) {
  const int g = blockIdx.x;
  for (int t = threadIdx.x; t < T; t += blockDim.x)
    out[(int64_t)g * T + t] = canvas[(int64_t)g * (1 + K) * T + t];
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

pvf_status launch_stage2(pvf_ctx *ctx, hipStream_t s, int G, int vocab, int mask_id,
                         const uint32_t *plan_bitmap, const pvf_decode_cfg &cfg,
                         const pvf_state &st) {
  Stage2Args a;
  a.st = st; a.cfg = cfg; a.plan_bitmap = plan_bitmap; a.vocab = vocab; a.mask_id = mask_id;
  a.T = cfg.prompt_len + cfg.gen_len;
  a.R = (2 * cfg.block_len < cfg.gen_len) ? 2 * cfg.block_len : cfg.gen_len;
  a.n_blocks = cfg.gen_len / cfg.block_len;
  const size_t lds = (size_t)(1 + cfg.K) * a.R * 8 + (size_t)a.R * 4 + (size_t)cfg.block_len * 4;
  PVF_REQUIRE(ctx, lds <= 64 * 1024, PVF_ESHAPE, "stage2: (1+K)*R too large for LDS (%zu bytes)", lds);
  stage2_kernel<<<G, kStage2Threads, lds, s>>>(a);
  PVF_LAUNCH_CHECK(ctx, "stage2");
  return PVF_OK;
}

pvf_status launch_state_init(pvf_ctx *ctx, hipStream_t s, const int32_t *prompt, int G,
                             int mask_id, const pvf_decode_cfg &cfg, const pvf_state &st) {
  state_init_kernel<<<G, 256, 0, s>>>(prompt, G, cfg.K, cfg.prompt_len,
                                      cfg.prompt_len + cfg.gen_len, mask_id, st);
  PVF_LAUNCH_CHECK(ctx, "state_init");
  return PVF_OK;
}

pvf_status launch_build_batch(pvf_ctx *ctx, hipStream_t s, int G, int n_seq,
                              const pvf_decode_cfg &cfg, const pvf_state &st,
                              int32_t *seq_slot, int32_t *row_pos) {
  const int T = cfg.prompt_len + cfg.gen_len;
  const int R = (2 * cfg.block_len < cfg.gen_len) ? 2 * cfg.block_len : cfg.gen_len;
  build_batch_kernel<<<1, 256, 0, s>>>(G, cfg.K, n_seq, R, T, cfg.prompt_len, cfg.block_len, st,
                                       seq_slot, row_pos);
  PVF_LAUNCH_CHECK(ctx, "build_batch");
  return PVF_OK;
}

pvf_status launch_copy_out(pvf_ctx *ctx, hipStream_t s, int G, int K, int T,
                           const int32_t *canvas, int32_t *out_tokens) {
  copy_out_kernel<<<G, 256, 0, s>>>(K, T, canvas, out_tokens);
  PVF_LAUNCH_CHECK(ctx, "copy_out");
  return PVF_OK;
}

}  // namespace pvf
