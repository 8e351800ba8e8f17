// Stage 2 of the decision epilogue and the small state kernels around it.
//
// One workgroup per canvas group takes the stage-1 summaries (top-1 token and probability of
// every window row of the backbone and of each live draft) and performs, in the paper's order:
//   verify   impact set (Eq. impact_set), verified compatibility A_j (Eq. at), Filter 2 by
//            C_total (Sec. 4.2), or the AR acceptance set and its longest member (Sec. 4.3);
//   commit   y <- winner branch; the active block advances to the first block with a mask
//            (App. A.1);
//   propose  working set B_t (active block, plus the next block once at most N_s masks are
//            left: Eq. block_expansion), confidence-threshold commit (Sec. 2) with the
//            single-best fallback, planning candidates + Top-K (Sec. 4.1) or AR candidates
//            (Sec. 4.3), and the next batch of canvases (Eq. plan_branch / AR branches).
// Everything is integer / compare work on at most (1+K) * R summaries; C_total is summed in
// float64, which is exact for these inputs and therefore independent of the order.
//
// Calibration trajectory (App. A.2; routes == PVF_ROUTES_CAL): the same machinery with two
// changes.  propose: the drafts are the non-base masks whose confidence lies in the calibration
// band, whatever their token, the K most confident first.  verify: each draft is only measured
// -- A_j as above and Delta H_j, the mean entropy drop over the masked positions of the working
// set other than the draft's own (Sec. 3) -- and added to the token statistics n_v, m_v, sum A,
// sum A * Delta H of its token v; nothing but the base branch is ever committed.
#include "common.h"

namespace pvf {
namespace {

struct Stage2Args {
  pvf_state st;
  pvf_decode_cfg cfg;
  const uint32_t *plan_bitmap;
  int32_t vocab, mask_id, R, T, n_blocks;
};

constexpr int kStage2Threads = 256;

// SplitMix64 step (Steele, Lea, Flood 2014): the counter-based generator of the ablation decoders
__device__ __forceinline__ uint64_t splitmix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
constexpr int kMaxWinBlocks = 4;

// Dynamic LDS layout: conf[(1+K)*R] | tok[(1+K)*R] | x[R] | flag[2*block_len]
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
  __shared__ int32_t s_cnt[4];     // 0: impact size, 1: base commits, 2: candidates, 3: masks in the proposing set
  __shared__ int32_t s_blk[kMaxWinBlocks];   // masks per window block after the commit
  __shared__ int32_t s_winner, s_knew, s_done, s_wsnew;

  uint8_t *accept = a.st.accept + (int64_t)g * K;
  int32_t *ncommit = a.st.n_commit + (int64_t)g * 3;
  const int ka = a.st.k_active[g];
  if (a.st.done[g] || ka < 0 || ka >= a.n_blocks) {   // finished (or invalid) group: report an empty round
    for (int j = tid; j < K; j += nth) accept[j] = 0;
    if (tid == 0) {
      a.st.winner[g] = 0; ncommit[0] = ncommit[1] = ncommit[2] = 0; a.st.n_drafts[g] = 0; a.st.done[g] = 1;
    }
    return;
  }

  int Kt = a.st.n_drafts[g];
  Kt = Kt < 0 ? 0 : (Kt > K ? K : Kt);
  const int route = Kt ? a.st.draft_route[g] : PVF_ROUTE_NONE;
  // working set this batch was formed on: 1 block, or 2 with early cross-block revelation
  int ws = (a.cfg.n_sparse > 0 && a.st.n_ws_blocks[g] == 2 && ka + 1 < a.n_blocks) ? 2 : 1;
  const int wlen = ws * bl;
  const int w0 = a.cfg.prompt_len + ka * bl;
  const int nwb = min(R / bl, a.n_blocks - ka);          // window blocks that exist
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
      if (fp < 0 || fp >= wlen) fp = -1;                 // a fill outside the working set voids its draft
    }
    s_fpos[tid] = fp; s_ftok[tid] = ft; s_ok[tid] = 0;
  }
  if (tid < 4) s_cnt[tid] = 0;
  if (tid < kMaxWinBlocks) s_blk[tid] = 0;
  __syncthreads();

  // ---------------- verify ----------------
  if (route == PVF_ROUTE_PLAN) {
    // impact set: masked in the base branch and confident under the base branch
    for (int i = tid; i < wlen; i += nth) {
      const int imp = (s_x[i] == MASK) && (s_conf[i] >= a.cfg.tau_high);
      s_flag[i] = imp;
      if (imp) atomicAdd(&s_cnt[0], 1);
    }
    __syncthreads();
    if (tid >= 1 && tid <= Kt) {          // one thread per draft
      const int j = tid, fp = s_fpos[j - 1];
      bool ok = (s_cnt[0] > 0) && (fp >= 0);
      double C = 0.0;
      for (int i = 0; i < wlen; ++i) {
        if (s_flag[i] && s_tok[j * R + i] != s_tok[i]) ok = false;
        if (s_x[i] == MASK && i != fp) C += (double)s_conf[j * R + i];
      }
      s_ok[j - 1] = ok;
      s_C[j - 1] = C;
    }
  } else if (route == PVF_ROUTE_CAL) {
    for (int i = tid; i < wlen; i += nth) {
      const int imp = (s_x[i] == MASK) && (s_conf[i] >= a.cfg.tau_high);
      s_flag[i] = imp;
      if (imp) atomicAdd(&s_cnt[0], 1);
    }
    __syncthreads();
    if (tid >= 1 && tid <= Kt) {          // one thread per measured draft
      const int j = tid, fp = s_fpos[j - 1], v = s_ftok[j - 1];
      bool ok = (s_cnt[0] > 0) && (fp >= 0);
      const float *ent0 = a.st.ent + (int64_t)g * slots * R, *entj = ent0 + (int64_t)j * R;
      double sum = 0.0;
      int cnt = 0;
      for (int i = 0; i < wlen; ++i) {
        if (s_flag[i] && s_tok[j * R + i] != s_tok[i]) ok = false;
        if (s_x[i] == MASK && i != fp) { sum += (double)ent0[i] - (double)entj[i]; ++cnt; }
      }
      const double dH = cnt ? sum / cnt : 0.0;
      s_ok[j - 1] = ok;
      a.st.dh[(int64_t)g * K + j - 1] = dH;
      if (fp >= 0 && v >= 0 && v < a.vocab) {
        atomicAdd(&a.st.cal_n[v], 1u);
        if (s_cnt[0] > 0) atomicAdd(&a.st.cal_m[v], 1u);
        if (ok) { atomicAdd(&a.st.cal_a[v], 1u); atomicAdd(&a.st.cal_vig[v], dH); }
      }
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
  for (int r = tid; r < nwb * bl; r += nth) if (s_x[r] == MASK) atomicAdd(&s_blk[r / bl], 1);
  __syncthreads();
  // blocks past the window have never been in a working set: they are fully masked
  const int masks_beyond = max(0, a.n_blocks - ka - nwb) * bl;
  if (tid == 0) {
    int kn = -1;
    for (int b = 0; b < nwb && kn < 0; ++b) if (s_blk[b] > 0) kn = ka + b;
    int dn = 0, wsn = 1;
    if (kn < 0) { if (masks_beyond > 0) kn = ka + nwb; else { kn = ka; dn = 1; } }
    if (!dn && a.cfg.n_sparse > 0 && kn + 1 < a.n_blocks && kn - ka < nwb && s_blk[kn - ka] <= a.cfg.n_sparse) wsn = 2;
    s_knew = kn; s_done = dn; s_wsnew = wsn;
  }
  __syncthreads();
  const int winner = s_winner, k_new = s_knew, ws_new = s_wsnew;
  const int off = (k_new - ka) * bl;             // window row of the (possibly new) active block
  const int plen = ws_new * bl;                  // length of the proposing working set
  int K_next = 0, route_next = PVF_ROUTE_NONE;
  const bool in_window = off + plen <= R;        // always true for states this library produced

  if (!s_done && in_window) {
    // ---------------- propose from the winner's own predictions ----------------
    const float *cw = s_conf + winner * R + off;
    const int32_t *tw = s_tok + winner * R + off;
    int32_t *xb = s_x + off;
    // flag: 0 known, 1 masked (stays), 2 masked and committed by the threshold
    for (int i = tid; i < plen; i += nth) {
      int f = 0;
      if (xb[i] == MASK) {
        f = (cw[i] >= a.cfg.tau_high) ? 2 : 1;
        atomicAdd(&s_cnt[3], 1);
        if (f == 2) atomicAdd(&s_cnt[1], 1);
      }
      s_flag[i] = f;
    }
    __syncthreads();
    if (tid == 0 && s_cnt[1] == 0) {             // progress rule: the single most confident mask
      int best = -1;
      for (int i = 0; i < plen; ++i)
        if (s_flag[i] == 1 && (best < 0 || cw[i] > cw[best])) best = i;
      if (best >= 0) { s_flag[best] = 2; s_cnt[1] = 1; }
    }
    __syncthreads();
    for (int i = tid; i < plen; i += nth) if (s_flag[i] == 2) xb[i] = tw[i];
    if (tid == 0) {
      ncommit[0] = s_cnt[1];
      int total = masks_beyond;                  // masked positions of the whole canvas before this step's commits
      for (int b = 0; b < nwb; ++b) total += s_blk[b];
      int extra = 0;
      if (a.cfg.routes & (PVF_ROUTES_XRANDOM | PVF_ROUTES_XPLANNING)) {
        // Ablation decoders (App. A.3.1): one more commit among the remaining masks whose
        // confidence lies in the closed bin; planning tokens first if asked for.
        int n_el = 0, n_pl = 0;
        for (int i = 0; i < plen; ++i) {
          if (s_flag[i] != 1 || !(cw[i] >= a.cfg.tau_plan_lo && cw[i] <= a.cfg.tau_plan_hi)) continue;
          ++n_el;
          const int t = tw[i];
          if (t >= 0 && t < a.vocab && ((a.plan_bitmap[t >> 5] >> (t & 31)) & 1u)) ++n_pl;
        }
        const bool use_plan = (a.cfg.routes & PVF_ROUTES_XPLANNING) && n_pl > 0;
        const int n_pool = use_plan ? n_pl : n_el;
        if (n_pool > 0) {
          const uint64_t key = ((uint64_t)a.cfg.seed << 32) + ((uint64_t)(g & 0xFFF) << 20) + (uint64_t)(total & 0xFFFFF);
          int pick = (int)(splitmix64(key) % (uint64_t)n_pool);
          for (int i = 0; i < plen; ++i) {
            if (s_flag[i] != 1 || !(cw[i] >= a.cfg.tau_plan_lo && cw[i] <= a.cfg.tau_plan_hi)) continue;
            const int t = tw[i];
            if (use_plan && !(t >= 0 && t < a.vocab && ((a.plan_bitmap[t >> 5] >> (t & 31)) & 1u))) continue;
            if (pick-- == 0) { s_flag[i] = 2; xb[i] = t; extra = 1; break; }
          }
        }
        ncommit[1] = extra;                      // reported in the planning slot of n_commit
      }
      s_cnt[1] += extra;
      if (total - s_cnt[1] == 0) s_done = 1;     // nothing left anywhere: no further forward
    }
    __syncthreads();
    const int n_left = s_cnt[3] - s_cnt[1];      // masks left in the proposing set

    if (!s_done && K > 0 && n_left > 0) {
      // planning candidates: non-base masks whose top-1 is a planning token, confidence in the band
      int32_t *s_cand = s_flag;                  // reuse: 3 = planning candidate, 4 = AR candidate
      if (a.cfg.routes & PVF_ROUTES_PLAN) {
        for (int i = tid; i < plen; i += nth) {
          if (s_flag[i] == 1) {
            const int t = tw[i];
            const bool in_plan = t >= 0 && t < a.vocab && ((a.plan_bitmap[t >> 5] >> (t & 31)) & 1u);
            if (in_plan && cw[i] >= a.cfg.tau_plan_lo && cw[i] < a.cfg.tau_plan_hi) {
              s_cand[i] = 3; atomicAdd(&s_cnt[2], 1);
            }
          }
        }
        __syncthreads();
        if (s_cnt[2] > 0) {
          route_next = PVF_ROUTE_PLAN;
          K_next = min(K, s_cnt[2]);
          for (int i = tid; i < plen; i += nth) {  // rank by (-confidence, position)
            if (s_cand[i] != 3) continue;
            int rank = 0;
            for (int i2 = 0; i2 < plen; ++i2)
              if (s_cand[i2] == 3 && (cw[i2] > cw[i] || (cw[i2] == cw[i] && i2 < i))) ++rank;
            if (rank < K) { s_npos[rank] = w0 + off + i; s_ntok[rank] = tw[i]; }
          }
        }
      }
      if (a.cfg.routes & PVF_ROUTES_CAL) {
        for (int i = tid; i < plen; i += nth)
          if (s_flag[i] == 1 && cw[i] >= a.cfg.tau_plan_lo && cw[i] < a.cfg.tau_plan_hi) {
            s_cand[i] = 3; atomicAdd(&s_cnt[2], 1);
          }
        __syncthreads();
        if (s_cnt[2] > 0) {
          route_next = PVF_ROUTE_CAL;
          K_next = min(K, s_cnt[2]);
          for (int i = tid; i < plen; i += nth) {  // rank by (-confidence, position)
            if (s_cand[i] != 3) continue;
            int rank = 0;
            for (int i2 = 0; i2 < plen; ++i2)
              if (s_cand[i2] == 3 && (cw[i2] > cw[i] || (cw[i2] == cw[i] && i2 < i))) ++rank;
            if (rank < K) { s_npos[rank] = w0 + off + i; s_ntok[rank] = tw[i]; }
          }
        }
      }
      if (route_next == PVF_ROUTE_NONE && (a.cfg.routes & PVF_ROUTES_AR)) {
        for (int i = tid; i < plen; i += nth)
          if (s_flag[i] == 1 && cw[i] >= a.cfg.tau_ar_lo) { s_cand[i] = 4; atomicAdd(&s_cnt[2], 1); }
        __syncthreads();
        if (s_cnt[2] > 0) {
          route_next = PVF_ROUTE_AR;
          K_next = min(K, s_cnt[2]);
          for (int i = tid; i < plen; i += nth) {  // leftmost first
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
      if (route_next != PVF_ROUTE_AR) { if (s_npos[j - 1] == pos) v = s_ntok[j - 1]; }
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
    a.st.n_ws_blocks[g] = ws_new;
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
    st.n_ws_blocks[g] = 1;
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
    row_pos[idx] = (pos >= 0 && pos < T) ? pos : -1;
  }
}

__global__ void copy_out_kernel(int K, int T, const int32_t *__restrict__ canvas,
                                int32_t *__restrict__ out) {
  const int g = blockIdx.x;
  for (int t = threadIdx.x; t < T; t += blockDim.x)
    out[(int64_t)g * T + t] = canvas[(int64_t)g * (1 + K) * T + t];
}

}  // namespace

int window_rows(const pvf_decode_cfg &c) {
  const int blocks = c.n_sparse > 0 ? 4 : 2;
  return (blocks * c.block_len < c.gen_len) ? blocks * c.block_len : c.gen_len;
}

pvf_status launch_stage2(pvf_ctx *ctx, hipStream_t s, int G, int vocab, int mask_id,
                         const uint32_t *plan_bitmap, const pvf_decode_cfg &cfg,
                         const pvf_state &st) {
  Stage2Args a;
  a.st = st; a.cfg = cfg; a.plan_bitmap = plan_bitmap; a.vocab = vocab; a.mask_id = mask_id;
  a.T = cfg.prompt_len + cfg.gen_len;
  a.R = window_rows(cfg);
  a.n_blocks = cfg.gen_len / cfg.block_len;
  const size_t lds = (size_t)(1 + cfg.K) * a.R * 8 + (size_t)a.R * 4 + (size_t)cfg.block_len * 8;
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
  build_batch_kernel<<<1, 256, 0, s>>>(G, cfg.K, n_seq, window_rows(cfg), T, cfg.prompt_len,
                                       cfg.block_len, st, seq_slot, row_pos);
  PVF_LAUNCH_CHECK(ctx, "build_batch");
  return PVF_OK;
}

__global__ void pack_status_kernel(int G, pvf_state st, int32_t *__restrict__ out) {
  const int g = blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= G) return;
  out[5 * g + 0] = st.done[g];
  out[5 * g + 1] = st.n_drafts[g];
  out[5 * g + 2] = st.n_commit[3 * g + 0];
  out[5 * g + 3] = st.n_commit[3 * g + 1];
  out[5 * g + 4] = st.n_commit[3 * g + 2];
}

pvf_status launch_pack_status(pvf_ctx *ctx, hipStream_t s, int G, const pvf_state &st, int32_t *out) {
  pack_status_kernel<<<(G + 255) / 256, 256, 0, s>>>(G, st, out);
  PVF_LAUNCH_CHECK(ctx, "pack_status");
  return PVF_OK;
}

pvf_status launch_copy_out(pvf_ctx *ctx, hipStream_t s, int G, int K, int T,
                           const int32_t *canvas, int32_t *out_tokens) {
  copy_out_kernel<<<G, 256, 0, s>>>(K, T, canvas, out_tokens);
  PVF_LAUNCH_CHECK(ctx, "copy_out");
  return PVF_OK;
}

}  // namespace pvf
