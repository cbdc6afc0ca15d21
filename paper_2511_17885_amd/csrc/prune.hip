// Routing-aware sliding-window pruning of visual tokens (paper Sec. 3.2): per-sequence visual
// ordinals, window similarity scores (Eq.8-10), attention term (Eq.11-13), budget, drop
// selection and compaction.
//
// The kept-token set is a decision, so every float here follows the same fixed-order fp32
// arithmetic as the router (compiled with contraction off): a dot product over the E routing
// probabilities is taken with one partial per lane (element e in lane e mod 64, ascending e,
// fmaf from +0) and the 6-level xor butterfly; means, cosines and the window average are plain
// sequential fp32 operations in window order; '/' and sqrtf are correctly rounded.
//
// Indexing trick: window i of sequence b lives at slot cu_seqlens[b] + i (a sequence has fewer
// windows than tokens), so no per-sequence window offsets have to be scanned; a slot finds its
// sequence by binary search over cu_seqlens.

#include "common.h"
#include "prune_dev.h"
#include "tiles.h"

namespace {

__device__ __forceinline__ float wave_sum_butterfly(float p) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) p = p + __shfl_xor(p, s, 64);
  return p;
}

// ---- A: visual ordinals.  One block per sequence.
// vis_ord[t] = number of visual tokens before t in its sequence (for visual t), -1 for text;
// vis_tok[cu[b] + j] = global index of the j-th visual token of sequence b; seq_nv[b] = N_v.
__global__ __launch_bounds__(256) void seq_ordinals_kernel(
    const uint8_t* __restrict__ is_visual, const int32_t* __restrict__ cu, int T,
    int32_t* __restrict__ vis_ord, int32_t* __restrict__ vis_tok, int32_t* __restrict__ seq_nv) {
  __shared__ int wave_tot[4];
  seq_ordinals_block(is_visual, cu, blockIdx.x, T, vis_ord, vis_tok, seq_nv, wave_tot);
}

// ---- B: window scores.  One wavefront per window; lanes <-> experts.
// win_s[g] = S_i (Eq.10 or Eq.8), win_a[g] = raw window attention sum (Eq.11) if attn, g = the window's slot.
// Launch over window units: sequence b owns the units cu[b]/W + b ... (it has at most
// floor(cu[b+1]/W) - floor(cu[b]/W) + 1 windows, so consecutive sequences never overlap and
// floor(T/W) + B units cover every window); a unit finds its sequence by binary search.
// STAGED: the wavefront copies the window's routing-probability rows into its own LDS tile once (coalesced
// row reads) and both passes over the window -- the mean row, then the cosines (Eq.9-10), or all pairs
// (Eq.8) -- read the tile; a lane only ever reads back the columns it stored itself, so no
// synchronisation is involved.  Windows whose rows do not fit the tile (W*E > WS_TILE) take the
// instantiation that re-reads global memory.  The arithmetic and its order are the same either way.
constexpr int WS_TILE = 2048;   // floats of LDS per wavefront
__device__ __forceinline__ int unit_base(const int32_t* cu, int b, int T, int W) {
  return clampi(cu[b], 0, T) / W + b;
}
template <bool STAGED>
__global__ __launch_bounds__(256) void window_score_kernel(
    const float* __restrict__ probs, const int32_t* __restrict__ cu, int B, int T, int E, int W,
    int sim_mode, const int32_t* __restrict__ vis_tok, const int32_t* __restrict__ seq_nv,
    const float* __restrict__ attn, float* __restrict__ win_s, float* __restrict__ win_a,
    int32_t* __restrict__ precede, int32_t* __restrict__ rank_c) {
  __shared__ float tile_all[STAGED ? 4 * WS_TILE : 1];
  const int lane = threadIdx.x & 63;
  // counters of the drop order (accumulated by select_kernel), cleared for every slot
  for (int g = blockIdx.x * 256 + threadIdx.x; g < T; g += gridDim.x * 256) {
    precede[g] = 0;
    if (rank_c != nullptr) rank_c[g] = 0;
  }
  const int u = blockIdx.x * 4 + (threadIdx.x >> 6);
  int lo = 0, hi = B - 1;   // largest b with unit_base(b) <= u
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (unit_base(cu, mid, T, W) <= u) lo = mid; else hi = mid - 1;
  }
  const int b = lo;
  int s, e;
  seq_range(cu, b, T, s, e);
  const int i = u - unit_base(cu, b, T, W);
  int nv = seq_nv[b];
  nv = nv < e - s ? nv : e - s;                 // a sequence has no more visual tokens than tokens
  if (i < 0 || (long long)i * W >= nv) return;  // not a window of this sequence
  const int g = s + i;                          // < s + nv <= T
  const int first = i * W;
  const int w = (nv - first < W) ? (nv - first) : W;
  const int32_t* toks = vis_tok + s + first;

  if (attn != nullptr) {
    float a = 0.0f;
    for (int j = 0; j < w; ++j) a = a + attn[toks[j]];
    if (lane == 0) win_a[g] = a;
  }
  if (w == 1) {
    if (lane == 0) win_s[g] = 1.0f;
    return;
  }
  float* tile = tile_all + (STAGED ? (threadIdx.x >> 6) * WS_TILE : 0);
  if (STAGED) {
    for (int j = 0; j < w; ++j) {
      const float* src = probs + (size_t)toks[j] * E;
      for (int ex = lane; ex < E; ex += 64) tile[j * E + ex] = src[ex];
    }
  }
  // element ex of the window's row j
  auto row = [&](int j, int ex) -> float {
    return STAGED ? tile[j * E + ex] : probs[(size_t)toks[j] * E + ex];
  };
  float S;
  if (sim_mode == 0) {
    // Eq.9: mean row (sequential over the window, one divide), Eq.10: mean cosine to it
    float mean[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int ex = lane + 64 * r;
      float acc = 0.0f;
      if (ex < E) {
        acc = row(0, ex);
        for (int j = 1; j < w; ++j) acc = acc + row(j, ex);
        acc = acc / (float)w;
      }
      mean[r] = acc;
    }
    float pm = 0.0f;
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (lane + 64 * r < E) pm = fmaf(mean[r], mean[r], pm);
    const float norm_mean = sqrtf(wave_sum_butterfly(pm));
    float acc = 0.0f;
    for (int j = 0; j < w; ++j) {
      float pd = 0.0f, pn = 0.0f;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int ex = lane + 64 * r;
        if (ex < E) {
          const float v = row(j, ex);
          pd = fmaf(v, mean[r], pd);
          pn = fmaf(v, v, pn);
        }
      }
      const float dot = wave_sum_butterfly(pd);
      const float nrm = sqrtf(wave_sum_butterfly(pn));
      const float c = dot / (nrm * norm_mean);
      acc = acc + c;
    }
    S = acc / (float)w;
  } else {
    // Eq.8: mean cosine over all pairs q < j
    float acc = 0.0f;
    for (int j = 1; j < w; ++j) {
      float rj[4];
      float pn = 0.0f;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int ex = lane + 64 * r;
        rj[r] = (ex < E) ? row(j, ex) : 0.0f;
        if (ex < E) pn = fmaf(rj[r], rj[r], pn);
      }
      const float nj = sqrtf(wave_sum_butterfly(pn));
      for (int q = 0; q < j; ++q) {
        float pd = 0.0f, pq = 0.0f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int ex = lane + 64 * r;
          if (ex < E) {
            const float v = row(q, ex);
            pd = fmaf(rj[r], v, pd);
            pq = fmaf(v, v, pq);
          }
        }
        const float dot = wave_sum_butterfly(pd);
        const float nq = sqrtf(wave_sum_butterfly(pq));
        const float c = dot / (nj * nq);
        acc = acc + c;
      }
    }
    S = acc / (float)(w * (w - 1) / 2);
  }
  if (lane == 0) win_s[g] = S;
}

// ---- C: drop order.  The drop order (normalised attention asc, score desc, index asc) is total, so
// "how many windows precede window i" fixes everything.  The count is an all-pairs comparison on
// integer sort keys, split two ways over the grid: blockIdx.x owns 256 window slots (i), blockIdx.y
// a run of 64 candidate windows (j) of the same sequence, staged through LDS; partial counts are
// added with integer atomics (order-free).  Bit 30 of the sum records that the sequence's last
// (possibly shorter) window precedes i.
constexpr int SEL_JC = 64;

__global__ __launch_bounds__(256) void select_kernel(
    const int32_t* __restrict__ cu, int B, int T, int W, float alpha,
    const int32_t* __restrict__ seq_nv, const float* __restrict__ win_s,
    const float* __restrict__ win_a, int32_t* __restrict__ precede, float* __restrict__ scores_out,
    int32_t* __restrict__ rank_c, const int32_t* __restrict__ only_merged) {
  // rank_c (window merging): also count the predecessors in the merge order (C desc, index asc).
  // only_merged (second pass of window merging): count only predecessors whose flag is set.
  __shared__ __align__(16) unsigned long long tileK[SEL_JC];   // (~key(C) << 32) | index: ascending = drop order
  __shared__ __align__(16) uint32_t tileA[SEL_JC];             // key(A)
  __shared__ float red[4];
  const int g0 = blockIdx.x * 256;
  const int g = g0 + threadIdx.x;
  const int g_last = (g0 + 255 < T - 1) ? g0 + 255 : T - 1;
  const int jbase = blockIdx.y * SEL_JC;
  const int b_first = find_seq(cu, B, g0), b_last = find_seq(cu, B, g_last);
  const bool has_attn = (win_a != nullptr);
  const float one_minus_alpha = 1.0f - alpha;
  for (int b = b_first; b <= b_last; ++b) {   // uniform over the block
    int s, e;
    seq_range(cu, b, T, s, e);
    const int nv = seq_nv[b];
    const int n = (nv + W - 1) / W;
    if (jbase >= n || s + n <= g0 || s > g_last) continue;
    // per-sequence attention maximum (Eq.12)
    float amax = 0.0f;
    if (has_attn) {
      float m = 0.0f;
      for (int j = threadIdx.x; j < n; j += 256) {
        const float a = win_a[s + j];
        m = (a > m) ? a : m;
      }
#pragma unroll
      for (int sh = 32; sh >= 1; sh >>= 1) {
        const float o = __shfl_xor(m, sh, 64);
        m = (o > m) ? o : m;
      }
      __syncthreads();
      if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
      __syncthreads();
      amax = red[0];
#pragma unroll
      for (int w = 1; w < 4; ++w) amax = (red[w] > amax) ? red[w] : amax;
    }
    auto score = [&](int j, float& Aj) -> float {   // Eq.13 (C = S exactly without attention)
      return redundancy_score(win_s[s + j], has_attn, has_attn ? win_a[s + j] : 0.0f, amax, alpha,
                              one_minus_alpha, Aj);
    };
    const int i = g - s;
    const bool mine = (g < T) && i >= 0 && i < n;
    unsigned long long Ki = 0ull;
    uint32_t Ai = 0u;
    if (mine) {
      float a;
      const float c = score(i, a);
      if (scores_out != nullptr && blockIdx.y == 0) scores_out[g] = c;
      Ki = ((unsigned long long)(~float_order_key(c)) << 32) | (uint32_t)i;
      Ai = float_order_key(a);
    }
    int count = 0, last_first = 0, count_c = 0;
    for (int j0 = jbase; j0 < n; j0 += (int)gridDim.y * SEL_JC) {   // uniform
      __syncthreads();
      if (threadIdx.x < SEL_JC) {
        const int jl = j0 + threadIdx.x;
        unsigned long long kj = ~0ull;   // sentinel: precedes nothing
        uint32_t aj = ~0u;
        if (jl < n && (only_merged == nullptr || only_merged[s + jl] != 0)) {
          float a;
          const float c = score(jl, a);
          kj = ((unsigned long long)(~float_order_key(c)) << 32) | (uint32_t)jl;
          aj = float_order_key(a);
        }
        tileK[threadIdx.x] = kj;
        tileA[threadIdx.x] = aj;
      }
      __syncthreads();
      if (mine) {
#pragma unroll
        for (int jj = 0; jj < SEL_JC; ++jj) {
          const unsigned long long K = tileK[jj];
          const uint32_t A = tileA[jj];
          const int first = (int)(A < Ai) | ((int)(A == Ai) & (int)(K < Ki));
          count += first;
          last_first |= first & (int)(j0 + jj == n - 1);
          count_c += (int)(K < Ki);
        }
      }
    }
    if (mine && (count | last_first)) atomicAdd(&precede[g], count + (last_first << 30));
    if (mine && rank_c != nullptr && count_c) atomicAdd(&rank_c[g], count_c);
  }
}

// ---- C2: window merging (Sec. 3.2.3, Eq.14-15): which windows merge.  One thread per window slot;
// the greedy walk is evaluated in closed form from the window's place in the merge order and the
// place of the sequence's last window (merge_plan).  Also clears the counter of the second counting
// pass.
__global__ __launch_bounds__(256) void merge_decide_kernel(
    const int32_t* __restrict__ cu, int B, int T, int W, float retention, float gamma,
    const int32_t* __restrict__ seq_nv, const int32_t* __restrict__ rank_c,
    int32_t* __restrict__ win_merged, int32_t* __restrict__ merged_before) {
  const int g = blockIdx.x * 256 + threadIdx.x;
  if (g >= T) return;
  merged_before[g] = 0;
  win_merged[g] = 0;
  const int b = find_seq(cu, B, g);
  int s, e;
  seq_range(cu, b, T, s, e);
  const int nv = seq_nv[b];
  const int n = (nv + W - 1) / W;
  const int i = g - s;
  if (i < 0 || i >= n) return;
  const int w_last = nv - (n - 1) * W;
  const bool short_last = w_last < W;
  const int L = short_last ? rank_c[s + n - 1] : n;
  const fmoe_merge_plan p = merge_plan(nv, W, retention, gamma, L);
  int m;
  if (short_last && i == n - 1) {
    m = p.last_m;
  } else {
    const int r = rank_c[g];
    const int k = r - ((short_last && L < r) ? 1 : 0);   // place among the full-size windows
    m = k < p.q_full ? 1 : 0;
  }
  win_merged[g] = m;
}

// ---- D: budget + compaction, in two launches over blocks of CP_BLOCK positions (a position is a token
// index, or T itself, which only carries the total).
//   compact_flag_kernel:  every position decides keep / drop on its own (text tokens and the leading tokens
//                         of each window stay) and stores (kept positions before it in its block) * 4 +
//                         merged * 2 + keep in keep_code; every block stores its number of kept tokens.
//   compact_write_kernel: a block's first output index is the sum of the counts of the blocks before it;
//                         kept tokens write their ascending index lists; new_cu[b] = kept tokens before
//                         cu[b], read off the same two arrays.
// The decision is a chain of dependent loads per token (its visual ordinal -> its sequence -> its
// window's counters), which is why it is spread over the chip instead of walked by one block.
constexpr int CP_BLOCK = 1024;

struct CompactArgs {
  const uint8_t* is_visual;
  const int32_t* cu;
  int B, T, W;
  float retention, gamma;
  const int32_t* vis_ord;
  const int32_t* seq_nv;
  const int32_t* precede;
  const int32_t* rank_c;          // gamma > 0
  const int32_t* win_merged;      // gamma > 0 with an attention term; nullptr: closed form (see below)
  const int32_t* merged_before;
  int32_t* keep_code;             // [T + 1]
  int32_t* blk_kept;              // [ceil((T + 1) / CP_BLOCK)]
  int32_t* kept_idx;
  int32_t* new_cu;
  uint8_t* is_visual_out;         // or nullptr
  uint8_t* is_merged_out;         // or nullptr
};

// largest b in [0,n) with clamp(cu[b]) <= g
__device__ __forceinline__ int find_seq_clamped(const int32_t* cu, int n, int T, int g) {
  int lo = 0, hi = n - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (clampi(cu[mid], 0, T) <= g) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// bit 0: token t survives, bit 1: it is the token a merged window collapses into.
// gamma > 0 (window merging): a merged window keeps exactly its first token; the others follow the
// drop rule with the merged windows taken out of the walk and the budget merging left.
// win_merged == nullptr (no attention term: drop order and merge order are the same order): which
// windows merge and how many merged windows precede a window follow in closed form from the
// window's place rank_c in that order and the place of the sequence's last window.
__device__ __forceinline__ int keep_decision(const CompactArgs& a, int t, int t_end) {
  // tokens past the last sequence have no ordinal and count as text
  const int ord = t < t_end ? a.vis_ord[t] : -1;
  if (ord < 0) return 1;
  const int T = a.T, W = a.W;
  const int b = find_seq_clamped(a.cu, a.B, T, t);
  const int s = clampi(a.cu[b], 0, T);
  const int nv = a.seq_nv[b];
  const int n = (nv + W - 1) / W;
  const int last = T - 1;
  int slot = s + ord / W;
  slot = slot < last ? slot : last;            // (always inside for the ordinals seq_ordinals writes)
  int slot_last = s + n - 1;
  slot_last = slot_last < 0 ? 0 : (slot_last < last ? slot_last : last);
  const int pc = a.precede[slot];
  const int in_win = ord % W;
  const bool merging = a.gamma > 0.0f;
  if (!merging) return in_win < window_keep_lead(ord, nv, W, a.retention, pc) ? 1 : 0;
  const bool closed = a.win_merged == nullptr;
  const int rl = a.rank_c[slot_last];
  const bool short_last = nv - (n - 1) * W < W;
  const int L = short_last ? rl : n;
  const fmoe_merge_plan p = merge_plan(nv, W, a.retention, a.gamma, L);
  int is_m, mb, last_m;
  if (closed) {
    const int r = a.rank_c[slot];                                  // place of this window
    const int k = r - ((short_last && L < r) ? 1 : 0);             // full-size windows ahead of it
    const bool is_last = short_last && (ord / W == n - 1);
    is_m = is_last ? p.last_m : (k < p.q_full ? 1 : 0);
    last_m = short_last ? p.last_m : (rl < p.q_full ? 1 : 0);
    mb = (k < p.q_full ? k : p.q_full) + ((short_last && p.last_m && L < r) ? 1 : 0);
  } else {
    is_m = a.win_merged[slot];
    mb = a.merged_before[slot];
    last_m = a.win_merged[slot_last];
  }
  if (is_m) return in_win == 0 ? 3 : 0;
  return in_win < window_keep_lead_merge(ord, nv, W, pc, mb, last_m != 0, p.u_rem) ? 1 : 0;
}

__global__ __launch_bounds__(CP_BLOCK) void compact_flag_kernel(CompactArgs a) {
  __shared__ int wave_tot[CP_BLOCK / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t = blockIdx.x * CP_BLOCK + threadIdx.x;
  const int t_end = clampi(a.cu[a.B], 0, a.T);
  const int bits = t < a.T ? keep_decision(a, t, t_end) : 0;
  const unsigned long long mask = __ballot(bits & 1);
  const int before = __popcll(mask & ((1ull << lane) - 1ull));
  if (lane == 0) wave_tot[wave] = __popcll(mask);
  __syncthreads();
  int wave_base = 0, total = 0;
#pragma unroll
  for (int w = 0; w < CP_BLOCK / 64; ++w) {
    if (w < wave) wave_base += wave_tot[w];
    total += wave_tot[w];
  }
  if (t <= a.T) a.keep_code[t] = ((wave_base + before) << 2) | bits;
  if (threadIdx.x == 0) a.blk_kept[blockIdx.x] = total;
}

__global__ __launch_bounds__(CP_BLOCK) void compact_write_kernel(CompactArgs a) {
  __shared__ int part[CP_BLOCK / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // kept tokens in the blocks before this one
  int sum = 0;
  for (int k = threadIdx.x; k < (int)blockIdx.x; k += CP_BLOCK) sum += a.blk_kept[k];
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d, 64);
  if (lane == 0) part[wave] = sum;
  __syncthreads();
  int first = 0;
#pragma unroll
  for (int w = 0; w < CP_BLOCK / 64; ++w) first += part[w];
  const int t = blockIdx.x * CP_BLOCK + threadIdx.x;
  if (t < a.T) {
    const int code = a.keep_code[t];
    const int pos = first + (code >> 2);
    if ((code & 1) && pos >= 0 && pos < a.T) {   // pos <= t by construction
      a.kept_idx[pos] = t;
      if (a.is_visual_out != nullptr) a.is_visual_out[pos] = a.is_visual[t];
      if (a.is_merged_out != nullptr) a.is_merged_out[pos] = (code >> 1) & 1;
    }
  }
  // sequence bounds of the kept tokens: kept tokens before cu[b]
  for (int b = blockIdx.x * CP_BLOCK + threadIdx.x; b <= a.B; b += gridDim.x * CP_BLOCK) {
    const int c = clampi(a.cu[b], 0, a.T);
    const int blk = c / CP_BLOCK;
    int before = 0;
    for (int k = 0; k < blk; ++k) before += a.blk_kept[k];
    a.new_cu[b] = before + (a.keep_code[c] >> 2);
  }
}

// ---- D2: the layer input after merging (Eq.16-18).  One block per kept position: an ordinary token's
// row is copied; a merged token becomes the mean of its window's rows, rescaled to the largest row
// norm of the window.  The few merged rows are computed in fp64 with one rounding to the storage
// type, so that the routing decisions taken on them afterwards see the correctly rounded token.
__device__ __forceinline__ double block_sum_f64(double v, double* red) {
#pragma unroll
  for (int sh = 32; sh >= 1; sh >>= 1) v += __shfl_xor(v, sh, 64);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

template <typename T>
__global__ __launch_bounds__(256) void merge_gather_kernel(
    const T* __restrict__ x, int d, const int32_t* __restrict__ kept_idx, const int32_t* __restrict__ n_dev,
    const uint8_t* __restrict__ is_merged, const int32_t* __restrict__ cu, int B, int Ttot, int W,
    const int32_t* __restrict__ vis_ord, const int32_t* __restrict__ vis_tok,
    const int32_t* __restrict__ seq_nv, T* __restrict__ x_merged, int mean_only) {
  __shared__ double red[4];
  const int p = blockIdx.x;
  if (p >= *n_dev) return;
  const int t = kept_idx[p];
  const T* src = x + (size_t)t * d;
  T* dst = x_merged + (size_t)p * d;
  if (!is_merged[p]) {
    for (int c = threadIdx.x; c < d; c += 256) dst[c] = src[c];
    return;
  }
  const int b = find_seq(cu, B, t);
  const int s = clampi(cu[b], 0, Ttot);
  const int ord = vis_ord[t];
  const int nv = seq_nv[b];
  const int w = (nv - ord < W) ? (nv - ord) : W;
  const int32_t* toks = vis_tok + s + ord;
  double max_row_sq = 0.0;
  for (int j = 0; j < w; ++j) {   // Eq.18: the largest token norm of the window
    const T* row = x + (size_t)toks[j] * d;
    double part = 0.0;
    for (int c = threadIdx.x; c < d; c += 256) {
      const double v = (double)to_f32(row[c]);
      part += v * v;
    }
    const double tot = block_sum_f64(part, red);
    max_row_sq = tot > max_row_sq ? tot : max_row_sq;
  }
  auto column_mean = [&](int c) -> double {   // Eq.16-17 with the window's real size
    double acc = 0.0;
    for (int j = 0; j < w; ++j) acc += (double)to_f32(x[(size_t)toks[j] * d + c]);
    return acc / (double)w;
  };
  double mean_sq = 0.0;
  for (int c = threadIdx.x; c < d; c += 256) {
    const double mu = column_mean(c);
    mean_sq += mu * mu;
  }
  const double mean_norm = sqrt(block_sum_f64(mean_sq, red));
  // mean_only: the plain mean of the merge-method ablation instead of MLERP's rescaling
  const double scale = mean_only ? 1.0 : (mean_norm > 0.0 ? sqrt(max_row_sq) / mean_norm : 0.0);
  for (int c = threadIdx.x; c < d; c += 256) dst[c] = from_f64<T>(column_mean(c) * scale);
}

__global__ void identity_kept_kernel(const uint8_t* __restrict__ is_visual,
                                     const int32_t* __restrict__ cu, int B, int T,
                                     int32_t* __restrict__ kept_idx, int32_t* __restrict__ new_cu,
                                     uint8_t* __restrict__ is_visual_out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < T) {
    if (kept_idx != nullptr) kept_idx[i] = i;
    if (is_visual_out != nullptr) is_visual_out[i] = is_visual[i];
  }
  if (i <= B && new_cu != nullptr) new_cu[i] = clampi(cu[i], 0, T);
}

// v of lane (l xor 2^jb).  jb is a constant after unrolling: distances 1 and 2 are quad permutes,
// 4 and 8 a pair of row shifts (lanes with the bit clear read upwards, the others downwards), all
// executed inside the ALU; 16 and 32 cross rows and go through the LDS crossbar.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_mov(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xf, 0xf, false);
}
__device__ __forceinline__ uint32_t lane_xor_pow2(int jb, uint32_t v, int lane) {
  switch (jb) {
    case 0: return dpp_mov<0xB1>(v);    // quad_perm [1,0,3,2]
    case 1: return dpp_mov<0x4E>(v);    // quad_perm [2,3,0,1]
    case 2: {
      const uint32_t up = dpp_mov<0x104>(v), dn = dpp_mov<0x114>(v);   // row_shl:4, row_shr:4
      return (lane & 4) ? dn : up;
    }
    case 3: {
      const uint32_t up = dpp_mov<0x108>(v), dn = dpp_mov<0x118>(v);   // row_shl:8, row_shr:8
      return (lane & 8) ? dn : up;
    }
    default: return (uint32_t)__shfl_xor((int)v, 1 << jb, 64);
  }
}

// ---- E: small batches.  One 1024-thread block takes the whole chain after the window scores:
// drop order, budget, compaction, permutation by expert and the grouped-GEMM tile lists, with the
// intermediate arrays in LDS.  At a few thousand tokens each of those steps is a few microseconds
// of work and the launches between them cost more than the steps themselves.
//   * every global input is fetched up front (thread i owns tokens i, i+1024, ...), every global
//     output is stored at the very end, so no barrier in between waits on memory;
//   * drop order: the order (normalised attention asc, score desc, index asc) is total, so a
//     bitonic sort of the integer keys (one window per thread; exchanges inside a wavefront by
//     lane shuffles, across wavefronts through LDS) gives every window its number of predecessors;
//   * permutation: as in the stand-alone kernels (per-expert position masks, popcount ranks), one
//     pass per 1024 tokens, one 64-bit mask word per wavefront.
constexpr int SB_THREADS = 1024;
constexpr int SB_MAX_TP = 4;                       // tokens per thread, at most
constexpr int SB_MAX_T = SB_THREADS * SB_MAX_TP;   // tokens
constexpr int SB_MAX_NW = 1024;                // windows of one sequence: one sort element per thread
constexpr int SB_MROW = 17;                    // 64-bit mask words per expert (16 + 1 against bank conflicts)
constexpr int SB_MAX_B = 512;                  // sequences whose bounds are cached in LDS

struct SmallArgs {
  int prune;                       // 0: keep every token
  const int32_t* T_dev;            // PERM_ONLY instantiation: device count of the tokens present (<= T)
  const uint8_t* is_visual;
  const int32_t* cu;
  int B, T, W;
  float retention, alpha;
  const int32_t* vis_ord;
  const int32_t* seq_nv;
  const float* win_s;
  const float* win_a;              // null without attention importance
  int32_t* kept_idx;
  int32_t* new_cu;
  uint8_t* is_visual_out;          // may be null
  const int32_t* topk_idx;
  int E, Kmax;
  int32_t* expert_offsets;
  int32_t* perm_src;
  int32_t* inv_perm;
  fmoe_ffn_geom geom;
  int n_shared, row_cap;
  fmoe_tile* tiles1;
  fmoe_tile* tiles2;
  int32_t* tile_count;
};

// SB_TP tokens per thread, at most KM experts per token (both fix the size of register arrays).
// PERM_ONLY: every token up to the device count *T_dev is kept (a.prune is 0); only the permutation
// and the tile lists are produced, kept_idx / new_cu / is_visual_out stay untouched.
template <int SB_TP, int KM, bool PERM_ONLY>
__global__ __launch_bounds__(SB_THREADS) void prune_dispatch_small_kernel(SmallArgs a) {
  __shared__ uint16_t s_kept[SB_MAX_T];
  // phase 1: precede u16[SB_MAX_T] | 2 x sort keys u64[SB_MAX_NW] | 2 x sort keys u32[SB_MAX_NW]
  // phase 2: position masks u64[FMOE_MAX_EXPERTS][SB_MROW]
  constexpr int U_BYTES = FMOE_MAX_EXPERTS * SB_MROW * 8;
  static_assert(SB_MAX_T * 2 + SB_MAX_NW * 24 <= U_BYTES, "phase-1 arrays fit");
  __shared__ __align__(16) unsigned char s_u[U_BYTES];
  __shared__ int s_off[FMOE_MAX_EXPERTS + 1], s_base[FMOE_MAX_EXPERTS];
  __shared__ int s_cu[SB_MAX_B + 1], s_nv[SB_MAX_B];
  __shared__ __align__(8) int s_scr[513];
  __shared__ uint16_t s_pfx[FMOE_MAX_EXPERTS * 16];   // rows of an expert ahead of each wavefront's tokens
  __shared__ int wave_tot[16];
  __shared__ float red[16];
  __shared__ int s_last;
  uint16_t* s_pre = reinterpret_cast<uint16_t*>(s_u);
  unsigned long long* sK = reinterpret_cast<unsigned long long*>(s_u + SB_MAX_T * 2);
  uint32_t* sA = reinterpret_cast<uint32_t*>(s_u + SB_MAX_T * 2 + SB_MAX_NW * 16);
  unsigned long long* mask = reinterpret_cast<unsigned long long*>(s_u);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int W = a.W, E = a.E, Kmax = a.Kmax, B = a.B;
  int T = a.T;
  if constexpr (PERM_ONLY) {
    const int Td = *a.T_dev;
    T = Td < T ? (Td > 0 ? Td : 0) : T;
  }

  // ---- all global inputs of this thread's tokens
  const int t_end = a.prune ? clampi(a.cu[B], 0, T) : T;
  int ord_r[SB_TP];
  uint8_t vis_r[SB_TP];
  int ex[SB_TP][KM];   // expert per slot, later (expert << 16 | row within the expert)
#pragma unroll
  for (int k = 0; k < SB_TP; ++k) {
    const int t = k * SB_THREADS + tid;
    ord_r[k] = (a.prune && t < t_end) ? a.vis_ord[t] : -1;   // past the last sequence: no ordinal, text
    vis_r[k] = (t < T && a.is_visual_out != nullptr) ? a.is_visual[t] : 0;
#pragma unroll
    for (int sl = 0; sl < KM; ++sl) {
      int e = -1;
      if (sl < Kmax && t < T) e = a.topk_idx[(size_t)t * Kmax + sl];
      ex[k][sl] = (e >= 0 && e < E) ? e : -1;
    }
  }
  const bool cached = B <= SB_MAX_B;
  if (cached) {
    for (int b = tid; b <= B; b += SB_THREADS) s_cu[b] = clampi(a.cu[b], 0, T);
    if (a.prune)
      for (int b = tid; b < B; b += SB_THREADS) s_nv[b] = a.seq_nv[b];
  }
  __syncthreads();
  const int32_t* cu = cached ? s_cu : a.cu;   // clamping a clamped bound changes nothing
  const int32_t* seq_nv = cached ? s_nv : a.seq_nv;

  // ---- drop order per sequence
  if (a.prune) {
    const bool has_attn = (a.win_a != nullptr);
    const float one_minus_alpha = 1.0f - a.alpha;
    for (int b = 0; b < B; ++b) {   // uniform over the block
      int s, e;
      seq_range(cu, b, T, s, e);
      const int nv = seq_nv[b];
      int n = (nv + W - 1) / W;
      n = n < SB_MAX_NW ? n : SB_MAX_NW;   // the launcher only takes batches where this holds
      if (n <= 0) continue;
      const float ws_r = (tid < n) ? a.win_s[s + tid] : 0.0f;
      const float wa_r = (has_attn && tid < n) ? a.win_a[s + tid] : 0.0f;
      float amax = 0.0f;
      if (has_attn) {   // per-sequence attention maximum (Eq.12)
        float m = (wa_r > 0.0f) ? wa_r : 0.0f;
#pragma unroll
        for (int sh = 32; sh >= 1; sh >>= 1) {
          const float o = __shfl_xor(m, sh, 64);
          m = (o > m) ? o : m;
        }
        __syncthreads();
        if (lane == 0) red[wave] = m;
        __syncthreads();
        amax = red[0];
#pragma unroll
        for (int w = 1; w < 16; ++w) amax = (red[w] > amax) ? red[w] : amax;
      }
      uint32_t ka = ~0u;               // padding sorts behind every window
      unsigned long long kk = ~0ull;
      if (tid < n) {
        float A;
        const float c = redundancy_score(ws_r, has_attn, wa_r, amax, a.alpha, one_minus_alpha, A);
        kk = ((unsigned long long)(~float_order_key(c)) << 32) | (uint32_t)tid;
        ka = float_order_key(A);
      }
      int N = 64;
      while (N < n) N <<= 1;
      const bool active = tid < N;   // whole wavefronts; the others only keep the barriers company
      int buf = 0;
      for (int k = 2; k <= N; k <<= 1) {
#pragma unroll
        for (int jb = 9; jb >= 0; --jb) {   // partner distances 512 .. 1, those below k
          const int j = 1 << jb;
          if (j >= k) continue;             // uniform
          uint32_t pa = ka;
          unsigned long long pk = kk;
          if (j >= 64) {   // partner in another wavefront: through LDS, buffers alternate
            if (active) {
              sK[buf * SB_MAX_NW + tid] = kk;
              if (has_attn) sA[buf * SB_MAX_NW + tid] = ka;
            }
            __syncthreads();
            if (active) {
              pk = sK[buf * SB_MAX_NW + (tid ^ j)];
              if (has_attn) pa = sA[buf * SB_MAX_NW + (tid ^ j)];
            }
            buf ^= 1;
          } else if (active) {
            const uint32_t lo = lane_xor_pow2(jb, (uint32_t)kk, lane);
            const uint32_t hi = lane_xor_pow2(jb, (uint32_t)(kk >> 32), lane);
            pk = ((unsigned long long)hi << 32) | lo;
            if (has_attn) pa = lane_xor_pow2(jb, ka, lane);
          }
          if (active) {
            const bool partner_first = (pa < ka) || (pa == ka && pk < kk);
            const bool want_min = (((tid & j) == 0) == ((tid & k) == 0));
            if (want_min == partner_first) {
              ka = pa;
              kk = pk;
            }
          }
        }
      }
      // thread r < n now holds the window at place r of the drop order
      const int wi = (int)(kk & 0xffffffffu);
      if (tid < n && wi == n - 1) s_last = tid;
      __syncthreads();
      if (tid < n) s_pre[s + wi] = (uint16_t)(tid | ((s_last < tid) ? 0x8000 : 0));
      __syncthreads();
    }
  }

  // ---- budget: text tokens and the leading tokens of each window stay
  bool keep_r[SB_TP];
#pragma unroll
  for (int k = 0; k < SB_TP; ++k) {
    const int t = k * SB_THREADS + tid;
    bool keep = false;
    if (t < T) {
      const int ord = ord_r[k];
      if (ord < 0) {
        keep = true;
      } else {
        const int b = find_seq(cu, B, t);
        const int s = clampi(cu[b], 0, T);
        const int pc = s_pre[s + ord / W];
        keep = (ord % W) < window_keep_lead(ord, seq_nv[b], W, a.retention,
                                            (pc & 0x7fff) | ((pc >> 15) << 30));
      }
    }
    keep_r[k] = keep;
  }
  __syncthreads();   // s_pre is dead from here on: the masks take its place

  // ---- compaction + per-expert ranks, one pass per 1024 tokens
  if (tid < FMOE_MAX_EXPERTS) s_base[tid] = 0;
  int pos_r[SB_TP];
  int running = 0;
#pragma unroll
  for (int k = 0; k < SB_TP; ++k) {
    pos_r[k] = -1;
    if (k * SB_THREADS < T) {   // uniform
      const int t = k * SB_THREADS + tid;
      const bool keep = keep_r[k];
      const unsigned long long m = __ballot(keep);
      const int before = __popcll(m & ((1ull << lane) - 1ull));
      if (lane == 0) wave_tot[wave] = __popcll(m);
      for (int i = tid; i < E * SB_MROW; i += SB_THREADS) mask[i] = 0ull;
      __syncthreads();
      int wave_base = 0, total = 0;
#pragma unroll
      for (int w = 0; w < 16; ++w) {
        if (w < wave) wave_base += wave_tot[w];
        total += wave_tot[w];
      }
      if (keep) {
        pos_r[k] = running + wave_base + before;
        s_kept[pos_r[k]] = (uint16_t)t;
#pragma unroll
        for (int sl = 0; sl < KM; ++sl)
          if (sl < Kmax && ex[k][sl] >= 0) atomicOr(&mask[ex[k][sl] * SB_MROW + wave], 1ull << lane);
      }
      running += total;
      __syncthreads();
      // item (expert, wavefront w): rows of the expert so far = earlier passes + wavefronts below w
      for (int it = tid; it < E * 16; it += SB_THREADS) {   // 16 consecutive lanes share an expert
        const int e = it >> 4, w = it & 15;
        const int c = __popcll(mask[e * SB_MROW + w]);
        const int base = s_base[e];
        int incl = c;
#pragma unroll
        for (int sh = 1; sh < 16; sh <<= 1) {
          const int o = __shfl_up(incl, sh, 16);
          if (w >= sh) incl += o;
        }
        s_pfx[it] = (uint16_t)(base + incl - c);
        if (w == 15) s_base[e] = base + incl;   // same wavefront: every lane has read the old value
      }
      __syncthreads();
      if (keep) {
#pragma unroll
        for (int sl = 0; sl < KM; ++sl) {
          if (sl < Kmax && ex[k][sl] >= 0) {
            const int e = ex[k][sl];
            const int rank = (int)s_pfx[e * 16 + wave] +
                             __popcll(mask[e * SB_MROW + wave] & ((1ull << lane) - 1ull));
            ex[k][sl] = (e << 16) | rank;
          }
        }
      } else {
#pragma unroll
        for (int sl = 0; sl < KM; ++sl) ex[k][sl] = -1;
      }
      __syncthreads();
    }
  }
  const int n = running;

  // ---- expert offsets: exclusive scan of the (at most 256) totals, four per lane
  __syncthreads();
  if (wave == 0) {
    int c[4], sum = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int e = 4 * lane + q;
      c[q] = (e < E) ? s_base[e] : 0;
      sum += c[q];
    }
    int incl = sum;
#pragma unroll
    for (int sh = 1; sh < 64; sh <<= 1) {
      const int o = __shfl_up(incl, sh, 64);
      if (lane >= sh) incl += o;
    }
    int excl = incl - sum;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      s_off[4 * lane + q] = excl;
      excl += c[q];
    }
    if (lane == 63) s_off[FMOE_MAX_EXPERTS] = incl;
  }
  __syncthreads();

  // ---- grouped-GEMM tile lists
  fmoe_build_tiles(s_off, E, a.row_cap, n, a.n_shared, a.geom.bm, a.geom.tile_cap, a.geom.cols1,
                   a.geom.scols1, a.tiles1, a.tiles2, a.tile_count, s_scr);

  // ---- outputs
  if (tid <= E) a.expert_offsets[tid] = s_off[tid];
  for (int b = tid; b <= B && !PERM_ONLY; b += SB_THREADS) {   // new_cu[b] = kept tokens before the sequence start
    const int c = clampi(cu[b], 0, T);
    int lo = 0, hi = n;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if ((int)s_kept[mid] < c) lo = mid + 1; else hi = mid;
    }
    a.new_cu[b] = lo;
  }
#pragma unroll
  for (int k = 0; k < SB_TP; ++k) {
    const int p = pos_r[k];
    if (p >= 0) {
      if constexpr (!PERM_ONLY) {
        a.kept_idx[p] = k * SB_THREADS + tid;
        if (a.is_visual_out != nullptr) a.is_visual_out[p] = vis_r[k];
      }
#pragma unroll
      for (int sl = 0; sl < KM; ++sl) {
        if (sl < Kmax) {
          int row = -1;
          if (ex[k][sl] >= 0) {
            row = s_off[ex[k][sl] >> 16] + (ex[k][sl] & 0xffff);
            if (row < a.row_cap) a.perm_src[row] = p;
          }
          a.inv_perm[(size_t)p * Kmax + sl] = row;
        }
      }
    }
  }
}

// One wavefront per window unit (floor(T/W) + B units cover every window), four per block.
void launch_window_scores(const float* probs, const int32_t* cu_seqlens, int B, int T, int E, int W,
                          int sim_mode, const int32_t* vis_tok, const int32_t* seq_nv, const float* attn,
                          float* win_s, float* win_a, int32_t* precede, int32_t* rank_c, hipStream_t stream) {
  const int n_units = T / W + B;
  const dim3 grid((n_units + 3) / 4);
  if ((long long)W * E <= WS_TILE)
    hipLaunchKernelGGL(window_score_kernel<true>, grid, dim3(256), 0, stream, probs, cu_seqlens, B, T, E, W,
                       sim_mode, vis_tok, seq_nv, attn, win_s, win_a, precede, rank_c);
  else
    hipLaunchKernelGGL(window_score_kernel<false>, grid, dim3(256), 0, stream, probs, cu_seqlens, B, T, E, W,
                       sim_mode, vis_tok, seq_nv, attn, win_s, win_a, precede, rank_c);
}

}  // namespace

int launch_prune(const fmoe_ctx* ctx, const fmoe_prune_params* pp, const float* probs,
                 const uint8_t* is_visual, const int32_t* cu_seqlens, int B, int T,
                 const float* attn, int32_t* kept_idx, int32_t* new_cu_seqlens, float* scores_out,
                 uint8_t* is_visual_out, const void* x_in, void* x_merged, uint8_t* is_merged_out,
                 void* ws, const fmoe_ws_layout& L, hipStream_t stream, bool ordinals_ready) {
  char* base = static_cast<char*>(ws);
  int32_t* vis_tok = reinterpret_cast<int32_t*>(base + L.vis_tok);
  int32_t* vis_ord = reinterpret_cast<int32_t*>(base + L.vis_ord);
  int32_t* seq_nv = reinterpret_cast<int32_t*>(base + L.seq_nv);
  float* win_s = reinterpret_cast<float*>(base + L.win_s);
  float* win_a = attn ? reinterpret_cast<float*>(base + L.win_a) : nullptr;
  int32_t* drop_from = reinterpret_cast<int32_t*>(base + L.drop_from);
  int32_t* keep_prefix = reinterpret_cast<int32_t*>(base + L.keep_prefix);
  const bool merging = pp->gamma > 0.0f;
  int32_t* rank_c = merging ? reinterpret_cast<int32_t*>(base + L.rank_c) : nullptr;
  int32_t* win_merged = merging ? reinterpret_cast<int32_t*>(base + L.win_merged) : nullptr;
  int32_t* merged_before = merging ? reinterpret_cast<int32_t*>(base + L.merged_before) : nullptr;
  uint8_t* is_merged = is_merged_out;
  if (merging && is_merged == nullptr) is_merged = reinterpret_cast<uint8_t*>(base + L.is_merged);
  const int E = ctx->cfg.n_experts;
  if (T == 0 || B == 0) return launch_identity_kept(is_visual, cu_seqlens, B, T, kept_idx,
                                                    new_cu_seqlens, is_visual_out, stream);

  if (!ordinals_ready) {
    fmoe_prof_scope prof(ctx, SLOT_ORDINALS, stream);
    hipLaunchKernelGGL(seq_ordinals_kernel, dim3(B), dim3(256), 0, stream, is_visual, cu_seqlens, T,
                       vis_ord, vis_tok, seq_nv);
  }
  {
    fmoe_prof_scope prof(ctx, SLOT_SCORES, stream);
    launch_window_scores(probs, cu_seqlens, B, T, E, pp->window, pp->sim_mode, vis_tok, seq_nv, attn, win_s,
                         win_a, drop_from, rank_c, stream);
  }
  const int n_max = (T + pp->window - 1) / pp->window;   // no sequence has more windows
  const int gy = (n_max + SEL_JC - 1) / SEL_JC;
  const dim3 sel_grid((T + 255) / 256, gy < 4096 ? gy : 4096);
  {
    fmoe_prof_scope prof(ctx, SLOT_SELECT, stream);
    hipLaunchKernelGGL(select_kernel, sel_grid, dim3(256), 0, stream, cu_seqlens, B, T, pp->window,
                       pp->alpha, seq_nv, win_s, win_a, drop_from, scores_out, rank_c,
                       static_cast<const int32_t*>(nullptr));
  }
  const bool closed_form = merging && attn == nullptr;   // one order: the compaction derives the merged set
  if (merging && !closed_form) {   // which windows merge, then how many merged windows precede each window in drop order
    hipLaunchKernelGGL(merge_decide_kernel, dim3((T + 255) / 256), dim3(256), 0, stream, cu_seqlens, B, T,
                       pp->window, pp->retention, pp->gamma, seq_nv, rank_c, win_merged, merged_before);
    hipLaunchKernelGGL(select_kernel, sel_grid, dim3(256), 0, stream, cu_seqlens, B, T, pp->window,
                       pp->alpha, seq_nv, win_s, win_a, merged_before, static_cast<float*>(nullptr),
                       static_cast<int32_t*>(nullptr), static_cast<const int32_t*>(win_merged));
  }
  {
    fmoe_prof_scope prof(ctx, SLOT_COMPACT, stream);
    CompactArgs ca;
    ca.is_visual = is_visual; ca.cu = cu_seqlens; ca.B = B; ca.T = T; ca.W = pp->window;
    ca.retention = pp->retention; ca.gamma = pp->gamma;
    ca.vis_ord = vis_ord; ca.seq_nv = seq_nv; ca.precede = drop_from; ca.rank_c = rank_c;
    ca.win_merged = closed_form ? nullptr : win_merged; ca.merged_before = merged_before;
    ca.keep_code = keep_prefix; ca.blk_kept = reinterpret_cast<int32_t*>(base + L.compact_blk);
    ca.kept_idx = kept_idx; ca.new_cu = new_cu_seqlens; ca.is_visual_out = is_visual_out;
    ca.is_merged_out = merging ? is_merged : nullptr;
    const dim3 cgrid((T + 1 + CP_BLOCK - 1) / CP_BLOCK);
    hipLaunchKernelGGL(compact_flag_kernel, cgrid, dim3(CP_BLOCK), 0, stream, ca);
    hipLaunchKernelGGL(compact_write_kernel, cgrid, dim3(CP_BLOCK), 0, stream, ca);
  }
  if (merging) {
    if (ctx->cfg.dtype == FMOE_BF16)
      hipLaunchKernelGGL(merge_gather_kernel<bf16_t>, dim3(T), dim3(256), 0, stream,
                         static_cast<const bf16_t*>(x_in), ctx->cfg.d_model, kept_idx, new_cu_seqlens + B,
                         is_merged, cu_seqlens, B, T, pp->window, vis_ord, vis_tok, seq_nv,
                         static_cast<bf16_t*>(x_merged), pp->merge_mode);
    else
      hipLaunchKernelGGL(merge_gather_kernel<float>, dim3(T), dim3(256), 0, stream,
                         static_cast<const float*>(x_in), ctx->cfg.d_model, kept_idx, new_cu_seqlens + B,
                         is_merged, cu_seqlens, B, T, pp->window, vis_ord, vis_tok, seq_nv,
                         static_cast<float*>(x_merged), pp->merge_mode);
  }
  FMOE_HIP_CHECK(hipGetLastError());
  return FMOE_OK;
}

int launch_identity_kept(const uint8_t* is_visual, const int32_t* cu_seqlens, int B, int T,
                         int32_t* kept_idx, int32_t* new_cu_seqlens, uint8_t* is_visual_out,
                         hipStream_t stream) {
  const int n = (T > B + 1) ? T : B + 1;
  hipLaunchKernelGGL(identity_kept_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, is_visual,
                     cu_seqlens, B, T, kept_idx, new_cu_seqlens, is_visual_out);
  FMOE_HIP_CHECK(hipGetLastError());
  return FMOE_OK;
}

bool dispatch_small_fits(int T, int window, bool prune) {
  if (T <= 0 || T > SB_MAX_T) return false;
  return !prune || (T + window - 1) / window <= SB_MAX_NW;
}

int launch_prune_dispatch_small(const fmoe_ctx* ctx, const fmoe_prune_params* pp, bool prune,
                                const float* probs, const uint8_t* is_visual, const int32_t* cu_seqlens,
                                int B, int T, const float* attn, const int32_t* topk_idx,
                                int32_t* kept_idx, int32_t* new_cu_seqlens, uint8_t* is_visual_out,
                                int32_t* expert_offsets, int32_t* perm_src, int32_t* inv_perm, void* ws,
                                const fmoe_ws_layout& L, hipStream_t stream, const int32_t* T_dev,
                                bool write_kept) {
  char* base = static_cast<char*>(ws);
  int32_t* vis_tok = reinterpret_cast<int32_t*>(base + L.vis_tok);
  int32_t* vis_ord = reinterpret_cast<int32_t*>(base + L.vis_ord);
  int32_t* seq_nv = reinterpret_cast<int32_t*>(base + L.seq_nv);
  float* win_s = reinterpret_cast<float*>(base + L.win_s);
  float* win_a = attn ? reinterpret_cast<float*>(base + L.win_a) : nullptr;
  int32_t* drop_from = reinterpret_cast<int32_t*>(base + L.drop_from);
  const int E = ctx->cfg.n_experts;
  if (prune) {   // the visual ordinals were produced in the router's launch
    fmoe_prof_scope prof(ctx, SLOT_SCORES, stream);
    launch_window_scores(probs, cu_seqlens, B, T, E, pp->window, pp->sim_mode, vis_tok, seq_nv, attn, win_s,
                         win_a, drop_from, nullptr, stream);
  }
  SmallArgs a;
  a.prune = prune ? 1 : 0;
  a.T_dev = T_dev;
  a.is_visual = is_visual;
  a.cu = cu_seqlens;
  a.B = B; a.T = T; a.W = prune ? pp->window : 1;
  a.retention = prune ? pp->retention : 1.0f;
  a.alpha = prune ? pp->alpha : 1.0f;
  a.vis_ord = vis_ord; a.seq_nv = seq_nv; a.win_s = win_s; a.win_a = win_a;
  a.kept_idx = kept_idx; a.new_cu = new_cu_seqlens; a.is_visual_out = is_visual_out;
  a.topk_idx = topk_idx;
  a.E = E; a.Kmax = ctx->kmax;
  a.expert_offsets = expert_offsets; a.perm_src = perm_src; a.inv_perm = inv_perm;
  a.geom = fmoe_geom(ctx, T);
  a.n_shared = ctx->cfg.n_shared;
  a.row_cap = T * ctx->kmax;
  a.tiles1 = reinterpret_cast<fmoe_tile*>(base + L.tiles);
  a.tiles2 = reinterpret_cast<fmoe_tile*>(base + L.tiles2);
  a.tile_count = reinterpret_cast<int32_t*>(base + L.tile_count);
  {
    fmoe_prof_scope prof(ctx, SLOT_DISPATCH, stream);
    const bool fast = T <= 2 * SB_THREADS && ctx->kmax <= 8;
    if (!write_kept) {
      if (prune || T_dev == nullptr)
        return fmoe_fail(FMOE_ERR_INVALID_ARG, "small dispatch: the permutation-only form needs a device token count and no pruning");
      if (fast)
        hipLaunchKernelGGL((prune_dispatch_small_kernel<2, 8, true>), dim3(1), dim3(SB_THREADS), 0, stream, a);
      else
        hipLaunchKernelGGL((prune_dispatch_small_kernel<SB_MAX_TP, FMOE_MAX_TOPK, true>), dim3(1),
                           dim3(SB_THREADS), 0, stream, a);
    } else if (fast) {
      hipLaunchKernelGGL((prune_dispatch_small_kernel<2, 8, false>), dim3(1), dim3(SB_THREADS), 0, stream, a);
    } else {
      hipLaunchKernelGGL((prune_dispatch_small_kernel<SB_MAX_TP, FMOE_MAX_TOPK, false>), dim3(1),
                         dim3(SB_THREADS), 0, stream, a);
    }
  }
  FMOE_HIP_CHECK(hipGetLastError());
  return FMOE_OK;
}

