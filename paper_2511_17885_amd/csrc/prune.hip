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

namespace {

__device__ __forceinline__ float wave_sum_butterfly(float p) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) p = p + __shfl_xor(p, s, 64);
  return p;
}

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// sequence b covers [seq_begin, seq_end) after clamping to [0,T] and to non-decreasing order, so
// that a malformed cu_seqlens can never index outside the token arrays.
__device__ __forceinline__ void seq_range(const int32_t* cu, int b, int T, int& s, int& e) {
  s = clampi(cu[b], 0, T);
  e = clampi(cu[b + 1], s, T);
}

// largest b in [0,B) with cu[b] <= g (cu is non-decreasing, cu[0] = 0)
__device__ __forceinline__ int find_seq(const int32_t* cu, int B, int g) {
  int lo = 0, hi = B - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (cu[mid] <= g) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// ---- A: visual ordinals.  One block per sequence.
// vis_ord[t] = number of visual tokens before t in its sequence (for visual t), -1 for text;
// vis_tok[cu[b] + j] = global index of the j-th visual token of sequence b; seq_nv[b] = N_v.
__global__ __launch_bounds__(256) void seq_ordinals_kernel(
    const uint8_t* __restrict__ is_visual, const int32_t* __restrict__ cu, int T,
    int32_t* __restrict__ vis_ord, int32_t* __restrict__ vis_tok, int32_t* __restrict__ seq_nv) {
  __shared__ int wave_tot[4];
  const int b = blockIdx.x;
  int s, e;
  seq_range(cu, b, T, s, e);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int running = 0;
  for (int base = s; base < e; base += 256) {
    const int t = base + threadIdx.x;
    const bool vis = (t < e) && (is_visual[t] != 0);
    const unsigned long long mask = __ballot(vis);
    const int before = __popcll(mask & ((1ull << lane) - 1ull));
    if (lane == 0) wave_tot[wave] = __popcll(mask);
    __syncthreads();
    int wave_base = 0, total = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      if (w < wave) wave_base += wave_tot[w];
      total += wave_tot[w];
    }
    if (t < e) {
      const int ord = running + wave_base + before;
      vis_ord[t] = vis ? ord : -1;
      if (vis) vis_tok[s + ord] = t;
    }
    running += total;
    __syncthreads();
  }
  if (threadIdx.x == 0) seq_nv[b] = running;
}

// ---- B: window scores.  One wavefront per slot g in [0,T); lanes <-> experts.
// win_s[g] = S_i (Eq.10 or Eq.8), win_a[g] = raw window attention sum (Eq.11) if attn.
__global__ __launch_bounds__(256) void window_score_kernel(
    const float* __restrict__ probs, const int32_t* __restrict__ cu, int B, int T, int E, int W,
    int sim_mode, const int32_t* __restrict__ vis_tok, const int32_t* __restrict__ seq_nv,
    const float* __restrict__ attn, float* __restrict__ win_s, float* __restrict__ win_a,
    int32_t* __restrict__ precede) {
  const int lane = threadIdx.x & 63;
  const int g = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (g >= T) return;
  if (lane == 0) precede[g] = 0;   // accumulated by select_kernel
  const int b = find_seq(cu, B, g);
  int s, e;
  seq_range(cu, b, T, s, e);
  const int i = g - s;
  const int nv = seq_nv[b];
  if (i < 0 || (long long)i * W >= nv) return;  // not a window of this sequence
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
  float S;
  if (sim_mode == 0) {
    // Eq.9: mean row (sequential over the window, one divide), Eq.10: mean cosine to it
    float mean[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int ex = lane + 64 * r;
      float acc = 0.0f;
      if (ex < E) {
        acc = probs[(size_t)toks[0] * E + ex];
        for (int j = 1; j < w; ++j) acc = acc + probs[(size_t)toks[j] * E + ex];
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
          const float v = probs[(size_t)toks[j] * E + ex];
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
        rj[r] = (ex < E) ? probs[(size_t)toks[j] * E + ex] : 0.0f;
        if (ex < E) pn = fmaf(rj[r], rj[r], pn);
      }
      const float nj = sqrtf(wave_sum_butterfly(pn));
      for (int q = 0; q < j; ++q) {
        float pd = 0.0f, pq = 0.0f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int ex = lane + 64 * r;
          if (ex < E) {
            const float v = probs[(size_t)toks[q] * E + ex];
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

__device__ __forceinline__ uint32_t float_order_key(float v) {   // monotone: a < b <=> key(a) < key(b)
  v = v + 0.0f;                                                   // -0 -> +0, so equal floats get equal keys
  const uint32_t u = __float_as_uint(v);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(256) void select_kernel(
    const int32_t* __restrict__ cu, int B, int T, int W, float alpha,
    const int32_t* __restrict__ seq_nv, const float* __restrict__ win_s,
    const float* __restrict__ win_a, int32_t* __restrict__ precede, float* __restrict__ scores_out) {
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
      const float Sj = win_s[s + j];
      if (!has_attn) {
        Aj = 0.0f;
        return Sj;
      }
      float a = win_a[s + j];
      if (amax > 0.0f) a = a / amax;
      Aj = a;
      const float t1 = alpha * Sj;
      const float t2 = one_minus_alpha * a;
      return t1 - t2;
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
    int count = 0, last_first = 0;
    for (int j0 = jbase; j0 < n; j0 += (int)gridDim.y * SEL_JC) {   // uniform
      __syncthreads();
      if (threadIdx.x < SEL_JC) {
        const int jl = j0 + threadIdx.x;
        unsigned long long kj = ~0ull;   // sentinel: precedes nothing
        uint32_t aj = ~0u;
        if (jl < n) {
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
        }
      }
    }
    if (mine && (count | last_first)) atomicAdd(&precede[g], count + (last_first << 30));
  }
}

// number of leading tokens of visual ordinal `ord`'s window that survive (Sec. 3.2.3 budget and the
// drop rule): windows are dropped whole in drop order while they fit in eps = N_v - eta and the
// next one loses its last tokens.
__device__ __forceinline__ int window_keep_lead(int ord, int nv, int W, float retention,
                                                const int32_t* precede_seq) {
  const int n = (nv + W - 1) / W;
  const int i = ord / W;
  int eta = (int)floor((double)retention * (double)nv + 0.5);   // eta = floor(r*N_v + 1/2), fp64
  eta = eta > nv ? nv : eta;
  eta = eta < 1 ? 1 : eta;
  const int eps = nv - eta;
  const int pc = precede_seq[i];
  const int count = pc & 0x3fffffff, last_first = pc >> 30;
  const int w_last = nv - (n - 1) * W;
  const int before = count * W - (last_first ? (W - w_last) : 0);
  const int wi = (i == n - 1) ? w_last : W;
  if (before + wi <= eps) return 0;
  if (before < eps) return wi - (eps - before);
  return wi;
}

// ---- D: budget + compaction.  A single block walks the tokens in order, keeps text tokens and the
// leading tokens of each window, and writes ascending kept indices; keep_prefix[t] = kept tokens
// before t.
__global__ __launch_bounds__(1024) void compact_kernel(
    const uint8_t* __restrict__ is_visual, const int32_t* __restrict__ cu, int B, int T, int W,
    float retention, const int32_t* __restrict__ vis_ord, const int32_t* __restrict__ seq_nv,
    const int32_t* __restrict__ precede, int32_t* __restrict__ keep_prefix,
    int32_t* __restrict__ kept_idx,
    int32_t* __restrict__ new_cu, uint8_t* __restrict__ is_visual_out) {
  __shared__ int wave_tot[16];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int running = 0;
  for (int base = 0; base < T; base += 1024) {
    const int t = base + threadIdx.x;
    bool keep = false;
    if (t < T) {
      const int ord = vis_ord[t];
      if (ord < 0) {
        keep = true;
      } else {
        const int b = find_seq(cu, B, t);
        const int s = clampi(cu[b], 0, T);
        keep = (ord % W) < window_keep_lead(ord, seq_nv[b], W, retention, precede + s);
      }
    }
    const unsigned long long mask = __ballot(keep);
    const int before = __popcll(mask & ((1ull << lane) - 1ull));
    if (lane == 0) wave_tot[wave] = __popcll(mask);
    __syncthreads();
    int wave_base = 0, total = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
      if (w < wave) wave_base += wave_tot[w];
      total += wave_tot[w];
    }
    if (t < T) {
      const int pos = running + wave_base + before;
      keep_prefix[t] = pos;
      if (keep) {
        kept_idx[pos] = t;
        if (is_visual_out != nullptr) is_visual_out[pos] = is_visual[t];
      }
    }
    running += total;
    __syncthreads();
  }
  if (threadIdx.x == 0) keep_prefix[T] = running;
  __syncthreads();
  for (int b = threadIdx.x; b <= B; b += 1024) new_cu[b] = keep_prefix[clampi(cu[b], 0, T)];
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

}  // namespace

int launch_prune(const fmoe_ctx* ctx, const fmoe_prune_params* pp, const float* probs,
                 const uint8_t* is_visual, const int32_t* cu_seqlens, int B, int T,
                 const float* attn, int32_t* kept_idx, int32_t* new_cu_seqlens, float* scores_out,
                 uint8_t* is_visual_out, void* ws, const fmoe_ws_layout& L, hipStream_t stream) {
  char* base = static_cast<char*>(ws);
  int32_t* vis_tok = reinterpret_cast<int32_t*>(base + L.vis_tok);
  int32_t* vis_ord = reinterpret_cast<int32_t*>(base + L.vis_ord);
  int32_t* seq_nv = reinterpret_cast<int32_t*>(base + L.seq_nv);
  float* win_s = reinterpret_cast<float*>(base + L.win_s);
  float* win_a = attn ? reinterpret_cast<float*>(base + L.win_a) : nullptr;
  int32_t* drop_from = reinterpret_cast<int32_t*>(base + L.drop_from);
  int32_t* keep_prefix = reinterpret_cast<int32_t*>(base + L.keep_prefix);
  const int E = ctx->cfg.n_experts;
  if (T == 0 || B == 0) return launch_identity_kept(is_visual, cu_seqlens, B, T, kept_idx,
                                                    new_cu_seqlens, is_visual_out, stream);

  {
    fmoe_prof_scope prof(ctx, SLOT_ORDINALS, stream);
    hipLaunchKernelGGL(seq_ordinals_kernel, dim3(B), dim3(256), 0, stream, is_visual, cu_seqlens, T,
                       vis_ord, vis_tok, seq_nv);
  }
  {
    fmoe_prof_scope prof(ctx, SLOT_SCORES, stream);
    hipLaunchKernelGGL(window_score_kernel, dim3((T + 3) / 4), dim3(256), 0, stream, probs, cu_seqlens,
                       B, T, E, pp->window, pp->sim_mode, vis_tok, seq_nv, attn, win_s, win_a, drop_from);
  }
  {
    fmoe_prof_scope prof(ctx, SLOT_SELECT, stream);
    const int n_max = (T + pp->window - 1) / pp->window;   // no sequence has more windows
    const int gy = (n_max + SEL_JC - 1) / SEL_JC;
    hipLaunchKernelGGL(select_kernel, dim3((T + 255) / 256, gy < 4096 ? gy : 4096), dim3(256), 0,
                       stream, cu_seqlens, B, T, pp->window, pp->alpha, seq_nv, win_s, win_a, drop_from,
                       scores_out);
  }
  {
    fmoe_prof_scope prof(ctx, SLOT_COMPACT, stream);
    hipLaunchKernelGGL(compact_kernel, dim3(1), dim3(1024), 0, stream, is_visual, cu_seqlens, B, T,
                       pp->window, pp->retention, vis_ord, seq_nv, drop_from, keep_prefix, kept_idx,
                       new_cu_seqlens, is_visual_out);
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
