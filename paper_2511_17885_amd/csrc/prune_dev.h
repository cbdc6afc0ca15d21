// Device helpers of the pruning stage (paper Sec. 3.2) used by more than one kernel file.
#pragma once

#include "common.h"

#if defined(__HIPCC__)
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

// Visual ordinals of sequence b, by one 256-thread block (wave_tot: 4 ints of LDS).
// vis_ord[t] = number of visual tokens before t in its sequence (for visual t), -1 for text;
// vis_tok[cu[b] + j] = global index of the j-th visual token of sequence b; seq_nv[b] = N_v.
__device__ __forceinline__ void seq_ordinals_block(const uint8_t* __restrict__ is_visual,
                                                   const int32_t* __restrict__ cu, int b, int T,
                                                   int32_t* __restrict__ vis_ord,
                                                   int32_t* __restrict__ vis_tok,
                                                   int32_t* __restrict__ seq_nv, int* wave_tot) {
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

// monotone map float -> uint32: a < b <=> key(a) < key(b); -0 and +0 get the same key
__device__ __forceinline__ uint32_t float_order_key(float v) {
  v = v + 0.0f;
  const uint32_t u = __float_as_uint(v);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Eq.12-13: redundancy score C of a window from its similarity S and raw attention sum; A receives
// the normalised attention term (0 without attention, where C = S exactly).
__device__ __forceinline__ float redundancy_score(float S, bool has_attn, float a_raw, float amax,
                                                  float alpha, float one_minus_alpha, float& A) {
  if (!has_attn) {
    A = 0.0f;
    return S;
  }
  float a = a_raw;
  if (amax > 0.0f) a = a / amax;
  A = a;
  const float t1 = alpha * S;
  const float t2 = one_minus_alpha * a;
  return t1 - t2;
}

// eta = floor(r*N_v + 1/2) in fp64, clamped to [min(1,N_v), N_v] (Sec. 3.2.3, exact-count rule)
__device__ __forceinline__ int token_budget(int nv, float retention) {
  int eta = (int)floor((double)retention * (double)nv + 0.5);
  eta = eta > nv ? nv : eta;
  const int lo = nv < 1 ? nv : 1;
  return eta < lo ? lo : eta;
}

// Outcome of the greedy merge walk of Sec. 3.2.3 (windows in the order (C desc, index asc); a window
// of w >= 2 tokens merges if w-1 <= u, u -= w-1, at most m = floor(eta*gamma) merges) in closed form.
// All windows cost W-1 except a shorter last one (w_last-1; not mergeable if w_last == 1), so the walk
// is determined by L, the place of the last window in that order:
//   full windows merge iff their place among the full windows is < q_full; the last window iff last_m.
struct fmoe_merge_plan {
  int q_full;     // number of merged full-size windows (the first q_full of them in merge order)
  int last_m;     // 1: the (shorter) last window is merged
  int u_rem;      // tokens still to drop after merging
};
__device__ __forceinline__ fmoe_merge_plan merge_plan(int nv, int W, float retention, float gamma, int L) {
  fmoe_merge_plan p;
  const int eta = token_budget(nv, retention);
  const int eps = nv - eta;
  p.q_full = 0; p.last_m = 0; p.u_rem = eps;
  const int n = (nv + W - 1) / W;
  if (!(gamma > 0.0f) || n == 0 || W < 2) return p;
  const int m = (int)floor((double)eta * (double)gamma);
  const int c = W - 1;
  const int w_last = nv - (n - 1) * W;
  const bool short_last = w_last < W;
  if (!short_last) {                         // every window costs c
    int q = eps / c;
    q = q < m ? q : m;
    q = q < n ? q : n;
    p.q_full = q;
    p.u_rem = eps - q * c;
    return p;
  }
  const int n_full = n - 1;
  const int c_last = w_last - 1;
  int q0 = eps / c;                          // full windows that merge if nothing else interferes
  q0 = q0 < m ? q0 : m;
  q0 = q0 < n_full ? q0 : n_full;
  if (q0 < L) {                              // the walk stalls on a full window before reaching the last one:
    p.q_full = q0;                           // full windows never resume; the last one may still fit
    const int u = eps - q0 * c;
    p.last_m = (c_last >= 1 && q0 < m && c_last <= u) ? 1 : 0;
    p.u_rem = u - p.last_m * c_last;
    return p;
  }
  // the L full windows ahead of the last one all merge, then the last one gets its turn
  int u = eps - L * c;
  p.last_m = (c_last >= 1 && L < m && c_last <= u) ? 1 : 0;
  u -= p.last_m * c_last;
  int more = u / c;
  const int room = m - L - p.last_m;
  more = more < room ? more : room;
  more = more < n_full - L ? more : n_full - L;
  more = more > 0 ? more : 0;
  p.q_full = L + more;
  p.u_rem = u - more * c;
  return p;
}

// Number of leading tokens of visual ordinal `ord`'s window that survive (Sec. 3.2.3 budget and the
// drop rule): windows are dropped whole in drop order while they fit in eps = N_v - eta and the
// next one loses its last tokens.  pc = number of windows ahead of this window in drop order, bit
// 30 set when the sequence's last (possibly shorter) window is one of them.
__device__ __forceinline__ int window_keep_lead(int ord, int nv, int W, float retention, int pc) {
  const int n = (nv + W - 1) / W;
  const int i = ord / W;
  const int eps = nv - token_budget(nv, retention);
  const int count = pc & 0x3fffffff, last_first = pc >> 30;
  const int w_last = nv - (n - 1) * W;
  const int before = count * W - (last_first ? (W - w_last) : 0);
  const int wi = (i == n - 1) ? w_last : W;
  if (before + wi <= eps) return 0;
  if (before < eps) return wi - (eps - before);
  return wi;
}

// The same with window merging: `merged_before` merged windows are among the `pc` predecessors (they
// are no longer part of the drop walk), the last window counts as a predecessor only if it was not
// merged, and the budget is what merging left.
__device__ __forceinline__ int window_keep_lead_merge(int ord, int nv, int W, int pc, int merged_before,
                                                      bool last_merged, int u_rem) {
  const int n = (nv + W - 1) / W;
  const int i = ord / W;
  const int count = (pc & 0x3fffffff) - (merged_before & 0x3fffffff);
  const int last_first = (pc >> 30) && !last_merged;
  const int w_last = nv - (n - 1) * W;
  const int before = count * W - (last_first ? (W - w_last) : 0);
  const int wi = (i == n - 1) ? w_last : W;
  if (before + wi <= u_rem) return 0;
  if (before < u_rem) return wi - (u_rem - before);
  return wi;
}
#endif
