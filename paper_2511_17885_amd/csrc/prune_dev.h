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

// Number of leading tokens of visual ordinal `ord`'s window that survive (Sec. 3.2.3 budget and the
// drop rule): windows are dropped whole in drop order while they fit in eps = N_v - eta and the
// next one loses its last tokens.  pc = number of windows ahead of this window in drop order, bit
// 30 set when the sequence's last (possibly shorter) window is one of them.
__device__ __forceinline__ int window_keep_lead(int ord, int nv, int W, float retention, int pc) {
  const int n = (nv + W - 1) / W;
  const int i = ord / W;
  int eta = (int)floor((double)retention * (double)nv + 0.5);   // eta = floor(r*N_v + 1/2), fp64
  eta = eta > nv ? nv : eta;
  eta = eta < 1 ? 1 : eta;
  const int eps = nv - eta;
  const int count = pc & 0x3fffffff, last_first = pc >> 30;
  const int w_last = nv - (n - 1) * W;
  const int before = count * W - (last_first ? (W - w_last) : 0);
  const int wi = (i == n - 1) ? w_last : W;
  if (before + wi <= eps) return 0;
  if (before < eps) return wi - (eps - before);
  return wi;
}
#endif
