// CPU oracle for the FastMMoE MoE-layer prefill path.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the tests, the
// smoke check and the benchmark's cpu_baseline leg compare the HIP library against.  It is
// never linked into, imported by, or called from the product path, and it shares no source
// with it.  Every function follows the paper's definition step by step (citations are to the
// paper's sections and equations; the equations of Sec. 3 are unnumbered there and are counted
// here in order of appearance: Eq.1 router logits ... Eq.18 MLERP rescale).
//
// Arithmetic.
//  * Every float that feeds a decision (expert ids, window ranking, kept set) is computed in
//    IEEE fp32 with a fixed operation order ("canonical arithmetic", below), because the
//    decisions must come out identical on any machine that follows the same order.
//  * Every value that is only compared within a tolerance (expert FFN, combine) is computed
//    in fp64, with the two roundings the bf16 data path has by definition: the SwiGLU
//    activation h is rounded to the storage dtype, and the layer output is rounded once.
//
// Canonical arithmetic (fp32, round-to-nearest-even, no contraction except written fmaf):
//  * dot_seq(a,b,n): the plain fp32 dot product in index order with fused multiply-add:
//    acc = +0; for k = 0..n-1: acc = fmaf(a[k], b[k], acc).  Used for the router logits (Eq.1).
//  * sum_canon(v[0..n)):  64 partials p[l] (l = 0..63); p[l] starts at +0 and adds v[l+64j] for
//    j = 0,1,.. in ascending order; then for s in 32,16,8,4,2,1: p[l] <- p[l] + p[l xor s]
//    for all l at once; the result is p[0].  Used for the softmax denominator (Eq.2).
//  * dot_canon(a,b,n): same shape as sum_canon, with p[l] <- fmaf(a[l+64j], b[l+64j], p[l]).
//    Used for the dot products over the E routing probabilities (Eq.8-10).
//  * exp_canon(x), x <= 0:  t = x*LOG2E; n = rint(t); r = fmaf(-n, LN2_HI, x);
//    r = fmaf(-n, LN2_LO, r); p = degree-7 Taylor polynomial of e^r in Horner form with fmaf;
//    result = p * 2^n, and exactly 0 when n < -125.
//  * '/' and sqrt are the correctly rounded IEEE operations.
//
// Pins: the paper prints no numeric worked example of the layer, so the functions here are pinned
// by closed forms, invariants, special cases that reduce to textbook routines and brute force on
// small inputs (tests/test_oracle_pins.py); none is left unpinned.
//
// Build: g++ -O2 -ffp-contract=off -mfma -fopenmp -shared -fPIC (see oracle/build.py).

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>
#include <algorithm>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

// ---------------------------------------------------------------- canonical fp32 arithmetic
inline float butterfly64(float* p) {
  for (int s = 32; s >= 1; s >>= 1) {
    float q[64];
    for (int l = 0; l < 64; ++l) q[l] = p[l] + p[l ^ s];
    for (int l = 0; l < 64; ++l) p[l] = q[l];
  }
  return p[0];
}

float sum_canon(const float* v, int n) {
  float p[64];
  for (int l = 0; l < 64; ++l) p[l] = 0.0f;
  for (int i = 0; i < n; ++i) p[i & 63] = p[i & 63] + v[i];
  return butterfly64(p);
}

float dot_canon(const float* a, const float* b, int n) {
  float p[64];
  for (int l = 0; l < 64; ++l) p[l] = 0.0f;
  for (int i = 0; i < n; ++i) p[i & 63] = std::fmaf(a[i], b[i], p[i & 63]);
  return butterfly64(p);
}

float dot_seq(const float* a, const float* b, int n) {
  float acc = 0.0f;
  for (int i = 0; i < n; ++i) acc = std::fmaf(a[i], b[i], acc);
  return acc;
}

float exp_canon(float x) {
  const float LOG2E = 0x1.715476p+0f;    // 1.44269502
  const float LN2_HI = 0x1.62e400p-1f;   // 0.693145752 (low mantissa bits zero)
  const float LN2_LO = 0x1.7f7d1cp-20f;  // 1.42860677e-6
  float t = x * LOG2E;
  float n = std::nearbyintf(t);          // default rounding mode: to nearest, ties to even
  float r = std::fmaf(-n, LN2_HI, x);
  r = std::fmaf(-n, LN2_LO, r);
  float p = 0x1.a01a02p-13f;             // 1/5040
  p = std::fmaf(p, r, 0x1.6c16c2p-10f);  // 1/720
  p = std::fmaf(p, r, 0x1.111112p-7f);   // 1/120
  p = std::fmaf(p, r, 0x1.555556p-5f);   // 1/24
  p = std::fmaf(p, r, 0x1.555556p-3f);   // 1/6
  p = std::fmaf(p, r, 0.5f);
  p = std::fmaf(p, r, 1.0f);
  p = std::fmaf(p, r, 1.0f);
  if (!(n >= -125.0f)) return 0.0f;
  int32_t bits = (int32_t)((int)n + 127) << 23;   // the float 2^n, n in [-125, 0]
  float scale;
  std::memcpy(&scale, &bits, 4);
  return p * scale;
}

// round an fp64 / fp32 value to bf16 (nearest even) and return it widened
inline float round_bf16(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  if ((u & 0x7f800000u) == 0x7f800000u) return f;  // inf / nan unchanged
  u += 0x7fffu + ((u >> 16) & 1u);
  u &= 0xffff0000u;
  std::memcpy(&f, &u, 4);
  return f;
}

// One rounding from fp64 to the storage dtype.  bf16: round the exact double directly (not
// through fp32 first) so that no double rounding enters the reference.
inline float round_store(double v, int is_bf16) {
  if (!is_bf16) return (float)v;
  if (!(std::fabs(v) < 3.3e38)) return (float)v;
  if (v == 0.0) return (float)v;
  int e;
  double m = std::frexp(v, &e);            // v = m * 2^e, 0.5 <= |m| < 1
  int shift = 8;                            // bf16 keeps 8 significant bits
  if (e - 1 < -126) shift -= (-126 - (e - 1));  // subnormal range: fewer bits
  if (shift < 0) return (float)(v < 0 ? -0.0 : 0.0);
  double scaled = std::ldexp(m, shift);
  double rn = std::nearbyint(scaled);       // ties to even
  return (float)std::ldexp(rn, e - shift);
}

// ---------------------------------------------------------------- Eq.1-2: logits, softmax
// Z[e] = dot_seq(x_t, W_E[e]) (+ bias[e], one rounded add); P = exp(Z - max) / sum.
void route_probs_row(const float* xt, int d, int E, const float* Wr, const float* bias,
                     float* P /*[E]*/) {
  std::vector<float> z(E), q(E);
  for (int e = 0; e < E; ++e) {
    float v = dot_seq(xt, Wr + (size_t)e * d, d);
    if (bias) v = v + bias[e];
    z[e] = v;
  }
  float m = z[0];
  for (int e = 1; e < E; ++e) m = (z[e] > m) ? z[e] : m;
  for (int e = 0; e < E; ++e) q[e] = exp_canon(z[e] - m);
  float s = sum_canon(q.data(), E);
  for (int e = 0; e < E; ++e) P[e] = q[e] / s;
}

// fp64 shadow of the same row, library exp, plain sums: used only to check that the canonical
// recipe is an accurate softmax.
void route_probs_row_f64(const float* xt, int d, int E, const float* Wr, const float* bias,
                         double* P) {
  std::vector<double> z(E);
  double m = -INFINITY;
  for (int e = 0; e < E; ++e) {
    double v = 0.0;
    for (int h = 0; h < d; ++h) v += (double)xt[h] * (double)Wr[(size_t)e * d + h];
    if (bias) v += (double)bias[e];
    z[e] = v;
    if (v > m) m = v;
  }
  double s = 0.0;
  for (int e = 0; e < E; ++e) { P[e] = std::exp(z[e] - m); s += P[e]; }
  for (int e = 0; e < E; ++e) P[e] /= s;
}

// ---------------------------------------------------------------- Eq.3, Eq.5: top-k and gates
// The k experts with the highest probability; ties go to the lower expert index; the list is
// ordered by (probability descending, index ascending).  Gates: P_j / sum of the selected P
// (sum taken sequentially in list order, fp32).
void topk_gates_row(const float* P, int E, int k, int Kmax, int renorm,
                    int32_t* idx /*[Kmax]*/, float* gate /*[Kmax]*/) {
  std::vector<char> taken(E, 0);
  for (int s = 0; s < Kmax; ++s) { idx[s] = -1; gate[s] = 0.0f; }
  for (int s = 0; s < k; ++s) {
    int best = -1;
    for (int e = 0; e < E; ++e) {
      if (taken[e]) continue;
      if (best < 0 || P[e] > P[best]) best = e;   // strict '>' keeps the lowest index on ties
    }
    taken[best] = 1;
    idx[s] = best;
  }
  float den = 0.0f;
  for (int s = 0; s < k; ++s) den = den + P[idx[s]];
  for (int s = 0; s < k; ++s) gate[s] = renorm ? (P[idx[s]] / den) : P[idx[s]];
}

// ---------------------------------------------------------------- selection-strategy ablation (Sec. 4)
// Which k of a token's K_base highest-probability experts stay active when its activation is
// reduced: the k highest (TopK, strategy 0 -- the method itself), k chosen at random (RandomK, 1)
// or the k lowest (MinK, 2).  The candidates are the token's top-K_base list in the order of
// topk_gates_row; the kept experts are listed in that same order and the gates are renormalised
// over them (Eq.5).  The paper does not say how RandomK draws; here every candidate position r of
// token t gets the 64-bit key splitmix64(seed, n = 16 t + r + 1) (the n-th output of the SplitMix64
// generator started at `seed`) and the k smallest keys win (equal keys: lower position).
uint64_t splitmix64_nth(uint64_t seed, uint64_t n) {
  uint64_t z = seed + n * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

void select_gates_row(const float* P, int E, int k, int k_base, int strategy, uint64_t seed, int t,
                      int Kmax, int renorm, int32_t* idx, float* gate) {
  std::vector<int32_t> cand(k_base);
  std::vector<float> unused(k_base);
  topk_gates_row(P, E, k_base, k_base, 0, cand.data(), unused.data());
  std::vector<int> keep;   // kept candidate positions, ascending
  if (strategy == 2) {
    for (int r = k_base - k; r < k_base; ++r) keep.push_back(r);
  } else if (strategy == 1) {
    std::vector<uint64_t> key(k_base);
    for (int r = 0; r < k_base; ++r) key[r] = splitmix64_nth(seed, (uint64_t)t * 16u + (uint64_t)r + 1u);
    for (int r = 0; r < k_base; ++r) {
      int rank = 0;
      for (int q = 0; q < k_base; ++q)
        if (key[q] < key[r] || (key[q] == key[r] && q < r)) ++rank;
      if (rank < k) keep.push_back(r);
    }
  } else {
    for (int r = 0; r < k; ++r) keep.push_back(r);
  }
  for (int s = 0; s < Kmax; ++s) { idx[s] = -1; gate[s] = 0.0f; }
  float den = 0.0f;
  for (int s = 0; s < k; ++s) {
    idx[s] = cand[keep[s]];
    den = den + P[idx[s]];
  }
  for (int s = 0; s < k; ++s) gate[s] = renorm ? (P[idx[s]] / den) : P[idx[s]];
}

// ---------------------------------------------------------------- Eq.8-10: window similarity
float norm_canon(const float* v, int E) { return std::sqrt(dot_canon(v, v, E)); }

// Mean-form (Eq.9-10): cosine of each row to the window mean, averaged.
float window_sim_mean(const float* const* rows, int w, int E) {
  if (w == 1) return 1.0f;
  std::vector<float> mean(E);
  for (int e = 0; e < E; ++e) {
    float acc = rows[0][e];
    for (int a = 1; a < w; ++a) acc = acc + rows[a][e];
    mean[e] = acc / (float)w;
  }
  float nm = norm_canon(mean.data(), E);
  float acc = 0.0f;
  for (int a = 0; a < w; ++a) {
    float c = dot_canon(rows[a], mean.data(), E) / (norm_canon(rows[a], E) * nm);
    acc = acc + c;
  }
  return acc / (float)w;
}

// Exact form (Eq.8): mean cosine over all pairs b < a.
float window_sim_pairs(const float* const* rows, int w, int E) {
  if (w == 1) return 1.0f;
  float acc = 0.0f;
  for (int a = 1; a < w; ++a)
    for (int b = 0; b < a; ++b) {
      float c = dot_canon(rows[a], rows[b], E) / (norm_canon(rows[a], E) * norm_canon(rows[b], E));
      acc = acc + c;
    }
  return acc / (float)(w * (w - 1) / 2);
}

// ---------------------------------------------------------------- expert FFN (Eq.4's FFN_j)
// y = W_d * round_dtype( silu(W_g x) .* (W_u x) ), SwiGLU with three matrices and no biases
// (the 6*H*S_m flop count of App. E).  fp64 throughout except the one storage rounding of h.
void ffn_row(const float* x, const float* Wg, const float* Wu, const float* Wd, int d, int F,
             int is_bf16, double* y /*[d], accumulated into*/) {
  std::vector<double> h(F);
  for (int f = 0; f < F; ++f) {
    double g = 0.0, u = 0.0;
    const float* wg = Wg + (size_t)f * d;
    const float* wu = Wu + (size_t)f * d;
    for (int c = 0; c < d; ++c) {
      g += (double)wg[c] * (double)x[c];
      u += (double)wu[c] * (double)x[c];
    }
    double act = g / (1.0 + std::exp(-g)) * u;
    h[f] = (double)round_store(act, is_bf16);
  }
  for (int c = 0; c < d; ++c) {
    const float* wd = Wd + (size_t)c * F;
    double acc = 0.0;
    for (int f = 0; f < F; ++f) acc += (double)wd[f] * h[f];
    y[c] += acc;
  }
}

struct Win { float C; float A; int first; int w; int idx; };

}  // namespace

extern "C" {

// -------- scalar probes of the canonical primitives (for the pin tests)
float orc_exp_canon(float x) { return exp_canon(x); }
float orc_sum_canon(const float* v, int n) { return sum_canon(v, n); }
float orc_dot_canon(const float* a, const float* b, int n) { return dot_canon(a, b, n); }
float orc_dot_seq(const float* a, const float* b, int n) { return dot_seq(a, b, n); }
float orc_round_store(double v, int is_bf16) { return round_store(v, is_bf16); }

// -------- Eq.1-3, Eq.5: route every token.
// probs [T,E] fp32 (all rows), topk_idx/topk_gate [T,Kmax] with Kmax = max(k_text,k_visual),
// pads -1 / 0.  probs_f64 (nullable) receives the fp64 shadow.
int orc_route(const float* x, const uint8_t* is_visual, int T, int d, int E,
              const float* router_w, const float* router_bias, int k_text, int k_visual,
              int renormalize, float* probs, int32_t* topk_idx, float* topk_gate,
              double* probs_f64) {
  if (k_text < 0 || k_visual < 0 || k_text > E || k_visual > E) return -1;
  int Kmax = std::max(k_text, k_visual);
#pragma omp parallel for schedule(dynamic, 16)
  for (int t = 0; t < T; ++t) {
    route_probs_row(x + (size_t)t * d, d, E, router_w, router_bias, probs + (size_t)t * E);
    if (probs_f64)
      route_probs_row_f64(x + (size_t)t * d, d, E, router_w, router_bias, probs_f64 + (size_t)t * E);
    int k = is_visual[t] ? k_visual : k_text;
    if (Kmax > 0)
      topk_gates_row(probs + (size_t)t * E, E, k, Kmax, renormalize,
                     topk_idx + (size_t)t * Kmax, topk_gate + (size_t)t * Kmax);
  }
  return 0;
}

// -------- the same with a selection strategy for tokens whose k is below k_base (see
// select_gates_row); tokens with k >= k_base are routed as in orc_route.
uint64_t orc_splitmix64_nth(uint64_t seed, uint64_t n) { return splitmix64_nth(seed, n); }

int orc_route_select(const float* x, const uint8_t* is_visual, int T, int d, int E,
                     const float* router_w, const float* router_bias, int k_text, int k_visual,
                     int renormalize, int strategy, int k_base, uint64_t seed, float* probs,
                     int32_t* topk_idx, float* topk_gate) {
  if (k_text < 0 || k_visual < 0 || k_text > E || k_visual > E) return -1;
  if (strategy < 0 || strategy > 2 || k_base < 0 || k_base > E || k_base > 16) return -1;
  int Kmax = std::max(k_text, k_visual);
#pragma omp parallel for schedule(dynamic, 16)
  for (int t = 0; t < T; ++t) {
    const float* P = probs + (size_t)t * E;
    route_probs_row(x + (size_t)t * d, d, E, router_w, router_bias, probs + (size_t)t * E);
    int k = is_visual[t] ? k_visual : k_text;
    if (Kmax == 0) continue;
    if (k < k_base)
      select_gates_row(P, E, k, k_base, strategy, seed, t, Kmax, renormalize, topk_idx + (size_t)t * Kmax,
                       topk_gate + (size_t)t * Kmax);
    else
      topk_gates_row(P, E, k, Kmax, renormalize, topk_idx + (size_t)t * Kmax, topk_gate + (size_t)t * Kmax);
  }
  return 0;
}

// -------- Sec. 3.2.2: number of windows per sequence, n = ceil(N_v / W); returns the total.
int orc_window_counts(const uint8_t* is_visual, const int32_t* cu_seqlens, int B, int W,
                      int32_t* win_offsets /*[B+1]*/) {
  win_offsets[0] = 0;
  for (int b = 0; b < B; ++b) {
    int nv = 0;
    for (int t = cu_seqlens[b]; t < cu_seqlens[b + 1]; ++t) nv += is_visual[t] ? 1 : 0;
    win_offsets[b + 1] = win_offsets[b] + (nv + W - 1) / W;
  }
  return win_offsets[B];
}

// -------- Sec. 3.2.1-3.2.3 and the drop rule that follows Table 1: prune visual tokens.
//  1. per sequence, visual tokens in position order; windows of W consecutive visual tokens
//     (the last one may be shorter; a 1-token window has similarity 1);
//  2. S_i by Eq.10 (sim_mode 0) or Eq.8 (sim_mode 1) on the canonical fp32 routing rows;
//  3. if attn (per-token importance, Eq.7) is given: A_i = sum over the window, divided by the
//     sequence's max A (Eq.11-12); C_i = alpha*S_i - (1-alpha)*A_i (Eq.13).  Without attn,
//     A = 0 and C_i = S_i exactly;
//  4. budget: eta = floor(r*N_v + 0.5) in fp64, clamped to [min(1,N_v), N_v]; eps = N_v - eta;
//  5. drop: walk windows in the order (A ascending, C descending, index ascending); drop whole
//     windows while they fit in the remaining budget u; the first window that does not fit
//     loses its last u tokens; then stop.  Exactly eta visual tokens survive;
//  6. kept_idx = ascending global indices of all text tokens and surviving visual tokens;
//     new_cu_seqlens counts them per sequence.
// scores_out (nullable) receives C per window, sequences concatenated.
// Window merging (Sec. 3.2.3, Eq.14-18), gamma > 0, between steps 4 and 5:
//  4a. at most m = floor(eta*gamma) windows are merged (Eq.14; the product is not an integer in
//      general, the floor is this build's reading).  Walk the windows in the order (C descending,
//      index ascending) -- the highest redundancy scores, Eq.15; a window of w >= 2 tokens is merged
//      if the w-1 tokens this removes still fit in the budget u (u starts at eps, u -= w-1), until m
//      windows are merged or the list ends.  (The paper's text subtracts the number of merges from
//      eps; its derivation of the largest useful gamma needs every merge to remove W-1 tokens,
//      which is the accounting used here.)
//  4b. a merged window is replaced by ONE token at the position of its first token (the paper keeps
//      the positions of merged tokens): the mean of its tokens (Eq.16-17, with the window's real size
//      where the paper writes W), rescaled to the largest token norm of the window (Eq.18);
//  5.  the drop walk then runs over the windows that were not merged, with the budget left.
// x_in [T,d] (values already rounded to the storage type) is needed iff gamma > 0; is_merged
// [kept] and x_merged [kept,d] (nullable) receive, per kept position, whether it is a merged token
// and the layer input row after merging (rounded once to the storage type).
// Returns the number of kept tokens, or <0 on bad arguments.
int orc_prune(const float* probs, const uint8_t* is_visual, const int32_t* cu_seqlens, int B,
              int T, int E, float retention, int W, float alpha, float gamma, int sim_mode,
              const float* attn, int32_t* kept_idx, int32_t* new_cu_seqlens, float* scores_out,
              const float* x_in, int d, int is_bf16, uint8_t* is_merged, float* x_merged, int merge_mean) {
  if (W < 1 || !(retention > 0.0f) || retention > 1.0f || !(gamma >= 0.0f) || gamma >= 1.0f) return -1;
  if (gamma > 0.0f && !x_in) return -1;
  if (cu_seqlens[B] != T) return -1;
  std::vector<char> keep(T, 1);
  std::vector<int> merge_w(T, 0);   // at the first token of a merged window: the window's size
  int score_base = 0;
  for (int b = 0; b < B; ++b) {
    std::vector<int> vis;
    for (int t = cu_seqlens[b]; t < cu_seqlens[b + 1]; ++t)
      if (is_visual[t]) vis.push_back(t);
    int Nv = (int)vis.size();
    int n = (Nv + W - 1) / W;
    std::vector<Win> win(n);
    for (int i = 0; i < n; ++i) {
      int first = i * W, w = std::min(W, Nv - first);
      std::vector<const float*> rows(w);
      for (int a = 0; a < w; ++a) rows[a] = probs + (size_t)vis[first + a] * E;
      float S = sim_mode ? window_sim_pairs(rows.data(), w, E) : window_sim_mean(rows.data(), w, E);
      float A = 0.0f;
      if (attn)
        for (int a = 0; a < w; ++a) A = A + attn[vis[first + a]];
      win[i] = Win{S, A, first, w, i};
    }
    if (attn) {
      float mx = 0.0f;
      for (int i = 0; i < n; ++i) mx = (win[i].A > mx) ? win[i].A : mx;
      for (int i = 0; i < n; ++i) {
        if (mx > 0.0f) win[i].A = win[i].A / mx;
        float t1 = alpha * win[i].C;
        float t2 = (1.0f - alpha) * win[i].A;
        win[i].C = t1 - t2;
      }
    }
    if (scores_out)
      for (int i = 0; i < n; ++i) scores_out[score_base + i] = win[i].C;
    score_base += n;

    int eta = (int)std::floor((double)retention * (double)Nv + 0.5);
    eta = std::max(std::min(1, Nv), std::min(eta, Nv));
    int u = Nv - eta;
    std::vector<char> merged(n, 0);
    if (gamma > 0.0f) {
      const int m = (int)std::floor((double)eta * (double)gamma);
      std::vector<Win> by_score(win);
      std::stable_sort(by_score.begin(), by_score.end(), [](const Win& p, const Win& q) {
        if (p.C != q.C) return p.C > q.C;
        return p.idx < q.idx;
      });
      int cnt = 0;
      for (int j = 0; j < n && cnt < m; ++j) {
        const Win& wj = by_score[j];
        if (wj.w >= 2 && wj.w - 1 <= u) {
          merged[wj.idx] = 1;
          merge_w[vis[wj.first]] = wj.w;
          for (int a = 1; a < wj.w; ++a) keep[vis[wj.first + a]] = 0;
          u -= wj.w - 1;
          ++cnt;
        }
      }
    }
    std::vector<Win> order;
    for (int i = 0; i < n; ++i)
      if (!merged[i]) order.push_back(win[i]);
    std::stable_sort(order.begin(), order.end(), [](const Win& p, const Win& q) {
      if (p.A != q.A) return p.A < q.A;
      if (p.C != q.C) return p.C > q.C;
      return p.idx < q.idx;
    });
    for (int j = 0; j < (int)order.size() && u > 0; ++j) {
      const Win& wj = order[j];
      if (wj.w <= u) {
        for (int a = 0; a < wj.w; ++a) keep[vis[wj.first + a]] = 0;
        u -= wj.w;
      } else {
        for (int a = wj.w - u; a < wj.w; ++a) keep[vis[wj.first + a]] = 0;
        u = 0;
      }
    }
  }
  int nk = 0;
  new_cu_seqlens[0] = 0;
  for (int b = 0; b < B; ++b) {
    // the visual tokens after t in its sequence, for the members of a merged window
    std::vector<int> vis;
    for (int t = cu_seqlens[b]; t < cu_seqlens[b + 1]; ++t)
      if (is_visual[t]) vis.push_back(t);
    size_t vpos = 0;
    for (int t = cu_seqlens[b]; t < cu_seqlens[b + 1]; ++t) {
      const size_t my_v = vpos;
      if (is_visual[t]) ++vpos;
      if (!keep[t]) continue;
      if (is_merged) is_merged[nk] = merge_w[t] > 0 ? 1 : 0;
      if (x_merged && x_in) {
        float* out = x_merged + (size_t)nk * d;
        if (merge_w[t] == 0) {
          for (int c = 0; c < d; ++c) out[c] = x_in[(size_t)t * d + c];
        } else {
          const int w = merge_w[t];
          std::vector<double> mean(d, 0.0);
          double max_norm = 0.0;
          for (int a = 0; a < w; ++a) {
            const float* row = x_in + (size_t)vis[my_v + a] * d;
            double nn = 0.0;
            for (int c = 0; c < d; ++c) {
              mean[c] += (double)row[c];
              nn += (double)row[c] * (double)row[c];
            }
            max_norm = std::max(max_norm, std::sqrt(nn));
          }
          double mn = 0.0;
          for (int c = 0; c < d; ++c) {
            mean[c] /= (double)w;
            mn += mean[c] * mean[c];
          }
          mn = std::sqrt(mn);
          // merge_mean: the plain arithmetic mean the paper compares MLERP with (merge-method ablation)
          const double scale = merge_mean ? 1.0 : (mn > 0.0 ? max_norm / mn : 0.0);
          for (int c = 0; c < d; ++c) out[c] = round_store(mean[c] * scale, is_bf16);
        }
      }
      kept_idx[nk++] = t;
    }
    new_cu_seqlens[b + 1] = nk;
  }
  return nk;
}

// -------- permutation by expert (dispatch order; not in the paper, fixed by this build):
// rows = all (kept position p, slot s) with topk_idx >= 0, sorted by (expert asc, p asc).
// expert_offsets [E+1] = exclusive scan of per-expert counts; perm_src[row] = p;
// inv_perm[p*Kmax+s] = row (or -1).  kept_idx NULL = all tokens kept.  Returns M.
int orc_permute(const int32_t* topk_idx, int Kmax, const int32_t* kept_idx, int n_kept, int E,
                int32_t* expert_offsets, int32_t* perm_src, int32_t* inv_perm) {
  std::vector<int> count(E, 0);
  for (int p = 0; p < n_kept; ++p) {
    int t = kept_idx ? kept_idx[p] : p;
    for (int s = 0; s < Kmax; ++s) {
      int e = topk_idx[(size_t)t * Kmax + s];
      inv_perm[(size_t)p * Kmax + s] = -1;
      if (e >= 0) count[e]++;
    }
  }
  expert_offsets[0] = 0;
  for (int e = 0; e < E; ++e) expert_offsets[e + 1] = expert_offsets[e] + count[e];
  std::vector<int> cursor(expert_offsets, expert_offsets + E);
  for (int p = 0; p < n_kept; ++p) {
    int t = kept_idx ? kept_idx[p] : p;
    for (int s = 0; s < Kmax; ++s) {
      int e = topk_idx[(size_t)t * Kmax + s];
      if (e < 0) continue;
      int row = cursor[e]++;
      perm_src[row] = p;
      inv_perm[(size_t)p * Kmax + s] = row;
    }
  }
  return expert_offsets[E];
}

// -------- routed expert FFN on the permuted rows: y[row] = FFN_e(x[token(perm_src[row])]).
// y is fp64 [M, d] (not rounded).  rows_sel (nullable) restricts the work to the listed rows.
int orc_expert_ffn(const float* x, const int32_t* kept_idx, const int32_t* expert_offsets,
                   const int32_t* perm_src, int E, int d, int F, int is_bf16,
                   const float* w_gate, const float* w_up, const float* w_down,
                   const int32_t* rows_sel, int n_rows_sel, double* y) {
  int M = expert_offsets[E];
  std::vector<int> row_expert(M);
  for (int e = 0; e < E; ++e)
    for (int r = expert_offsets[e]; r < expert_offsets[e + 1]; ++r) row_expert[r] = e;
  int n = rows_sel ? n_rows_sel : M;
#pragma omp parallel for schedule(dynamic, 1)
  for (int i = 0; i < n; ++i) {
    int r = rows_sel ? rows_sel[i] : i;
    int e = row_expert[r];
    int p = perm_src[r];
    int t = kept_idx ? kept_idx[p] : p;
    double* yr = y + (size_t)r * d;
    for (int c = 0; c < d; ++c) yr[c] = 0.0;
    ffn_row(x + (size_t)t * d, w_gate + (size_t)e * F * d, w_up + (size_t)e * F * d,
            w_down + (size_t)e * d * F, d, F, is_bf16, yr);
  }
  return 0;
}

// -------- shared experts (first sum of Eq.4): y_shared[p] = sum_i FFN^s_i(x[token(p)]), fp64.
int orc_shared_ffn(const float* x, const int32_t* kept_idx, int n_kept, int d, int n_shared,
                   int F_shared, int is_bf16, const float* ws_gate, const float* ws_up,
                   const float* ws_down, const int32_t* pos_sel, int n_pos_sel, double* y_shared) {
  int n = pos_sel ? n_pos_sel : n_kept;
#pragma omp parallel for schedule(dynamic, 1)
  for (int i = 0; i < n; ++i) {
    int p = pos_sel ? pos_sel[i] : i;
    int t = kept_idx ? kept_idx[p] : p;
    double* yr = y_shared + (size_t)p * d;
    for (int c = 0; c < d; ++c) yr[c] = 0.0;
    for (int s = 0; s < n_shared; ++s)
      ffn_row(x + (size_t)t * d, ws_gate + (size_t)s * F_shared * d, ws_up + (size_t)s * F_shared * d,
              ws_down + (size_t)s * d * F_shared, d, F_shared, is_bf16, yr);
  }
  return 0;
}

// -------- Eq.4: out[p] = (residual x[token(p)]) + y_shared[p] + sum_s gate[t,s] * y[inv_perm[p,s]],
// fp64, rounded once to the storage dtype.  out [n_kept, d] fp32 container; out_f64 nullable.
int orc_combine(const double* y, const double* y_shared, const int32_t* inv_perm,
                const float* topk_gate, const int32_t* kept_idx, int n_kept, int Kmax, int d,
                const float* residual, int is_bf16, const int32_t* pos_sel, int n_pos_sel,
                float* out, double* out_f64) {
  int n = pos_sel ? n_pos_sel : n_kept;
#pragma omp parallel for
  for (int i = 0; i < n; ++i) {
    int p = pos_sel ? pos_sel[i] : i;
    int t = kept_idx ? kept_idx[p] : p;
    for (int c = 0; c < d; ++c) {
      double acc = residual ? (double)residual[(size_t)t * d + c] : 0.0;
      if (y_shared) acc += y_shared[(size_t)p * d + c];
      for (int s = 0; s < Kmax; ++s) {
        int row = inv_perm[(size_t)p * Kmax + s];
        if (row >= 0) acc += (double)topk_gate[(size_t)t * Kmax + s] * y[(size_t)row * d + c];
      }
      out[(size_t)p * d + c] = round_store(acc, is_bf16);
      if (out_f64) out_f64[(size_t)p * d + c] = acc;
    }
  }
  return 0;
}

// -------- Eq.4 evaluated directly for selected kept positions, without the permutation:
// out[i] = residual + sum_shared FFN^s(x_t) + sum_s gate[t,s] FFN_{idx[t,s]}(x_t).
// Used to check sampled outputs at sizes where the whole layer is too slow on the CPU.
int orc_token_outputs(const float* x, const int32_t* tokens, int n_tokens, int d, int E, int F,
                      int n_shared, int F_shared, int is_bf16, int Kmax,
                      const int32_t* topk_idx, const float* topk_gate,
                      const float* w_gate, const float* w_up, const float* w_down,
                      const float* ws_gate, const float* ws_up, const float* ws_down,
                      int add_residual, float* out /*[n_tokens,d]*/, double* out_f64) {
  (void)E;
#pragma omp parallel for schedule(dynamic, 1)
  for (int i = 0; i < n_tokens; ++i) {
    int t = tokens[i];
    const float* xt = x + (size_t)t * d;
    std::vector<double> acc(d, 0.0), y(d);
    if (add_residual)
      for (int c = 0; c < d; ++c) acc[c] = (double)xt[c];
    for (int s = 0; s < n_shared; ++s) {
      std::fill(y.begin(), y.end(), 0.0);
      ffn_row(xt, ws_gate + (size_t)s * F_shared * d, ws_up + (size_t)s * F_shared * d,
              ws_down + (size_t)s * d * F_shared, d, F_shared, is_bf16, y.data());
      for (int c = 0; c < d; ++c) acc[c] += y[c];
    }
    for (int s = 0; s < Kmax; ++s) {
      int e = topk_idx[(size_t)t * Kmax + s];
      if (e < 0) continue;
      std::fill(y.begin(), y.end(), 0.0);
      ffn_row(xt, w_gate + (size_t)e * F * d, w_up + (size_t)e * F * d, w_down + (size_t)e * d * F,
              d, F, is_bf16, y.data());
      double g = (double)topk_gate[(size_t)t * Kmax + s];
      for (int c = 0; c < d; ++c) acc[c] += g * y[c];
    }
    for (int c = 0; c < d; ++c) {
      out[(size_t)i * d + c] = round_store(acc[c], is_bf16);
      if (out_f64) out_f64[(size_t)i * d + c] = acc[c];
    }
  }
  return 0;
}

// -------- analysis statistics of the paper (diagnostics; they feed no decision of the layer).
//
// Fig. 1: routing similarity of adjacent tokens -- Eq.8 on a two-token window: the cosine of the
// routing-probability rows of tokens t and t+1.  A pair counts when both tokens lie in the same
// sequence and have the same modality (the paper compares consecutive visual tokens with
// consecutive text tokens; pairs across a modality switch belong to neither curve).
// pair_sim [T]: cosine for the pair (t, t+1), -2 where t starts no pair; mean/count [2]: index 0
// text pairs, 1 visual pairs (mean 0 when there is no pair).
int orc_adjacent_similarity(const float* probs, const uint8_t* is_visual, const int32_t* cu_seqlens, int B,
                            int T, int E, float* pair_sim, double* mean, int32_t* count) {
  double sum[2] = {0.0, 0.0};
  count[0] = count[1] = 0;
  for (int t = 0; t < T; ++t) pair_sim[t] = -2.0f;
  for (int b = 0; b < B; ++b) {
    for (int t = cu_seqlens[b]; t + 1 < cu_seqlens[b + 1]; ++t) {
      const int m = is_visual[t] ? 1 : 0;
      if ((is_visual[t + 1] ? 1 : 0) != m) continue;
      const float* a = probs + (size_t)t * E;
      const float* c = a + E;
      double ab = 0.0, aa = 0.0, cc = 0.0;
      for (int e = 0; e < E; ++e) {
        ab += (double)a[e] * c[e];
        aa += (double)a[e] * a[e];
        cc += (double)c[e] * c[e];
      }
      const double den = std::sqrt(aa) * std::sqrt(cc);
      const double cosv = den > 0.0 ? ab / den : 0.0;
      pair_sim[t] = (float)cosv;
      sum[m] += cosv;
      count[m] += 1;
    }
  }
  for (int m = 0; m < 2; ++m) mean[m] = count[m] ? sum[m] / count[m] : 0.0;
  return 0;
}

// App. C.1: magnitude stability of expert outputs.  l = Euclidean norm of every expert-output row
// (before the gate-weighted fusion); per modality mu, sigma (population), CV = sigma/mu and
// V = 1/(1+CV).  row_is_visual [M]; row_norm [M] out (nullable); stats [2][4] = {mu, sigma, CV, V}
// for text (0) and vision (1); a modality without rows, or with mu = 0, reports CV = 0, V = 1.
int orc_magnitude_stability(const float* y, int M, int d, const uint8_t* row_is_visual, float* row_norm,
                            double* stats) {
  double s1[2] = {0, 0}, s2[2] = {0, 0};
  long n[2] = {0, 0};
  std::vector<double> norms(M);
  for (int r = 0; r < M; ++r) {
    double q = 0.0;
    for (int c = 0; c < d; ++c) q += (double)y[(size_t)r * d + c] * y[(size_t)r * d + c];
    norms[r] = std::sqrt(q);
    if (row_norm) row_norm[r] = (float)norms[r];
    const int m = row_is_visual[r] ? 1 : 0;
    s1[m] += norms[r];
    n[m] += 1;
  }
  for (int m = 0; m < 2; ++m) {
    const double mu = n[m] ? s1[m] / n[m] : 0.0;
    for (int r = 0; r < M; ++r)
      if ((row_is_visual[r] ? 1 : 0) == m) s2[m] += (norms[r] - mu) * (norms[r] - mu);
    const double sigma = n[m] ? std::sqrt(s2[m] / n[m]) : 0.0;
    const double cv = mu > 0.0 ? sigma / mu : 0.0;
    stats[m * 4 + 0] = mu;
    stats[m * 4 + 1] = sigma;
    stats[m * 4 + 2] = cv;
    stats[m * 4 + 3] = 1.0 / (1.0 + cv);
  }
  return 0;
}

// cosine of the angle between corresponding rows of two [n,d] tensors (the measured angle between
// the layer output with K experts and with m experts, App. C); 0 where a row is all zero.
int orc_row_cosine(const float* a, const float* b, int n, int d, float* out) {
  for (int r = 0; r < n; ++r) {
    double ab = 0.0, aa = 0.0, bb = 0.0;
    for (int c = 0; c < d; ++c) {
      const double u = a[(size_t)r * d + c], v = b[(size_t)r * d + c];
      ab += u * v;
      aa += u * u;
      bb += v * v;
    }
    const double den = std::sqrt(aa) * std::sqrt(bb);
    out[r] = (float)(den > 0.0 ? ab / den : 0.0);
  }
  return 0;
}

// App. C: the angle predicted for orthonormal expert outputs, cos(theta) = sqrt(sum_{i<=m} a_i^2 /
// sum_{i<=K} a_i^2), from a token's K gates in descending order (a common scale cancels, so the
// gates may be normalised or not); rows whose first K entries are not all positive report 0.
int orc_gate_cosine(const float* gates, int T, int K, int m, float* out) {
  if (m < 0 || m > K) return -1;
  for (int t = 0; t < T; ++t) {
    double top = 0.0, all = 0.0;
    bool ok = K > 0;
    for (int i = 0; i < K; ++i) {
      const double a = gates[(size_t)t * K + i];
      if (!(a > 0.0)) ok = false;
      all += a * a;
      if (i < m) top += a * a;
    }
    out[t] = ok ? (float)std::sqrt(top / all) : 0.0f;
  }
  return 0;
}

int orc_num_threads(void) {
  int n = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp master
    n = omp_get_num_threads();
  }
#endif
  return n;
}

}  // extern "C"
