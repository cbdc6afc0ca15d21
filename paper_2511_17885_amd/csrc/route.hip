// Router: logits (Eq.1), softmax (Eq.2), modality-dependent top-k (Eq.3), gates (Eq.5).
//
// Every float here feeds a decision (which experts a token uses), so the arithmetic follows a
// fixed order that any IEEE-754 machine reproduces bit for bit.  This file is compiled with
// floating-point contraction off; fused multiply-adds appear only where fmaf is written.
//
//  logit:  the plain fp32 dot product in index order, acc = fmaf(x[k], w[k], acc) for k = 0..d-1
//          from +0.  The fp32 matrix-core instruction v_mfma_f32_16x16x4_f32 performs exactly this
//          chain (its four k per instruction are applied in ascending order, one rounding each;
//          verified bit for bit on gfx950), so a 16-token x 16-expert tile of logits costs one
//          instruction per four k and the chain is reproduced by a scalar fmaf loop anywhere else.
//  exp:    range reduction by rint(x*log2 e) with a two-constant ln 2, degree-7 Taylor polynomial
//          in Horner form, exact scaling by 2^n; flushed to 0 once 2^n leaves the normal range.
//  sum:    lane l adds q[l], q[l+64], ... in that order from +0, then a 6-level xor butterfly
//          (p[l] += p[l xor s], s = 32,16,..,1).
//
// Work split: a 256-thread block owns 16 tokens; its 4 wavefronts split the experts (NB blocks of
// 16 experts each).  Token rows are staged through LDS in 128-wide k chunks, widened to fp32 and
// de-interleaved so that a lane fetches the operands of four consecutive MFMAs with one 16-byte
// LDS read; router weights come from a private fp32 copy that fmoe_set_weights lays out in
// exactly the per-lane order the MFMA consumes (one coalesced 16-byte global load per four
// MFMAs); several chunks of both are kept in flight in registers.  Logits meet in LDS, then each wavefront does softmax /
// top-k for four tokens with lanes mapped to experts.

#include <type_traits>

#include "common.h"
#include "prune_dev.h"

namespace {

typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef float fx4_t __attribute__((ext_vector_type(4)));

constexpr int TOKB = 16;           // tokens per block
constexpr int KC = 128;            // k per LDS chunk
constexpr int NG = KC / 16;        // groups of four MFMAs per chunk
constexpr int RS = KC / 4 + 4;     // LDS row stride in floats (rows = kq*16 + token)

// k groups (of 16) in the packed router weights: d rounded up to whole chunks, then to a multiple of
// 5 chunks or 4 chunks (the prefetch depths the kernel is instantiated with), whichever is larger
__host__ __device__ inline int router_groups(int d) {
  const int chunks = (d + KC - 1) / KC;
  const int p4 = (chunks + 3) / 4 * 4, p5 = (chunks + 4) / 5 * 5;
  return (p4 > p5 ? p4 : p5) * NG;
}

__device__ __forceinline__ float wave_sum_butterfly(float p) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) p = p + __shfl_xor(p, s, 64);
  return p;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) {
    float o = __shfl_xor(v, s, 64);
    v = (o > v) ? o : v;
  }
  return v;
}

// Maximum over the 64 lanes, returned in every lane.  Inside a row of 16 lanes: xor-1 and xor-2 quad
// permutes, then the half-row and full-row mirrors (each step pairs lanes holding different partial
// maxima); across the four rows: one lane read per row.
__device__ __forceinline__ float wave_max_all(float v) {
  auto step = [](float x, auto ctrl) {
    const int o = __builtin_amdgcn_update_dpp(0, __float_as_int(x), decltype(ctrl)::value, 0xf, 0xf, false);
    const float y = __int_as_float(o);
    return (y > x) ? y : x;
  };
  v = step(v, std::integral_constant<int, 0xB1>{});    // quad_perm [1,0,3,2]
  v = step(v, std::integral_constant<int, 0x4E>{});    // quad_perm [2,3,0,1]
  v = step(v, std::integral_constant<int, 0x141>{});   // row_half_mirror
  v = step(v, std::integral_constant<int, 0x140>{});   // row_mirror
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
  const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
  const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
  const float a = (r1 > r0) ? r1 : r0, b = (r3 > r2) ? r3 : r2;
  return (b > a) ? b : a;
}

__device__ __forceinline__ float exp_fixed(float x) {
  const float kLog2e = 0x1.715476p+0f;
  const float kLn2Hi = 0x1.62e400p-1f;
  const float kLn2Lo = 0x1.7f7d1cp-20f;
  float n = rintf(x * kLog2e);
  float r = fmaf(-n, kLn2Hi, x);
  r = fmaf(-n, kLn2Lo, r);
  float p = 0x1.a01a02p-13f;
  p = fmaf(p, r, 0x1.6c16c2p-10f);
  p = fmaf(p, r, 0x1.111112p-7f);
  p = fmaf(p, r, 0x1.555556p-5f);
  p = fmaf(p, r, 0x1.555556p-3f);
  p = fmaf(p, r, 0.5f);
  p = fmaf(p, r, 1.0f);
  p = fmaf(p, r, 1.0f);
  if (!(n >= -125.0f)) return 0.0f;
  float scale = __uint_as_float((uint32_t)((int)n + 127) << 23);
  return p * scale;
}

// Private router-weight layout: for expert block eb (16 experts) and k group g (16 k), lane l
// holds the float4 { w[eb*16 + l%16][16g + 4j + l/16] : j = 0..3 } at ((eb*G + g)*64 + l).
// Experts >= E and k >= d are zero (a zero product leaves the chain's value unchanged); G covers
// d rounded up to whole 128-wide chunks, so the kernel's loads need no bounds predicate.
template <typename WT>
__global__ void pack_router_kernel(const WT* __restrict__ w, float* __restrict__ wp, int E, int d,
                                   int Eb, int G) {
  const size_t n = (size_t)Eb * G * 256;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (size_t)gridDim.x * blockDim.x) {
    const int j = (int)(i & 3), l = (int)((i >> 2) & 63);
    const size_t eg = i >> 8;
    const int g = (int)(eg % G), eb = (int)(eg / G);
    const int e = eb * 16 + (l & 15), k = 16 * g + 4 * j + (l >> 4);
    wp[i] = (e < E && k < d) ? to_f32(w[(size_t)e * d + k]) : 0.0f;
  }
}

template <typename XT> struct XStage;
template <> struct XStage<bf16_t> {
  static constexpr int UNITS = 1;  // 16 tokens x 128 k / 8 per 16-byte load / 256 threads
  u32x4_t v[UNITS];
  // Unpredicated: a token past T re-reads the last token (its logits are never used) and k past d
  // re-reads the row's last chunk (the packed weights are zero there).
  __device__ __forceinline__ void load(const bf16_t* x, int t0, int T, int d, int c0, int tid) {   // t0: the tile's first token
    const int tok = tid >> 4, cu = tid & 15;
    int k = c0 + 8 * cu, t = t0 + tok;
    k = k < d ? k : d - 8;
    t = t < T ? t : T - 1;
    v[0] = *reinterpret_cast<const u32x4_t*>(x + (size_t)t * d + k);
  }
  __device__ __forceinline__ void store(float* xs, int tid) const {
    const int tok = tid >> 4, cu = tid & 15;
    const uint32_t w[4] = {v[0][0], v[0][1], v[0][2], v[0][3]};
    float f[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
    // element i of the unit has k = 8cu + i: kq = i%4, step = 2cu + i/4
#pragma unroll
    for (int kq = 0; kq < 4; ++kq)
      *reinterpret_cast<float2*>(&xs[(kq * 16 + tok) * RS + 2 * cu]) = make_float2(f[kq], f[kq + 4]);
  }
};
template <> struct XStage<float> {
  static constexpr int UNITS = 2;  // 16 x 128 / 4 / 256
  fx4_t v[UNITS];
  __device__ __forceinline__ void load(const float* x, int t0, int T, int d, int c0, int tid) {
#pragma unroll
    for (int u = 0; u < UNITS; ++u) {
      const int unit = tid + u * 256;
      const int tok = unit >> 5, cu = unit & 31;
      int k = c0 + 4 * cu, t = t0 + tok;
      k = k < d ? k : d - 4;
      t = t < T ? t : T - 1;
      v[u] = *reinterpret_cast<const fx4_t*>(x + (size_t)t * d + k);
    }
  }
  __device__ __forceinline__ void store(float* xs, int tid) const {
#pragma unroll
    for (int u = 0; u < UNITS; ++u) {
      const int unit = tid + u * 256;
      const int tok = unit >> 5, cu = unit & 31;
      xs[(0 * 16 + tok) * RS + cu] = v[u][0];
      xs[(1 * 16 + tok) * RS + cu] = v[u][1];
      xs[(2 * 16 + tok) * RS + cu] = v[u][2];
      xs[(3 * 16 + tok) * RS + cu] = v[u][3];
    }
  }
};

// Selection-strategy ablation (Sec. 4): which k of a token's k_base highest experts stay active.
struct fmoe_selection {
  int strategy;              // 0 the k highest (the method), 1 k at random, 2 the k lowest
  int k_base;
  unsigned long long seed;
};

// n-th output of the SplitMix64 generator started at `seed` (the key of a candidate position for
// the random strategy)
__device__ __forceinline__ unsigned long long splitmix64_nth(unsigned long long seed, unsigned long long n) {
  unsigned long long z = seed + n * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// TT = token tiles of 16 per block (1 or 2).  With two tiles every wavefront runs two independent
// accumulation chains on the same weight fragments: a logit's own chain keeps its order (so its bits),
// the matrix pipe gets a second instruction to issue while the first chain's next link waits for its
// predecessor, and a token costs half the weight loads.  Taken for large batches, where there are
// enough blocks to fill the chip either way.
template <typename XT, int NB, int PF, bool SEL, int TT>
__global__ __launch_bounds__(256) void route_kernel(
    const XT* __restrict__ x, const fx4_t* __restrict__ wp, const float* __restrict__ bias,
    const uint8_t* __restrict__ is_visual, int T, int d, int E, int Eb, int G, int nch, int k_text,
    int k_visual, int Kmax, int renorm, float* __restrict__ probs, int32_t* __restrict__ topk_idx,
    float* __restrict__ topk_gate, int route_blocks, fmoe_ordinals_job ord, const int32_t* __restrict__ T_dev,
    fmoe_selection selp) {
  __shared__ __align__(16) float xs[TT][64 * RS];
  __shared__ float zs[TT * TOKB][4 * NB * 16 + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if ((int)blockIdx.x >= route_blocks) {   // rider blocks: per-sequence visual ordinals for the pruning stage
    seq_ordinals_block(is_visual, ord.cu, (int)blockIdx.x - route_blocks, T, ord.vis_ord, ord.vis_tok,
                       ord.seq_nv, reinterpret_cast<int*>(&xs[0][0]));
    return;
  }
  const int t0 = blockIdx.x * (TT * TOKB);
  if (T_dev != nullptr) {   // the batch holds fewer tokens than its capacity
    const int Td = *T_dev;
    T = Td < T ? Td : T;
    if (t0 >= T) return;
  }

  f32x4_t acc[TT][NB];
#pragma unroll
  for (int tt = 0; tt < TT; ++tt)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[tt][nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // PF chunks of operands are kept in flight in registers (the block's wavefronts are often alone
  // on their SIMDs, so memory latency has to be covered inside the wavefront)
  fx4_t wbuf[PF][NG][NB];
  XStage<XT> xbuf[PF][TT];
  const fx4_t* wsrc[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    int eb = wave * NB + nb;
    eb = eb < Eb ? eb : Eb - 1;   // expert blocks past E recompute the last one; never read back
    wsrc[nb] = wp + (size_t)eb * G * 64 + lane;
  }
  auto load_chunk = [&](int slot, int c0) {
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) xbuf[slot][tt].load(x, t0 + tt * TOKB, T, d, c0, tid);
#pragma unroll
    for (int gl = 0; gl < NG; ++gl)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) wbuf[slot][gl][nb] = wsrc[nb][(size_t)(c0 / 16 + gl) * 64];
  };
  // nch chunks (a multiple of PF; d is zero-padded up to it in the packed weights).  The loop body
  // is straight-line code with a fixed number of loads per step so that the waits on them can be
  // counted exactly: chunk c is multiplied while chunks c+1 .. c+PF are in flight.
  const int xrow = ((lane >> 4) * 16 + (lane & 15)) * RS;
  auto step = [&](int p) {
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) xbuf[p][tt].store(xs[tt], tid);
    __syncthreads();
#pragma unroll
    for (int gl = 0; gl < NG; ++gl) {
      fx4_t xa[TT];
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) xa[tt] = *reinterpret_cast<const fx4_t*>(&xs[tt][xrow + gl * 4]);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const fx4_t wv = wbuf[p][gl][nb];
#pragma unroll
        for (int q = 0; q < 4; ++q)   // each chain in ascending k; the chains of the tiles alternate
#pragma unroll
          for (int tt = 0; tt < TT; ++tt)
            acc[tt][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[tt][q], wv[q], acc[tt][nb], 0, 0, 0);
      }
    }
  };
#pragma unroll
  for (int p = 0; p < PF; ++p) load_chunk(p, p * KC);
  int c = 0;
  for (; c + PF < nch; c += PF) {
#pragma unroll
    for (int p = 0; p < PF; ++p) {
      step(p);
      load_chunk(p, (c + p + PF) * KC);
      __syncthreads();
    }
  }
#pragma unroll
  for (int p = 0; p < PF; ++p) {
    step(p);
    __syncthreads();
  }

  // accumulator register v of lane l: token 4*(l/16) + v, expert (block)*16 + l%16
#pragma unroll
  for (int tt = 0; tt < TT; ++tt)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int e = (wave * NB + nb) * 16 + (lane & 15);
#pragma unroll
      for (int v = 0; v < 4; ++v) zs[tt * TOKB + 4 * (lane >> 4) + v][e] = acc[tt][nb][v];
    }
  __syncthreads();

  // softmax, top-k and gates: lanes <-> experts (expert e lives in lane e%64, register e/64).
  // The wavefront's four tokens are processed side by side so that the cross-lane reduction
  // chains of different tokens overlap.
  for (int tile = 0; tile < TT; ++tile) {   // four tokens per wavefront at a time
    constexpr int TQ = 4;
    float P[TQ][NB], part[TQ], mx[TQ];
    int tt[TQ];
    bool tv[TQ];
  #pragma unroll
    for (int tq = 0; tq < TQ; ++tq) {
      const int tok = tile * TOKB + wave * TQ + tq;
      tv[tq] = (t0 + tok) < T;
      tt[tq] = tv[tq] ? t0 + tok : T - 1;
      mx[tq] = -INFINITY;
  #pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int e = lane + 64 * i;
        float v = -INFINITY;
        if (e < E) {
          v = zs[tok][e];
          if (bias != nullptr) v = v + bias[e];
        }
        P[tq][i] = v;
        mx[tq] = (v > mx[tq]) ? v : mx[tq];
      }
    }
  #pragma unroll
    for (int s = 32; s >= 1; s >>= 1)
  #pragma unroll
      for (int tq = 0; tq < TQ; ++tq) {
        const float o = __shfl_xor(mx[tq], s, 64);
        mx[tq] = (o > mx[tq]) ? o : mx[tq];
      }
  #pragma unroll
    for (int tq = 0; tq < TQ; ++tq) {
      part[tq] = 0.0f;
  #pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int e = lane + 64 * i;
        float q = 0.0f;
        if (e < E) {
          q = exp_fixed(P[tq][i] - mx[tq]);
          part[tq] = part[tq] + q;
        }
        P[tq][i] = q;
      }
    }
  #pragma unroll
    for (int s = 32; s >= 1; s >>= 1)
  #pragma unroll
      for (int tq = 0; tq < TQ; ++tq) part[tq] = part[tq] + __shfl_xor(part[tq], s, 64);
    // Inside the fused layer (the launch that also carries the ordinal blocks) the probabilities only feed
    // the window scores, which read visual tokens: text rows are not written.
    const bool visual_rows_only = ord.cu != nullptr;
  #pragma unroll
    for (int tq = 0; tq < TQ; ++tq) {
      const bool store_row = probs != nullptr && tv[tq] && (!visual_rows_only || is_visual[tt[tq]] != 0);
  #pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int e = lane + 64 * i;
        P[tq][i] = (e < E) ? P[tq][i] / part[tq] : -1.0f;   // -1 ranks below every probability
        if (store_row && e < E) probs[(size_t)tt[tq] * E + e] = P[tq][i];
      }
    }

    // Top-k as k rounds of "take the largest remaining probability" (ties: lowest expert index), which
    // yields the list in the order (probability desc, index asc) directly.  The maximum over the
    // wavefront is order-free, so it uses the cheap lane-crossing modifiers (two quad permutes, two
    // mirrors) inside a row of 16 lanes and four lane reads across rows.  The four tokens run side by
    // side and a token that needs fewer than Kmax experts idles branch-free.
    float work[TQ][NB];
    int sel[TQ][NB];     // position of this lane's expert in the token's list, -1: not selected
    float den[TQ];
    int kk[TQ];
  #pragma unroll
    for (int tq = 0; tq < TQ; ++tq) {
      kk[tq] = is_visual[tt[tq]] ? k_visual : k_text;
      den[tq] = 0.0f;
  #pragma unroll
      for (int i = 0; i < NB; ++i) {
        work[tq][i] = P[tq][i];
        sel[tq][i] = -1;
      }
    }
    // with a selection strategy a token with k < k_base first lists its k_base candidates
    int kc[TQ];
  #pragma unroll
    for (int tq = 0; tq < TQ; ++tq) kc[tq] = (SEL && kk[tq] < selp.k_base) ? selp.k_base : kk[tq];
    const int rounds = (SEL && selp.k_base > Kmax) ? selp.k_base : Kmax;
    for (int r = 0; r < rounds; ++r) {
  #pragma unroll
      for (int tq = 0; tq < TQ; ++tq) {
        float v = work[tq][0];
  #pragma unroll
        for (int i = 1; i < NB; ++i) v = (work[tq][i] > v) ? work[tq][i] : v;
        const float m = wave_max_all(v);
        const bool active = r < kc[tq];
        bool taken = false;
  #pragma unroll
        for (int i = 0; i < NB; ++i) {   // lowest expert index first: register i holds experts 64i..64i+63
          const unsigned long long eq = __ballot(work[tq][i] == m);
          const int owner = __ffsll((long long)eq) - 1;
          if (active && !taken && lane == owner) {
            sel[tq][i] = r;
            work[tq][i] = -2.0f;
          }
          taken = taken || (eq != 0ull);
        }
        den[tq] = den[tq] + (active ? m : 0.0f);   // list order, sequential (Eq.5)
      }
    }
    if constexpr (SEL) {
      // random strategy: lane 16q + r holds the key of candidate position r of the wavefront's q-th
      // token; a position is kept when fewer than k keys of its token are smaller (ties: lower position)
      unsigned long long random_masks = 0ull;
      if (selp.strategy == 1) {
        const int q = lane >> 4, r = lane & 15;
        const int tq_t = q == 0 ? tt[0] : (q == 1 ? tt[1] : (q == 2 ? tt[2] : tt[3]));
        const int tq_k = q == 0 ? kk[0] : (q == 1 ? kk[1] : (q == 2 ? kk[2] : kk[3]));
        const unsigned long long key = splitmix64_nth(selp.seed, (unsigned long long)tq_t * 16ull + (unsigned long long)r + 1ull);
        int rank = 0;
        for (int o = 0; o < 16; ++o) {
          const int src = (lane & 48) + o;
          const unsigned int lo = (unsigned int)__shfl((int)(unsigned int)key, src, 64);
          const unsigned int hi = (unsigned int)__shfl((int)(unsigned int)(key >> 32), src, 64);
          const unsigned long long ok = ((unsigned long long)hi << 32) | lo;
          rank += (o < selp.k_base && (ok < key || (ok == key && o < r))) ? 1 : 0;
        }
        random_masks = __ballot(r < selp.k_base && rank < tq_k);
      }
  #pragma unroll
      for (int tq = 0; tq < TQ; ++tq) {
        if (kk[tq] >= selp.k_base) continue;   // not reduced: the list stands (uniform over the wavefront)
        const int k = kk[tq];
        unsigned int mask;   // kept candidate positions
        if (selp.strategy == 1) mask = (unsigned int)(random_masks >> (16 * tq)) & 0xffffu;
        else if (selp.strategy == 2) mask = ((1u << k) - 1u) << (selp.k_base - k);
        else mask = (1u << k) - 1u;
  #pragma unroll
        for (int i = 0; i < NB; ++i) {
          const int p = sel[tq][i];
          if (p >= 0) sel[tq][i] = ((mask >> p) & 1u) ? __popc(mask & ((1u << p) - 1u)) : -1;
        }
        float d2 = 0.0f;   // Eq.5 over the kept experts, in list order
        for (int sl = 0; sl < k; ++sl) {
          float v = -1.0f;
  #pragma unroll
          for (int i = 0; i < NB; ++i) v = (sel[tq][i] == sl) ? P[tq][i] : v;
          d2 = d2 + wave_max_all(v);
        }
        den[tq] = d2;
      }
    }
  #pragma unroll
    for (int tq = 0; tq < TQ; ++tq) {
      if (!tv[tq]) continue;
      int32_t* oi = topk_idx + (size_t)tt[tq] * Kmax;
      float* og = topk_gate + (size_t)tt[tq] * Kmax;
  #pragma unroll
      for (int i = 0; i < NB; ++i) {
        if (sel[tq][i] >= 0) {
          oi[sel[tq][i]] = lane + 64 * i;
          og[sel[tq][i]] = renorm ? P[tq][i] / den[tq] : P[tq][i];
        }
      }
      if (lane < Kmax && lane >= kk[tq]) {   // unused tail of the list
        oi[lane] = -1;
        og[lane] = 0.0f;
      }
    }
  }
}

template <typename XT, int NB, int PF, bool TT2 = (NB <= 2)>
int launch_route_t(const fmoe_ctx* ctx, const void* x, const uint8_t* is_visual, int T, float* probs,
                   int32_t* topk_idx, float* topk_gate, const fmoe_ordinals_job& ord, hipStream_t stream, const int32_t* T_dev) {
  const int d = ctx->cfg.d_model, E = ctx->cfg.n_experts;
  const int Eb = (E + 15) / 16, G = router_groups(d);
  const int nch = (((d + KC - 1) / KC + PF - 1) / PF) * PF;   // <= G / NG by construction
  // two token tiles per block once that still leaves every CU several blocks (and only for the default
  // selection strategy and up to 128 experts, where the registers allow it)
  const bool two = TT2 && T >= FMOE_ROUTE_TT2_MIN_TOKENS && ctx->sel_strategy == 0;
  const int per_block = two ? 2 * TOKB : TOKB;
  const int grid = (T + per_block - 1) / per_block;
  fmoe_prof_scope prof(ctx, SLOT_ROUTE, stream);
  const int riders = ord.cu != nullptr ? ord.B : 0;
  const fmoe_selection selp{ctx->sel_strategy, ctx->sel_k_base, ctx->sel_seed};
#define FMOE_ROUTE_LAUNCH(SEL, TT)                                                                              \
  hipLaunchKernelGGL((route_kernel<XT, NB, PF, SEL, TT>), dim3(grid + riders), dim3(256), 0, stream,            \
                     static_cast<const XT*>(x), reinterpret_cast<const fx4_t*>(ctx->router_wp),                 \
                     ctx->router_bias, is_visual, T, d, E, Eb, G, nch, ctx->cfg.k_text, ctx->cfg.k_visual,      \
                     ctx->kmax, ctx->cfg.renormalize, probs, topk_idx, topk_gate, grid, ord, T_dev, selp)
  if (ctx->sel_strategy != 0) FMOE_ROUTE_LAUNCH(true, 1);
  else if constexpr (TT2) { if (two) FMOE_ROUTE_LAUNCH(false, 2); else FMOE_ROUTE_LAUNCH(false, 1); }
  else FMOE_ROUTE_LAUNCH(false, 1);
#undef FMOE_ROUTE_LAUNCH
  FMOE_HIP_CHECK(hipGetLastError());
  return FMOE_OK;
}

template <typename XT>
int launch_route_x(const fmoe_ctx* ctx, const void* x, const uint8_t* is_visual, int T, float* probs,
                   int32_t* topk_idx, float* topk_gate, const fmoe_ordinals_job& ord, hipStream_t stream, const int32_t* T_dev) {
  const int E = ctx->cfg.n_experts;
  const int chunks = (ctx->cfg.d_model + KC - 1) / KC;
  if (E <= 64) {
    if (chunks < 4) return launch_route_t<XT, 1, 1>(ctx, x, is_visual, T, probs, topk_idx, topk_gate, ord, stream, T_dev);
    // Large batches have several blocks per CU to hide memory latency with; two chunks in flight instead of
    // four or five then halve the registers of a wavefront, twice as many wavefronts share a SIMD, and
    // their accumulation chains keep the matrix pipe busier (91 -> 80 us at 22016 tokens).
    if (T >= FMOE_ROUTE_SHALLOW_MIN_TOKENS)
      return launch_route_t<XT, 1, 2>(ctx, x, is_visual, T, probs, topk_idx, topk_gate, ord, stream, T_dev);
    if (chunks % 5 == 0) return launch_route_t<XT, 1, 5>(ctx, x, is_visual, T, probs, topk_idx, topk_gate, ord, stream, T_dev);
    return launch_route_t<XT, 1, 4>(ctx, x, is_visual, T, probs, topk_idx, topk_gate, ord, stream, T_dev);
  }
  if (E <= 128) {
    if (chunks < 2) return launch_route_t<XT, 2, 1>(ctx, x, is_visual, T, probs, topk_idx, topk_gate, ord, stream, T_dev);
    return launch_route_t<XT, 2, 2>(ctx, x, is_visual, T, probs, topk_idx, topk_gate, ord, stream, T_dev);
  }
  return launch_route_t<XT, 4, 1>(ctx, x, is_visual, T, probs, topk_idx, topk_gate, ord, stream, T_dev);
}

}  // namespace

size_t router_pack_floats(const fmoe_ctx* ctx) {
  const int Eb = (ctx->cfg.n_experts + 15) / 16, G = router_groups(ctx->cfg.d_model);
  return (size_t)Eb * G * 256;
}

int launch_pack_router(const fmoe_ctx* ctx, const void* router_w, float* wp, hipStream_t stream) {
  const int E = ctx->cfg.n_experts, d = ctx->cfg.d_model;
  const int Eb = (E + 15) / 16, G = router_groups(d);
  const size_t n = router_pack_floats(ctx);
  const int grid = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
  if (ctx->cfg.dtype == FMOE_BF16)
    hipLaunchKernelGGL(pack_router_kernel<bf16_t>, dim3(grid), dim3(256), 0, stream,
                       static_cast<const bf16_t*>(router_w), wp, E, d, Eb, G);
  else
    hipLaunchKernelGGL(pack_router_kernel<float>, dim3(grid), dim3(256), 0, stream,
                       static_cast<const float*>(router_w), wp, E, d, Eb, G);
  FMOE_HIP_CHECK(hipGetLastError());
  return FMOE_OK;
}

int launch_route(const fmoe_ctx* ctx, const void* x, const uint8_t* is_visual, int T, float* probs,
                 int32_t* topk_idx, float* topk_gate, const fmoe_ordinals_job& ord, hipStream_t stream, const int32_t* T_dev) {
  if (T == 0) return FMOE_OK;
  if (ctx->cfg.dtype == FMOE_BF16)
    return launch_route_x<bf16_t>(ctx, x, is_visual, T, probs, topk_idx, topk_gate, ord, stream, T_dev);
  return launch_route_x<float>(ctx, x, is_visual, T, probs, topk_idx, topk_gate, ord, stream, T_dev);
}
