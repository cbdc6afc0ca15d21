// Router: logits (Eq.1), softmax (Eq.2), modality-dependent top-k (Eq.3), gates (Eq.5).
//
// Every float here feeds a decision (which experts a token uses), so the arithmetic follows a
// fixed order that any IEEE-754 machine reproduces bit for bit.  This file is compiled with
// floating-point contraction off; fused multiply-adds appear only where fmaf is written.
//
//  logit:  the d products of a (token, expert) pair are accumulated by 64 partial sums; element k
//          belongs to partial k mod 64, partials take their elements in ascending k starting
//          from +0 with fmaf, and are then combined by a 6-level butterfly
//          (p[l] += p[l xor s], s = 32,16,..,1).  One wavefront lane owns one partial, so a
//          lane reads a strided set of elements and the butterfly is a cross-lane exchange.
//  exp:    range reduction by rint(x*log2 e) with a two-constant ln 2, degree-7 Taylor polynomial
//          in Horner form, exact scaling by 2^n; flushed to 0 once 2^n leaves the normal range.
//  sum:    lane l adds q[l], q[l+64], ... in that order from +0, then the same butterfly.
//
// Work split: a 256-thread block holds 4 wavefronts; each wavefront owns TOK tokens whose rows
// sit in LDS, sweeps the experts EB at a time keeping TOK*EB partial sums per lane in
// registers, then does softmax / top-k for its tokens with lanes mapped to experts.

#include "common.h"

namespace {

constexpr int kWaves = 4;

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

template <typename XT, int TOK, int EB>
__global__ __launch_bounds__(256) void route_kernel(
    const XT* __restrict__ x, const float* __restrict__ wr, const float* __restrict__ bias,
    const uint8_t* __restrict__ is_visual, int T, int d, int E, int k_text, int k_visual, int Kmax,
    int renorm, float* __restrict__ probs, int32_t* __restrict__ topk_idx,
    float* __restrict__ topk_gate) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  XT* xs = reinterpret_cast<XT*>(smem) + (size_t)wave * TOK * d;                   // [TOK][d]
  float* zs = reinterpret_cast<float*>(smem + (size_t)kWaves * TOK * d * sizeof(XT)) +
              (size_t)wave * TOK * E;                                               // [TOK][E]
  const int t0 = (blockIdx.x * kWaves + wave) * TOK;

  // stage this wavefront's token rows into LDS (rows past T are zero and never written back)
  for (int tok = 0; tok < TOK; ++tok) {
    const int t = t0 + tok;
    for (int k = lane; k < d; k += 64) xs[tok * d + k] = (t < T) ? x[(size_t)t * d + k] : XT(0);
  }
  __builtin_amdgcn_wave_barrier();
  __syncthreads();

  // logits
  for (int e0 = 0; e0 < E; e0 += EB) {
    float acc[TOK][EB];
#pragma unroll
    for (int a = 0; a < TOK; ++a)
#pragma unroll
      for (int i = 0; i < EB; ++i) acc[a][i] = 0.0f;
    for (int k = lane; k < d; k += 64) {
      float xv[TOK];
#pragma unroll
      for (int a = 0; a < TOK; ++a) xv[a] = to_f32(xs[a * d + k]);
#pragma unroll
      for (int i = 0; i < EB; ++i) {
        if (e0 + i < E) {
          const float w = wr[(size_t)(e0 + i) * d + k];
#pragma unroll
          for (int a = 0; a < TOK; ++a) acc[a][i] = fmaf(xv[a], w, acc[a][i]);
        }
      }
    }
#pragma unroll
    for (int a = 0; a < TOK; ++a)
#pragma unroll
      for (int i = 0; i < EB; ++i) {
        float z = wave_sum_butterfly(acc[a][i]);
        if (lane == 0 && e0 + i < E) zs[a * E + e0 + i] = z;
      }
  }
  __syncthreads();

  // softmax, top-k and gates: lanes <-> experts (expert e lives in lane e%64, register e/64)
  for (int tok = 0; tok < TOK; ++tok) {
    const int t = t0 + tok;
    if (t >= T) break;  // uniform per wavefront
    float z[4], q[4];
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = lane + 64 * i;
      z[i] = -INFINITY;
      if (e < E) {
        float v = zs[tok * E + e];
        if (bias != nullptr) v = v + bias[e];
        z[i] = v;
        m = (v > m) ? v : m;
      }
    }
    m = wave_max(m);
    float part = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = lane + 64 * i;
      q[i] = 0.0f;
      if (e < E) {
        q[i] = exp_fixed(z[i] - m);
        part = part + q[i];
      }
    }
    const float denom = wave_sum_butterfly(part);
    float P[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = lane + 64 * i;
      P[i] = q[i] / denom;
      if (probs != nullptr && e < E) probs[(size_t)t * E + e] = P[i];
    }

    const int k = is_visual[t] ? k_visual : k_text;
    unsigned taken = 0;
    int my_e = -1;
    float my_p = 0.0f;
    for (int r = 0; r < k; ++r) {
      float bv = -1.0f;
      int be = 0x7fffffff;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int e = lane + 64 * i;
        if (e < E && !(taken & (1u << i)) && P[i] > bv) {
          bv = P[i];
          be = e;
        }
      }
#pragma unroll
      for (int s = 32; s >= 1; s >>= 1) {
        const float ov = __shfl_xor(bv, s, 64);
        const int oe = __shfl_xor(be, s, 64);
        if (ov > bv || (ov == bv && oe < be)) {
          bv = ov;
          be = oe;
        }
      }
      if ((be & 63) == lane) taken |= 1u << (be >> 6);
      if (lane == r) {
        my_e = be;
        my_p = bv;
      }
    }
    float den = 0.0f;
    for (int r = 0; r < k; ++r) den = den + __shfl(my_p, r, 64);
    if (lane < Kmax) {
      const bool live = lane < k;
      const float g = live ? (renorm ? my_p / den : my_p) : 0.0f;
      topk_idx[(size_t)t * Kmax + lane] = live ? my_e : -1;
      topk_gate[(size_t)t * Kmax + lane] = g;
    }
  }
}

__global__ void widen_bf16_kernel(const bf16_t* __restrict__ src, float* __restrict__ dst, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = bf16_to_f32(src[i]);
}

template <typename XT, int TOK, int EB>
int launch_route_t(const fmoe_ctx* ctx, const void* x, const uint8_t* is_visual, int T, float* probs,
                   int32_t* topk_idx, float* topk_gate, hipStream_t stream) {
  const int d = ctx->cfg.d_model, E = ctx->cfg.n_experts;
  const size_t lds = (size_t)kWaves * TOK * d * sizeof(XT) + (size_t)kWaves * TOK * E * sizeof(float);
  auto kern = route_kernel<XT, TOK, EB>;
  if (lds > 48 * 1024)
    FMOE_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  const int per_block = kWaves * TOK;
  const int grid = (T + per_block - 1) / per_block;
  fmoe_prof_scope prof(ctx, SLOT_ROUTE, stream);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, stream, static_cast<const XT*>(x),
                     ctx->router_w32, ctx->router_bias, is_visual, T, d, E, ctx->cfg.k_text,
                     ctx->cfg.k_visual, ctx->kmax, ctx->cfg.renormalize, probs, topk_idx, topk_gate);
  FMOE_HIP_CHECK(hipGetLastError());
  return FMOE_OK;
}

template <typename XT>
int launch_route_x(const fmoe_ctx* ctx, const void* x, const uint8_t* is_visual, int T, float* probs,
                   int32_t* topk_idx, float* topk_gate, hipStream_t stream) {
  const int d = ctx->cfg.d_model, E = ctx->cfg.n_experts;
  const size_t budget = 144 * 1024;
  auto lds = [&](int tok) {
    return (size_t)kWaves * tok * d * sizeof(XT) + (size_t)kWaves * tok * E * sizeof(float);
  };
  // more tokens per wavefront = more reuse of each router-weight load; fewer = more blocks
  int tok = 4;
  while (tok > 1 && (lds(tok) > budget || (T + kWaves * tok - 1) / (kWaves * tok) < 512)) tok >>= 1;
  if (lds(tok) > budget)
    return fmoe_fail(FMOE_ERR_UNSUPPORTED, "route: d_model %d too large for the LDS row stage", d);
  if (tok == 4) return launch_route_t<XT, 4, 8>(ctx, x, is_visual, T, probs, topk_idx, topk_gate, stream);
  if (tok == 2) return launch_route_t<XT, 2, 8>(ctx, x, is_visual, T, probs, topk_idx, topk_gate, stream);
  return launch_route_t<XT, 1, 8>(ctx, x, is_visual, T, probs, topk_idx, topk_gate, stream);
}

}  // namespace

int launch_widen_bf16(const void* src, float* dst, size_t n, hipStream_t stream) {
  if (n == 0) return FMOE_OK;
  const int grid = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
  hipLaunchKernelGGL(widen_bf16_kernel, dim3(grid), dim3(256), 0, stream,
                     static_cast<const bf16_t*>(src), dst, n);
  FMOE_HIP_CHECK(hipGetLastError());
  return FMOE_OK;
}

int launch_route(const fmoe_ctx* ctx, const void* x, const uint8_t* is_visual, int T, float* probs,
                 int32_t* topk_idx, float* topk_gate, hipStream_t stream) {
  if (T == 0) return FMOE_OK;
  if (ctx->cfg.dtype == FMOE_BF16)
    return launch_route_x<bf16_t>(ctx, x, is_visual, T, probs, topk_idx, topk_gate, stream);
  return launch_route_x<float>(ctx, x, is_visual, T, probs, topk_idx, topk_gate, stream);
}
