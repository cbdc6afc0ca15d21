// Gate-weighted un-permute / combine (Eq.4):
//   out[p] = (residual[t]) + sum_i y_shared[i][p] + sum_s gate[t,s] * y[inv_perm[p,s]],   t = kept_idx[p]
// A pure bandwidth kernel: one block per kept token, 16-byte loads of every contributing row,
// fp32 accumulation in the fixed order residual, shared, slot 0, 1, ... and a single rounding to
// the storage type, so the result does not depend on scheduling.

#include "common.h"

namespace {

template <typename T> struct Vec;
template <> struct Vec<bf16_t> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void load(const bf16_t* p, float* f) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float* f) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      w[i] = (uint32_t)f32_to_bf16(f[2 * i]) | ((uint32_t)f32_to_bf16(f[2 * i + 1]) << 16);
    *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
  }
};
template <> struct Vec<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void load(const float* p, float* f) {
    const float4 v = *reinterpret_cast<const float4*>(p);
    f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
  }
  static __device__ __forceinline__ void store(float* p, const float* f) {
    *reinterpret_cast<float4*>(p) = make_float4(f[0], f[1], f[2], f[3]);
  }
};

template <typename T>
__global__ __launch_bounds__(256) void combine_kernel(
    const T* __restrict__ y, const T* __restrict__ y_shared, const int32_t* __restrict__ inv_perm,
    const float* __restrict__ topk_gate, const int32_t* __restrict__ kept_idx, int n_cap,
    const int32_t* __restrict__ n_dev, int row_cap, int Kmax, int d, int n_shared,
    const T* __restrict__ residual, T* __restrict__ out) {
  constexpr int N = Vec<T>::N;
  const int n = resolve_count(n_cap, n_dev);
  const int p = blockIdx.x;
  if (p >= n) return;
  const int t = kept_idx ? kept_idx[p] : p;
  __shared__ int rows[FMOE_MAX_TOPK];
  __shared__ float gates[FMOE_MAX_TOPK];
  if (threadIdx.x < Kmax) {
    int r = inv_perm[(size_t)p * Kmax + threadIdx.x];
    if (r >= row_cap) r = -1;
    rows[threadIdx.x] = r;
    gates[threadIdx.x] = topk_gate[(size_t)t * Kmax + threadIdx.x];
  }
  __syncthreads();
  for (int c = threadIdx.x * N; c < d; c += 256 * N) {
    float acc[N], v[N];
#pragma unroll
    for (int i = 0; i < N; ++i) acc[i] = 0.0f;
    if (residual) {
      Vec<T>::load(residual + (size_t)t * d + c, v);
#pragma unroll
      for (int i = 0; i < N; ++i) acc[i] = v[i];
    }
    if (y_shared) {
      for (int s = 0; s < n_shared; ++s) {   // first sum of Eq.4, in expert order
        Vec<T>::load(y_shared + ((size_t)s * n_cap + p) * d + c, v);
#pragma unroll
        for (int i = 0; i < N; ++i) acc[i] += v[i];
      }
    }
    for (int s = 0; s < Kmax; ++s) {
      const int r = rows[s];
      if (r < 0) continue;
      const float g = gates[s];
      Vec<T>::load(y + (size_t)r * d + c, v);
#pragma unroll
      for (int i = 0; i < N; ++i) acc[i] = fmaf(g, v[i], acc[i]);
    }
    Vec<T>::store(out + (size_t)p * d + c, acc);
  }
}

}  // namespace

int launch_combine(const fmoe_ctx* ctx, const void* y, const void* y_shared, const int32_t* inv_perm,
                   const float* topk_gate, const int32_t* kept_idx, int n_cap, const int32_t* n_dev,
                   const void* residual, void* out, hipStream_t stream) {
  if (n_cap == 0) return FMOE_OK;
  const int d = ctx->cfg.d_model, Kmax = ctx->kmax;
  const int row_cap = n_cap * Kmax;
  fmoe_prof_scope prof(ctx, SLOT_COMBINE, stream);
  if (ctx->cfg.dtype == FMOE_BF16) {
    hipLaunchKernelGGL(combine_kernel<bf16_t>, dim3(n_cap), dim3(256), 0, stream,
                       static_cast<const bf16_t*>(y), static_cast<const bf16_t*>(y_shared), inv_perm,
                       topk_gate, kept_idx, n_cap, n_dev, row_cap, Kmax, d, ctx->cfg.n_shared,
                       static_cast<const bf16_t*>(residual), static_cast<bf16_t*>(out));
  } else {
    hipLaunchKernelGGL(combine_kernel<float>, dim3(n_cap), dim3(256), 0, stream,
                       static_cast<const float*>(y), static_cast<const float*>(y_shared), inv_perm,
                       topk_gate, kept_idx, n_cap, n_dev, row_cap, Kmax, d, ctx->cfg.n_shared,
                       static_cast<const float*>(residual), static_cast<float*>(out));
  }
  FMOE_HIP_CHECK(hipGetLastError());
  return FMOE_OK;
}
