// The paper's analysis statistics as device kernels (diagnostics: they read the layer's tensors and
// feed none of its decisions): adjacent-token routing similarity (Fig. 1; Eq.8 on a two-token
// window), magnitude stability of expert outputs (App. C.1), the measured cosine between two layer
// outputs and the closed-form angle of App. C.  fp32 arithmetic inside a row, fp64 for the sums over
// tokens; every reduction has a fixed order, so results are reproducible run to run.

#include "common.h"
#include "prune_dev.h"

namespace {

__device__ __forceinline__ float wave_sum_f32(float v) {
#pragma unroll
  for (int sh = 32; sh >= 1; sh >>= 1) v += __shfl_xor(v, sh, 64);
  return v;
}

// sum over the block's 256 threads in a fixed order; red: 4 doubles of LDS
__device__ __forceinline__ double block_sum_256(double v, double* red) {
#pragma unroll
  for (int sh = 32; sh >= 1; sh >>= 1) v += __shfl_xor(v, sh, 64);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

// One wavefront per token t: cosine of the routing rows of t and t+1 when both lie in one sequence
// and share the modality, -2 otherwise.
__global__ __launch_bounds__(256) void adjacent_sim_kernel(
    const float* __restrict__ probs, const uint8_t* __restrict__ is_visual, const int32_t* __restrict__ cu,
    int B, int T, int E, float* __restrict__ pair_sim) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  int s, e;
  seq_range(cu, find_seq(cu, B, t), T, s, e);
  const bool pair = t >= s && t + 1 < e && ((is_visual[t] != 0) == (is_visual[t + 1] != 0));
  if (!pair) {
    if (lane == 0) pair_sim[t] = -2.0f;
    return;
  }
  const float* a = probs + (size_t)t * E;
  const float* c = a + E;
  float ab = 0.0f, aa = 0.0f, cc = 0.0f;
  for (int j = lane; j < E; j += 64) {
    const float u = a[j], v = c[j];
    ab = fmaf(u, v, ab);
    aa = fmaf(u, u, aa);
    cc = fmaf(v, v, cc);
  }
  ab = wave_sum_f32(ab);
  aa = wave_sum_f32(aa);
  cc = wave_sum_f32(cc);
  const float den = sqrtf(aa) * sqrtf(cc);
  if (lane == 0) pair_sim[t] = den > 0.0f ? ab / den : 0.0f;
}

// Means of pair_sim per modality (one block; index 0 text, 1 vision).
__global__ __launch_bounds__(256) void adjacent_mean_kernel(
    const float* __restrict__ pair_sim, const uint8_t* __restrict__ is_visual, int T,
    float* __restrict__ mean, int32_t* __restrict__ count) {
  __shared__ double red[4];
  double sum[2] = {0.0, 0.0}, cnt[2] = {0.0, 0.0};
  for (int t = threadIdx.x; t < T; t += 256) {
    const float v = pair_sim[t];
    if (v < -1.5f) continue;
    const int m = is_visual[t] ? 1 : 0;
    sum[m] += (double)v;
    cnt[m] += 1.0;
  }
  for (int m = 0; m < 2; ++m) {
    const double s = block_sum_256(sum[m], red);
    const double n = block_sum_256(cnt[m], red);
    if (threadIdx.x == 0) {
      mean[m] = n > 0.0 ? (float)(s / n) : 0.0f;
      count[m] = (int32_t)n;
    }
  }
}

// One wavefront per row: Euclidean norm of an expert-output row.
template <typename T>
__global__ __launch_bounds__(256) void row_norm_kernel(const T* __restrict__ y, int M, const int32_t* __restrict__ M_dev,
                                                       int d, float* __restrict__ row_norm) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int n = M_dev ? (*M_dev < M ? *M_dev : M) : M;
  if (r >= n) return;
  const T* row = y + (size_t)r * d;
  float q = 0.0f;
  for (int c = lane; c < d; c += 64) {
    const float v = to_f32(row[c]);
    q = fmaf(v, v, q);
  }
  q = wave_sum_f32(q);
  if (lane == 0) row_norm[r] = sqrtf(q);
}

// mu, sigma (population, two passes), CV and V = 1/(1+CV) of the row norms per modality (one block).
// The modality of row r is that of the token it was computed for: is_visual[kept_idx[perm_src[r]]].
__global__ __launch_bounds__(256) void stability_kernel(
    const float* __restrict__ row_norm, int M, const int32_t* __restrict__ M_dev,
    const int32_t* __restrict__ perm_src, const int32_t* __restrict__ kept_idx,
    const uint8_t* __restrict__ is_visual, float* __restrict__ stats) {
  __shared__ double red[4];
  const int n = M_dev ? (*M_dev < M ? *M_dev : M) : M;
  auto modality = [&](int r) {
    int p = perm_src[r];
    if (kept_idx) p = kept_idx[p];
    return is_visual[p] ? 1 : 0;
  };
  double sum[2] = {0.0, 0.0}, cnt[2] = {0.0, 0.0};
  for (int r = threadIdx.x; r < n; r += 256) {
    const int m = modality(r);
    sum[m] += (double)row_norm[r];
    cnt[m] += 1.0;
  }
  double mu[2], num[2];
  for (int m = 0; m < 2; ++m) {
    const double s = block_sum_256(sum[m], red);
    num[m] = block_sum_256(cnt[m], red);
    mu[m] = num[m] > 0.0 ? s / num[m] : 0.0;
  }
  double dev[2] = {0.0, 0.0};
  for (int r = threadIdx.x; r < n; r += 256) {
    const int m = modality(r);
    const double q = (double)row_norm[r] - mu[m];
    dev[m] += q * q;
  }
  for (int m = 0; m < 2; ++m) {
    const double ss = block_sum_256(dev[m], red);
    if (threadIdx.x == 0) {
      const double sigma = num[m] > 0.0 ? sqrt(ss / num[m]) : 0.0;
      const double cv = mu[m] > 0.0 ? sigma / mu[m] : 0.0;
      stats[m * 4 + 0] = (float)mu[m];
      stats[m * 4 + 1] = (float)sigma;
      stats[m * 4 + 2] = (float)cv;
      stats[m * 4 + 3] = (float)(1.0 / (1.0 + cv));
    }
  }
}

// One wavefront per row: cosine between row r of a and of b.
template <typename T>
__global__ __launch_bounds__(256) void row_cosine_kernel(const T* __restrict__ a, const T* __restrict__ b, int n_cap,
                                                         const int32_t* __restrict__ n_dev, int d,
                                                         float* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int n = n_dev ? (*n_dev < n_cap ? *n_dev : n_cap) : n_cap;
  if (r >= n) return;
  const T* ra = a + (size_t)r * d;
  const T* rb = b + (size_t)r * d;
  float ab = 0.0f, aa = 0.0f, bb = 0.0f;
  for (int c = lane; c < d; c += 64) {
    const float u = to_f32(ra[c]), v = to_f32(rb[c]);
    ab = fmaf(u, v, ab);
    aa = fmaf(u, u, aa);
    bb = fmaf(v, v, bb);
  }
  ab = wave_sum_f32(ab);
  aa = wave_sum_f32(aa);
  bb = wave_sum_f32(bb);
  const float den = sqrtf(aa) * sqrtf(bb);
  if (lane == 0) out[r] = den > 0.0f ? ab / den : 0.0f;
}

// App. C closed form, one thread per token: sqrt(sum_{i<m} a_i^2 / sum_{i<K} a_i^2) of the token's K
// gates in descending order; 0 when fewer than K gates are positive.
__global__ void gate_cosine_kernel(const float* __restrict__ gates, int T, int K, int m, float* __restrict__ out) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  float top = 0.0f, all = 0.0f;
  bool ok = K > 0;
  for (int i = 0; i < K; ++i) {
    const float a = gates[(size_t)t * K + i];
    ok = ok && (a > 0.0f);
    all = fmaf(a, a, all);
    if (i < m) top = fmaf(a, a, top);
  }
  out[t] = ok ? sqrtf(top / all) : 0.0f;
}

}  // namespace

int launch_adjacent_similarity(const float* probs, const uint8_t* is_visual, const int32_t* cu, int B, int T,
                               int E, float* pair_sim, float* mean, int32_t* count, hipStream_t stream) {
  if (T > 0)
    hipLaunchKernelGGL(adjacent_sim_kernel, dim3((T + 3) / 4), dim3(256), 0, stream, probs, is_visual, cu, B,
                       T, E, pair_sim);
  hipLaunchKernelGGL(adjacent_mean_kernel, dim3(1), dim3(256), 0, stream, pair_sim, is_visual, T, mean, count);
  FMOE_HIP_CHECK(hipGetLastError());
  return FMOE_OK;
}

int launch_magnitude_stability(const fmoe_ctx* ctx, const void* y, int M, const int32_t* M_dev,
                               const int32_t* perm_src, const int32_t* kept_idx, const uint8_t* is_visual,
                               float* row_norm, float* stats, hipStream_t stream) {
  const int d = ctx->cfg.d_model;
  if (M > 0) {
    if (ctx->cfg.dtype == FMOE_BF16)
      hipLaunchKernelGGL(row_norm_kernel<bf16_t>, dim3((M + 3) / 4), dim3(256), 0, stream,
                         static_cast<const bf16_t*>(y), M, M_dev, d, row_norm);
    else
      hipLaunchKernelGGL(row_norm_kernel<float>, dim3((M + 3) / 4), dim3(256), 0, stream,
                         static_cast<const float*>(y), M, M_dev, d, row_norm);
  }
  hipLaunchKernelGGL(stability_kernel, dim3(1), dim3(256), 0, stream, row_norm, M, M_dev, perm_src, kept_idx,
                     is_visual, stats);
  FMOE_HIP_CHECK(hipGetLastError());
  return FMOE_OK;
}

int launch_row_cosine(const fmoe_ctx* ctx, const void* a, const void* b, int n, const int32_t* n_dev, float* out,
                      hipStream_t stream) {
  const int d = ctx->cfg.d_model;
  if (n == 0) return FMOE_OK;
  if (ctx->cfg.dtype == FMOE_BF16)
    hipLaunchKernelGGL(row_cosine_kernel<bf16_t>, dim3((n + 3) / 4), dim3(256), 0, stream,
                       static_cast<const bf16_t*>(a), static_cast<const bf16_t*>(b), n, n_dev, d, out);
  else
    hipLaunchKernelGGL(row_cosine_kernel<float>, dim3((n + 3) / 4), dim3(256), 0, stream,
                       static_cast<const float*>(a), static_cast<const float*>(b), n, n_dev, d, out);
  FMOE_HIP_CHECK(hipGetLastError());
  return FMOE_OK;
}

int launch_gate_cosine(const float* gates, int T, int K, int m, float* out, hipStream_t stream) {
  if (T == 0) return FMOE_OK;
  hipLaunchKernelGGL(gate_cosine_kernel, dim3((T + 255) / 256), dim3(256), 0, stream, gates, T, K, m, out);
  FMOE_HIP_CHECK(hipGetLastError());
  return FMOE_OK;
}
