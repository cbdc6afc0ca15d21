// Expert FFNs of Eq.4 as grouped GEMMs on the matrix cores.
//
//   GEMM-1 (per expert e, rows gathered through the permutation):
//       h = silu(X_e W_gate[e]^T) * (X_e W_up[e]^T)      fused SwiGLU epilogue, h stored in dtype
//   GEMM-2:  y = h W_down[e]^T
//
// Both are "NT" products: activations [rows, K] and weights [N, K] are K-contiguous, which is
// exactly the operand layout the 32x32 MFMA instructions want (a lane supplies consecutive k of
// one row / one output column), so tiles go global -> LDS -> MFMA without any transposition.
// The ragged per-expert row counts are handled by a device-built list of 64-row tiles; a block
// owns one (row tile, column tile) pair and leaves at once if its index is past the list.
// The always-on shared experts run through the same kernel as one dense group whose
// intermediate dimension is the concatenation of the N_s experts (sum of FFNs = one FFN with
// stacked hidden units), so their sum is accumulated in fp32 inside the down projection.

#include "common.h"

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

constexpr int BM = FMOE_TILE_M;  // 64 rows
constexpr int BN = 64;           // output columns per block (per matrix)
constexpr int BK = 32;           // k elements per LDS stage

template <typename T> struct Traits;
template <> struct Traits<bf16_t> {
  static constexpr int VEC = 8;            // elements per 16-byte chunk
  static constexpr int LDK = BK + 8;       // padded LDS row (80 bytes: conflict-free b128 reads)
};
template <> struct Traits<float> {
  static constexpr int VEC = 4;
  static constexpr int LDK = BK + 4;
};

struct GemmArgs {
  const void* A;            // [*, lda]
  int lda;
  const int32_t* map1;      // row -> index (perm_src) or null
  const int32_t* map2;      // index -> token (kept_idx) or null
  int map1_limit;           // clamp for map1 values (exclusive), <=0: no clamp
  const void* B0;           // [G, N, K] (gate / down)
  const void* B1;           // [G, N, K] (up) when SWIGLU
  long long group_stride;   // elements between groups
  int ldb;                  // elements between consecutive n rows
  int seg_len;              // K is cut in segments of seg_len ...
  long long seg_stride;     // ... that are seg_stride elements apart (shared down projection)
  void* C;                  // [*, ldc]
  int ldc;
  int N, K;
  const fmoe_tile* tiles;
  const int32_t* n_tiles;   // device
  int n_col_tiles;
};

__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.0f + expf(-g)) * u; }

template <typename T, bool SWIGLU>
__global__ __launch_bounds__(256) void grouped_gemm_kernel(GemmArgs a) {
  using TR = Traits<T>;
  constexpr int VEC = TR::VEC, LDK = TR::LDK;
  constexpr int CPR = BK / VEC;               // 16-byte chunks per tile row
  constexpr int ITERS = (BM * CPR) / 256;     // chunks per thread per tile (BM == BN)
  __shared__ __align__(16) T As[BM * LDK];
  __shared__ __align__(16) T B0s[BN * LDK];
  __shared__ __align__(16) T B1s[SWIGLU ? BN * LDK : 1];

  const int mt = blockIdx.x / a.n_col_tiles;
  const int nt = blockIdx.x - mt * a.n_col_tiles;
  if (mt >= *a.n_tiles) return;
  const fmoe_tile tile = a.tiles[mt];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  const T* Ag = static_cast<const T*>(a.A);
  const T* B0g = static_cast<const T*>(a.B0) + (size_t)tile.group * a.group_stride;
  const T* B1g = SWIGLU ? static_cast<const T*>(a.B1) + (size_t)tile.group * a.group_stride : nullptr;

  // per-thread chunk coordinates (fixed over the K loop)
  const T* a_ptr[ITERS];
  const T* b0_ptr[ITERS];
  const T* b1_ptr[ITERS];
  int c_row[ITERS], c_k[ITERS];
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int chunk = tid + it * 256;
    const int r = chunk / CPR, kc = (chunk % CPR) * VEC;
    c_row[it] = r;
    c_k[it] = kc;
    a_ptr[it] = nullptr;
    if (r < tile.rows) {
      int src = tile.row0 + r;
      if (a.map1) {
        src = a.map1[src];
        if (a.map1_limit > 0) src = src < 0 ? 0 : (src >= a.map1_limit ? a.map1_limit - 1 : src);
      }
      if (a.map2) src = a.map2[src];
      a_ptr[it] = Ag + (size_t)src * a.lda;
    }
    const int n = nt * BN + r;
    b0_ptr[it] = (n < a.N) ? B0g + (size_t)n * a.ldb : nullptr;
    b1_ptr[it] = (SWIGLU && n < a.N) ? B1g + (size_t)n * a.ldb : nullptr;
  }

  f32x16_t acc0, acc1;
#pragma unroll
  for (int v = 0; v < 16; ++v) { acc0[v] = 0.0f; acc1[v] = 0.0f; }

  const uint4 zero4 = make_uint4(0, 0, 0, 0);
  for (int k0 = 0; k0 < a.K; k0 += BK) {
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      const int k = k0 + c_k[it];
      const bool kin = k < a.K;
      // weights may be cut in K segments (shared experts' down projection)
      const int seg = k / a.seg_len;
      const size_t boff = (size_t)seg * a.seg_stride + (size_t)(k - seg * a.seg_len);
      uint4 va = zero4, vb0 = zero4, vb1 = zero4;
      if (kin && a_ptr[it]) va = *reinterpret_cast<const uint4*>(a_ptr[it] + k);
      if (kin && b0_ptr[it]) vb0 = *reinterpret_cast<const uint4*>(b0_ptr[it] + boff);
      if (SWIGLU && kin && b1_ptr[it]) vb1 = *reinterpret_cast<const uint4*>(b1_ptr[it] + boff);
      const int lo = c_row[it] * LDK + c_k[it];
      *reinterpret_cast<uint4*>(&As[lo]) = va;
      *reinterpret_cast<uint4*>(&B0s[lo]) = vb0;
      if (SWIGLU) *reinterpret_cast<uint4*>(&B1s[lo]) = vb1;
    }
    __syncthreads();
    if constexpr (sizeof(T) == 2) {
#pragma unroll
      for (int ks = 0; ks < BK; ks += 16) {
        const int ko = ks + (lane >> 5) * 8;
        const bf16x8_t fa = *reinterpret_cast<const bf16x8_t*>(&As[(wm * 32 + (lane & 31)) * LDK + ko]);
        const bf16x8_t fb0 = *reinterpret_cast<const bf16x8_t*>(&B0s[(wn * 32 + (lane & 31)) * LDK + ko]);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb0, acc0, 0, 0, 0);
        if (SWIGLU) {
          const bf16x8_t fb1 = *reinterpret_cast<const bf16x8_t*>(&B1s[(wn * 32 + (lane & 31)) * LDK + ko]);
          acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb1, acc1, 0, 0, 0);
        }
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < BK; ks += 2) {
        const int ko = ks + (lane >> 5);
        const float fa = As[(wm * 32 + (lane & 31)) * LDK + ko];
        const float fb0 = B0s[(wn * 32 + (lane & 31)) * LDK + ko];
        acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(fa, fb0, acc0, 0, 0, 0);
        if (SWIGLU) {
          const float fb1 = B1s[(wn * 32 + (lane & 31)) * LDK + ko];
          acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(fa, fb1, acc1, 0, 0, 0);
        }
      }
    }
    __syncthreads();
  }

  // epilogue: accumulator register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, column l%32
  T* Cg = static_cast<T*>(a.C);
  const int col = nt * BN + wn * 32 + (lane & 31);
  if (col < a.N) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int r = wm * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      if (r < tile.rows) {
        const float val = SWIGLU ? silu_mul(acc0[v], acc1[v]) : acc0[v];
        Cg[(size_t)(tile.row0 + r) * a.ldc + col] = from_f32<T>(val);
      }
    }
  }
}

// tile list of the routed experts from expert_offsets (one block)
__global__ __launch_bounds__(256) void build_tiles_kernel(const int32_t* __restrict__ expert_offsets,
                                                          int E, int row_cap, int tile_cap,
                                                          fmoe_tile* __restrict__ tiles,
                                                          int32_t* __restrict__ n_tiles) {
  __shared__ int start[FMOE_MAX_EXPERTS + 1];
  const int e = threadIdx.x;
  int r0 = 0, cnt = 0;
  if (e < E) {
    r0 = expert_offsets[e];
    const int r1 = expert_offsets[e + 1];
    cnt = r1 - r0;
    if (r0 < 0 || cnt < 0 || r1 > row_cap) cnt = 0;  // malformed offsets: skip the expert
  }
  const int nt = (cnt + BM - 1) / BM;
  if (e < E) start[e + 1] = nt;
  if (e == 0) start[0] = 0;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int i = 1; i <= E; ++i) start[i] += start[i - 1];
    n_tiles[0] = start[E] < tile_cap ? start[E] : tile_cap;
  }
  __syncthreads();
  if (e < E) {
    for (int j = 0; j < nt; ++j) {
      const int slot = start[e] + j;
      if (slot >= tile_cap) break;
      fmoe_tile t;
      t.group = e;
      t.row0 = r0 + j * BM;
      t.rows = (cnt - j * BM < BM) ? (cnt - j * BM) : BM;
      t.pad = 0;
      tiles[slot] = t;
    }
  }
}

// tile list of one dense group of n rows
__global__ void build_dense_tiles_kernel(int n_cap, const int32_t* __restrict__ n_dev,
                                         fmoe_tile* __restrict__ tiles, int32_t* __restrict__ n_tiles) {
  const int n = resolve_count(n_cap, n_dev);
  const int nt = (n + BM - 1) / BM;
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j == 0) n_tiles[0] = nt;
  if (j < nt) {
    fmoe_tile t;
    t.group = 0;
    t.row0 = j * BM;
    t.rows = (n - j * BM < BM) ? (n - j * BM) : BM;
    t.pad = 0;
    tiles[j] = t;
  }
}

template <typename T>
int run_ffn(const fmoe_ctx* ctx, const void* x, const int32_t* kept_idx, int n_cap,
            const int32_t* n_dev, const int32_t* expert_offsets, const int32_t* perm_src, void* y,
            void* y_shared, void* ws, const fmoe_ws_layout& L, hipStream_t stream) {
  const fmoe_config& c = ctx->cfg;
  const int d = c.d_model, E = c.n_experts, F = c.d_ffn, Kmax = ctx->kmax;
  char* base = static_cast<char*>(ws);
  fmoe_tile* tiles = reinterpret_cast<fmoe_tile*>(base + L.tiles);
  int32_t* tile_count = reinterpret_cast<int32_t*>(base + L.tile_count);
  const int row_cap = n_cap * Kmax;
  const int routed_tile_cap = row_cap / BM + E;
  const int dense_tile_cap = (n_cap + BM - 1) / BM;
  fmoe_tile* dense_tiles = tiles + routed_tile_cap;

  if (row_cap > 0) {
    {
      fmoe_prof_scope prof(ctx, SLOT_TILES, stream);
      hipLaunchKernelGGL(build_tiles_kernel, dim3(1), dim3(256), 0, stream, expert_offsets, E, row_cap,
                         routed_tile_cap, tiles, tile_count);
    }
    GemmArgs g1{};
    g1.A = x; g1.lda = d; g1.map1 = perm_src; g1.map2 = kept_idx; g1.map1_limit = n_cap;
    g1.B0 = ctx->w_gate; g1.B1 = ctx->w_up; g1.group_stride = (long long)F * d; g1.ldb = d;
    g1.seg_len = d; g1.seg_stride = 0;
    g1.C = base + L.h; g1.ldc = F; g1.N = F; g1.K = d;
    g1.tiles = tiles; g1.n_tiles = tile_count; g1.n_col_tiles = (F + BN - 1) / BN;
    {
      fmoe_prof_scope prof(ctx, SLOT_GEMM1, stream);
      hipLaunchKernelGGL((grouped_gemm_kernel<T, true>), dim3((unsigned)routed_tile_cap * g1.n_col_tiles),
                         dim3(256), 0, stream, g1);
    }
    GemmArgs g2{};
    g2.A = base + L.h; g2.lda = F; g2.map1 = nullptr; g2.map2 = nullptr; g2.map1_limit = 0;
    g2.B0 = ctx->w_down; g2.B1 = nullptr; g2.group_stride = (long long)d * F; g2.ldb = F;
    g2.seg_len = F; g2.seg_stride = 0;
    g2.C = y; g2.ldc = d; g2.N = d; g2.K = F;
    g2.tiles = tiles; g2.n_tiles = tile_count; g2.n_col_tiles = (d + BN - 1) / BN;
    {
      fmoe_prof_scope prof(ctx, SLOT_GEMM2, stream);
      hipLaunchKernelGGL((grouped_gemm_kernel<T, false>), dim3((unsigned)routed_tile_cap * g2.n_col_tiles),
                         dim3(256), 0, stream, g2);
    }
  }
  if (c.n_shared > 0 && n_cap > 0) {
    const int Fs = c.d_ffn_shared, Ft = c.n_shared * Fs;
    {
      fmoe_prof_scope prof(ctx, SLOT_SH_TILES, stream);
      hipLaunchKernelGGL(build_dense_tiles_kernel, dim3((dense_tile_cap + 255) / 256), dim3(256), 0,
                         stream, n_cap, n_dev, dense_tiles, tile_count + 1);
    }
    GemmArgs g1{};
    g1.A = x; g1.lda = d; g1.map1 = nullptr; g1.map2 = kept_idx; g1.map1_limit = 0;
    g1.B0 = ctx->ws_gate; g1.B1 = ctx->ws_up; g1.group_stride = 0; g1.ldb = d;
    g1.seg_len = d; g1.seg_stride = 0;
    g1.C = base + L.h_shared; g1.ldc = Ft; g1.N = Ft; g1.K = d;
    g1.tiles = dense_tiles; g1.n_tiles = tile_count + 1; g1.n_col_tiles = (Ft + BN - 1) / BN;
    {
      fmoe_prof_scope prof(ctx, SLOT_SH_GEMM1, stream);
      hipLaunchKernelGGL((grouped_gemm_kernel<T, true>), dim3((unsigned)dense_tile_cap * g1.n_col_tiles),
                         dim3(256), 0, stream, g1);
    }
    GemmArgs g2{};
    g2.A = base + L.h_shared; g2.lda = Ft; g2.map1 = nullptr; g2.map2 = nullptr; g2.map1_limit = 0;
    g2.B0 = ctx->ws_down; g2.B1 = nullptr; g2.group_stride = 0; g2.ldb = Fs;
    g2.seg_len = Fs; g2.seg_stride = (long long)d * Fs;
    g2.C = y_shared; g2.ldc = d; g2.N = d; g2.K = Ft;
    g2.tiles = dense_tiles; g2.n_tiles = tile_count + 1; g2.n_col_tiles = (d + BN - 1) / BN;
    {
      fmoe_prof_scope prof(ctx, SLOT_SH_GEMM2, stream);
      hipLaunchKernelGGL((grouped_gemm_kernel<T, false>), dim3((unsigned)dense_tile_cap * g2.n_col_tiles),
                         dim3(256), 0, stream, g2);
    }
  }
  FMOE_HIP_CHECK(hipGetLastError());
  return FMOE_OK;
}

}  // namespace

int launch_expert_ffn(const fmoe_ctx* ctx, const void* x, const int32_t* kept_idx, int n_cap,
                      const int32_t* n_dev, const int32_t* expert_offsets, const int32_t* perm_src,
                      void* y, void* y_shared, void* ws, const fmoe_ws_layout& L,
                      hipStream_t stream) {
  if (ctx->cfg.dtype == FMOE_BF16)
    return run_ffn<bf16_t>(ctx, x, kept_idx, n_cap, n_dev, expert_offsets, perm_src, y, y_shared, ws,
                           L, stream);
  return run_ffn<float>(ctx, x, kept_idx, n_cap, n_dev, expert_offsets, perm_src, y, y_shared, ws, L,
                        stream);
}
