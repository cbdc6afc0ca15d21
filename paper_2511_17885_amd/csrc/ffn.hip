// Expert FFNs of Eq.4 as grouped GEMMs on the matrix cores.
//
//   GEMM-1 (per expert e, rows gathered through the permutation):
//       h = silu(X_e W_gate[e]^T) * (X_e W_up[e]^T)      fused SwiGLU epilogue, h stored in dtype
//   GEMM-2:  y = h W_down[e]^T
//
// Both are "NT" products: activations [rows, K] and weights [N, K] are K-contiguous, which is
// exactly the operand layout the 32x32 MFMA instructions want (a lane supplies consecutive k of
// one row / one output column), so tiles go global -> registers -> LDS -> MFMA without any
// transposition.  With FastMMoE switched on an expert sees a few dozen to a few hundred rows, far
// below the ~315 rows at which a bf16 expert becomes compute bound on this chip, so the kernel
// is built to stream every expert's weights from HBM exactly once at full rate: a block owns a
// (row tile, 128 weight rows) pair, keeps the next k-tile in flight in registers while the
// matrix cores work on the current one, and several blocks share a CU.
//
// The ragged per-expert row counts become a device-built list of row tiles (tiles.h); the
// always-on shared experts are one more dense group in the same list and the same launch.  The
// N_s shared experts are treated as one FFN whose hidden dimension is the concatenation of
// theirs, so their sum is accumulated in fp32 inside the down projection.
//
// Block -> work mapping: workgroups are spread round-robin over the 8 XCDs (each with its own
// L2), so the linear block id is decoded as (batch of 8 row tiles, column tile, tile within the
// batch = XCD); all column tiles of one row tile then run on one XCD and the gathered
// activation rows are fetched from HBM once and re-read from that XCD's L2.

#include "common.h"
#include "tiles.h"

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));   // one 16-byte chunk

constexpr int BNW = 128;  // weight rows per block: 64 gate + 64 up columns, or 128 down columns

template <typename T> struct Traits;
template <> struct Traits<bf16_t> {
  static constexpr int VEC = 8;        // elements per 16-byte chunk
  static constexpr int BK = 64;        // k per LDS stage
  static constexpr int LDK = BK + 8;   // padded LDS row: 144 bytes, conflict-free 16-byte reads
};
template <> struct Traits<float> {
  static constexpr int VEC = 4;
  static constexpr int BK = 32;
  static constexpr int LDK = BK + 4;
};

struct GemmProblem {
  const void* A;            // [*, lda]
  int lda;
  const int32_t* map1;      // row -> index (perm_src) or null
  const int32_t* map2;      // index -> token (kept_idx) or null
  int map1_limit;           // clamp for map1 values (exclusive), <= 0: none
  const void* B0;           // [G, N, K] gate / down
  const void* B1;           // [G, N, K] up (SwiGLU only)
  long long group_stride;   // elements between groups (0 for the shared group)
  int ldb;                  // elements between consecutive weight rows
  int seg_len;              // K is cut in segments of seg_len ...
  long long seg_stride;     // ... seg_stride elements apart (shared down projection)
  void* C;                  // [*, ldc]
  int ldc;
  int N, K;
  int n_col_tiles;
};

struct GemmArgs {
  GemmProblem p0;           // routed experts
  GemmProblem p1;           // shared group (tile.group == E)
  int E;
  const fmoe_tile* tiles;
  const int32_t* n_tiles;   // device
  int n_col_tiles_max;
};

__device__ __forceinline__ float silu_mul(float g, float u) {
  return g * __frcp_rn(1.0f + __expf(-g)) * u;
}

template <typename T, bool SWIGLU, int MT>
__global__ __launch_bounds__(256) void grouped_gemm_kernel(GemmArgs a) {
  using TR = Traits<T>;
  constexpr int VEC = TR::VEC, BK = TR::BK, LDK = TR::LDK;
  constexpr int BM = 64 * MT;
  constexpr int CPR = BK / VEC;                 // 16-byte chunks per tile row (8)
  constexpr int A_IT = BM * CPR / 256;          // chunks per thread
  constexpr int B_IT = BNW * CPR / 256;
  __shared__ __align__(16) T As[BM * LDK];
  __shared__ __align__(16) T Bs[BNW * LDK];

  // XCD-aware decode of the linear block id
  const int xcd = blockIdx.x & 7;
  const int rr = blockIdx.x >> 3;
  const int batch = rr / a.n_col_tiles_max;
  const int nt = rr - batch * a.n_col_tiles_max;
  const int ti = batch * 8 + xcd;
  if (ti >= *a.n_tiles) return;
  const fmoe_tile tile = a.tiles[ti];
  const bool shared = tile.group >= a.E;
  // field-by-field select keeps the descriptors in scalar registers (indexing the kernel argument
  // dynamically would spill it to scratch memory)
  GemmProblem P;
#define FMOE_SEL(f) P.f = shared ? a.p1.f : a.p0.f
  FMOE_SEL(A); FMOE_SEL(lda); FMOE_SEL(map1); FMOE_SEL(map2); FMOE_SEL(map1_limit);
  FMOE_SEL(B0); FMOE_SEL(B1); FMOE_SEL(group_stride); FMOE_SEL(ldb); FMOE_SEL(seg_len);
  FMOE_SEL(seg_stride); FMOE_SEL(C); FMOE_SEL(ldc); FMOE_SEL(N); FMOE_SEL(K); FMOE_SEL(n_col_tiles);
#undef FMOE_SEL
  if (nt >= P.n_col_tiles) return;
  const int group = shared ? 0 : tile.group;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int N = P.N, K = P.K;

  const T* Ag = static_cast<const T*>(P.A);
  const T* B0g = static_cast<const T*>(P.B0) + (size_t)group * P.group_stride;
  const T* B1g = SWIGLU ? static_cast<const T*>(P.B1) + (size_t)group * P.group_stride : nullptr;

  // per-thread chunk sources (fixed over the K loop)
  const T* a_src[A_IT];
  const T* b_src[B_IT];
  int a_lo[A_IT], b_lo[B_IT], a_k[A_IT], b_k[B_IT];
#pragma unroll
  for (int it = 0; it < A_IT; ++it) {
    const int chunk = tid + it * 256;
    const int r = chunk / CPR, kc = (chunk % CPR) * VEC;
    a_lo[it] = r * LDK + kc;
    a_k[it] = kc;
    // rows past the tile reuse its last row: their products land in accumulator rows that are
    // never stored, and the loads stay unconditional (no branches in the pipelined loop)
    int src = tile.row0 + (r < tile.rows ? r : tile.rows - 1);
    if (P.map1) {
      src = P.map1[src];
      if (P.map1_limit > 0) src = src < 0 ? 0 : (src >= P.map1_limit ? P.map1_limit - 1 : src);
    }
    if (P.map2) src = P.map2[src];
    a_src[it] = Ag + (size_t)src * P.lda;
  }
#pragma unroll
  for (int it = 0; it < B_IT; ++it) {
    const int chunk = tid + it * 256;
    const int wr = chunk / CPR, kc = (chunk % CPR) * VEC;
    b_lo[it] = wr * LDK + kc;
    b_k[it] = kc;
    int n;
    const T* base;
    if (SWIGLU) {
      n = nt * 64 + (wr & 63);
      base = (wr < 64) ? B0g : B1g;
    } else {
      n = nt * BNW + wr;
      base = B0g;
    }
    b_src[it] = base + (size_t)(n < N ? n : N - 1) * P.ldb;   // same trick for columns past N
  }
  const bool segmented = P.seg_len < K;

  f32x16_t acc[MT][2];
#pragma unroll
  for (int r = 0; r < MT; ++r)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[r][c][v] = 0.0f;

  // which 32-row groups of this wavefront hold any valid row (uniform per wavefront)
  bool live[MT];
#pragma unroll
  for (int r = 0; r < MT; ++r) live[r] = (wm * 32 * MT + 32 * r) < tile.rows;

  u32x4_t ra[A_IT], rb[B_IT];
  const u32x4_t zero4 = {0u, 0u, 0u, 0u};
  // k past K (ragged last k-tile) must contribute zeros: the address is clamped into the row and
  // the loaded value replaced by a select, so the load itself is never predicated
  auto load_tile = [&](int k0) {
#pragma unroll
    for (int it = 0; it < A_IT; ++it) {
      const int k = k0 + a_k[it];
      const int kk = k < K ? k : K - VEC;
      const u32x4_t v = *reinterpret_cast<const u32x4_t*>(a_src[it] + kk);
      ra[it] = k < K ? v : zero4;
    }
#pragma unroll
    for (int it = 0; it < B_IT; ++it) {
      const int k = k0 + b_k[it];
      const int kk = k < K ? k : K - VEC;
      size_t off = (size_t)kk;
      if (segmented) {   // uniform: only the shared experts' down projection
        const int seg = kk / P.seg_len;
        off = (size_t)seg * P.seg_stride + (size_t)(kk - seg * P.seg_len);
      }
      const u32x4_t v = *reinterpret_cast<const u32x4_t*>(b_src[it] + off);
      rb[it] = k < K ? v : zero4;
    }
  };

  load_tile(0);
  for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
    for (int it = 0; it < A_IT; ++it) *reinterpret_cast<u32x4_t*>(&As[a_lo[it]]) = ra[it];
#pragma unroll
    for (int it = 0; it < B_IT; ++it) *reinterpret_cast<u32x4_t*>(&Bs[b_lo[it]]) = rb[it];
    __syncthreads();
    if (k0 + BK < K) load_tile(k0 + BK);   // in flight while the matrix cores work

    const int brow0 = SWIGLU ? (wn * 32 + (lane & 31)) : (wn * 64 + (lane & 31));
    const int brow1 = SWIGLU ? (64 + wn * 32 + (lane & 31)) : (wn * 64 + 32 + (lane & 31));
    if constexpr (sizeof(T) == 2) {
#pragma unroll
      for (int ks = 0; ks < BK; ks += 16) {
        const int ko = ks + (lane >> 5) * 8;
        const bf16x8_t fb0 = *reinterpret_cast<const bf16x8_t*>(&Bs[brow0 * LDK + ko]);
        const bf16x8_t fb1 = *reinterpret_cast<const bf16x8_t*>(&Bs[brow1 * LDK + ko]);
#pragma unroll
        for (int r = 0; r < MT; ++r) {
          if (live[r]) {
            const int arow = wm * 32 * MT + 32 * r + (lane & 31);
            const bf16x8_t fa = *reinterpret_cast<const bf16x8_t*>(&As[arow * LDK + ko]);
            acc[r][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb0, acc[r][0], 0, 0, 0);
            acc[r][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb1, acc[r][1], 0, 0, 0);
          }
        }
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < BK; ks += 2) {
        const int ko = ks + (lane >> 5);
        const float fb0 = Bs[brow0 * LDK + ko];
        const float fb1 = Bs[brow1 * LDK + ko];
#pragma unroll
        for (int r = 0; r < MT; ++r) {
          if (live[r]) {
            const int arow = wm * 32 * MT + 32 * r + (lane & 31);
            const float fa = As[arow * LDK + ko];
            acc[r][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa, fb0, acc[r][0], 0, 0, 0);
            acc[r][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa, fb1, acc[r][1], 0, 0, 0);
          }
        }
      }
    }
    __syncthreads();
  }

  // epilogue: accumulator register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, column l%32
  T* Cg = static_cast<T*>(P.C);
#pragma unroll
  for (int r = 0; r < MT; ++r) {
    if (!live[r]) continue;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = wm * 32 * MT + 32 * r + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      if (row >= tile.rows) continue;
      T* crow = Cg + (size_t)(tile.row0 + row) * P.ldc;
      if (SWIGLU) {
        const int col = nt * 64 + wn * 32 + (lane & 31);
        if (col < N) crow[col] = from_f32<T>(silu_mul(acc[r][0][v], acc[r][1][v]));
      } else {
        const int col = nt * BNW + wn * 64 + (lane & 31);
        if (col < N) crow[col] = from_f32<T>(acc[r][0][v]);
        if (col + 32 < N) crow[col + 32] = from_f32<T>(acc[r][1][v]);
      }
    }
  }
}

__global__ __launch_bounds__(256) void build_tiles_kernel(const int32_t* __restrict__ expert_offsets,
                                                          int E, int row_cap, int n_cap,
                                                          const int32_t* __restrict__ n_dev,
                                                          int has_shared, int bm, int tile_cap,
                                                          fmoe_tile* __restrict__ tiles,
                                                          int32_t* __restrict__ counts) {
  __shared__ int scratch[FMOE_MAX_EXPERTS + 1];
  fmoe_build_tiles(expert_offsets, E, row_cap, resolve_count(n_cap, n_dev), has_shared != 0, bm,
                   tile_cap, tiles, counts, scratch);
}

template <typename T, int MT>
int run_ffn(const fmoe_ctx* ctx, const void* x, const int32_t* kept_idx, int n_cap,
            const int32_t* n_dev, const int32_t* expert_offsets, const int32_t* perm_src, void* y,
            void* y_shared, void* ws, const fmoe_ws_layout& L, bool tiles_ready, hipStream_t stream) {
  const fmoe_config& c = ctx->cfg;
  const int d = c.d_model, E = c.n_experts, F = c.d_ffn, Kmax = ctx->kmax;
  const bool has_shared = c.n_shared > 0;
  char* base = static_cast<char*>(ws);
  fmoe_tile* tiles = reinterpret_cast<fmoe_tile*>(base + L.tiles);
  int32_t* tile_count = reinterpret_cast<int32_t*>(base + L.tile_count);
  const int row_cap = n_cap * Kmax;
  const int bm = 64 * MT;
  const int tile_cap = fmoe_tile_cap(ctx, n_cap);
  if (n_cap == 0 || (row_cap == 0 && !has_shared)) return FMOE_OK;

  if (!tiles_ready) {
    fmoe_prof_scope prof(ctx, SLOT_TILES, stream);
    hipLaunchKernelGGL(build_tiles_kernel, dim3(1), dim3(256), 0, stream, expert_offsets, E, row_cap,
                       n_cap, n_dev, has_shared ? 1 : 0, bm, tile_cap, tiles, tile_count);
  }
  const int Fs = c.d_ffn_shared, Ft = c.n_shared * Fs;
  GemmArgs g1{}, g2{};
  g1.E = g2.E = E;
  g1.tiles = g2.tiles = tiles;
  g1.n_tiles = g2.n_tiles = tile_count;
  // GEMM-1: gate/up + SwiGLU
  {
    GemmProblem& p = g1.p0;
    p.A = x; p.lda = d; p.map1 = perm_src; p.map2 = kept_idx; p.map1_limit = n_cap;
    p.B0 = ctx->w_gate; p.B1 = ctx->w_up; p.group_stride = (long long)F * d; p.ldb = d;
    p.seg_len = d; p.seg_stride = 0;
    p.C = base + L.h; p.ldc = F; p.N = F; p.K = d; p.n_col_tiles = (F + 63) / 64;
    GemmProblem& q = g1.p1;
    q = p;
    q.map1 = nullptr; q.map1_limit = 0;
    q.B0 = ctx->ws_gate; q.B1 = ctx->ws_up; q.group_stride = 0;
    q.C = base + L.h_shared; q.ldc = Ft; q.N = Ft; q.n_col_tiles = has_shared ? (Ft + 63) / 64 : 0;
    g1.n_col_tiles_max = p.n_col_tiles > q.n_col_tiles ? p.n_col_tiles : q.n_col_tiles;
  }
  // GEMM-2: down projection
  {
    GemmProblem& p = g2.p0;
    p.A = base + L.h; p.lda = F; p.map1 = nullptr; p.map2 = nullptr; p.map1_limit = 0;
    p.B0 = ctx->w_down; p.B1 = nullptr; p.group_stride = (long long)d * F; p.ldb = F;
    p.seg_len = F; p.seg_stride = 0;
    p.C = y; p.ldc = d; p.N = d; p.K = F; p.n_col_tiles = (d + BNW - 1) / BNW;
    GemmProblem& q = g2.p1;
    q = p;
    q.A = base + L.h_shared; q.lda = Ft;
    q.B0 = ctx->ws_down; q.group_stride = 0; q.ldb = Fs; q.seg_len = has_shared ? Fs : 1;
    q.seg_stride = (long long)d * Fs;
    q.C = y_shared; q.K = Ft; q.n_col_tiles = has_shared ? p.n_col_tiles : 0;
    g2.n_col_tiles_max = p.n_col_tiles;
  }
  const unsigned batches = (unsigned)((tile_cap + 7) / 8);
  {
    fmoe_prof_scope prof(ctx, SLOT_GEMM1, stream);
    hipLaunchKernelGGL((grouped_gemm_kernel<T, true, MT>), dim3(batches * 8 * g1.n_col_tiles_max),
                       dim3(256), 0, stream, g1);
  }
  {
    fmoe_prof_scope prof(ctx, SLOT_GEMM2, stream);
    hipLaunchKernelGGL((grouped_gemm_kernel<T, false, MT>), dim3(batches * 8 * g2.n_col_tiles_max),
                       dim3(256), 0, stream, g2);
  }
  FMOE_HIP_CHECK(hipGetLastError());
  return FMOE_OK;
}

}  // namespace

// Rows per grouped-GEMM tile for a call with capacity n_cap: larger tiles when experts can be
// expected to hold many rows (fewer re-reads of their weights), smaller ones otherwise.
int fmoe_tile_rows(const fmoe_ctx* ctx, int n_cap) {
  if (ctx->cfg.dtype != FMOE_BF16) return 64;
  const long long avg = (long long)n_cap * ctx->kmax / ctx->cfg.n_experts;
  return avg >= 1024 ? 256 : 128;
}

int fmoe_tile_cap(const fmoe_ctx* ctx, int n_cap) {
  const int bm = fmoe_tile_rows(ctx, n_cap);
  return (int)(((long long)n_cap * ctx->kmax) / bm) + ctx->cfg.n_experts + (n_cap + bm - 1) / bm;
}

int launch_expert_ffn(const fmoe_ctx* ctx, const void* x, const int32_t* kept_idx, int n_cap,
                      const int32_t* n_dev, const int32_t* expert_offsets, const int32_t* perm_src,
                      void* y, void* y_shared, void* ws, const fmoe_ws_layout& L, bool tiles_ready,
                      hipStream_t stream) {
  const int bm = fmoe_tile_rows(ctx, n_cap);
  if (ctx->cfg.dtype == FMOE_BF16) {
    if (bm == 256)
      return run_ffn<bf16_t, 4>(ctx, x, kept_idx, n_cap, n_dev, expert_offsets, perm_src, y, y_shared,
                                ws, L, tiles_ready, stream);
    return run_ffn<bf16_t, 2>(ctx, x, kept_idx, n_cap, n_dev, expert_offsets, perm_src, y, y_shared,
                              ws, L, tiles_ready, stream);
  }
  return run_ffn<float, 1>(ctx, x, kept_idx, n_cap, n_dev, expert_offsets, perm_src, y, y_shared, ws,
                           L, tiles_ready, stream);
}
