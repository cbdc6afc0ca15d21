// Token permutation by expert: histogram, prefix sums, stable scatter.  The paper leaves the
// dispatch to the framework; this build fixes the order as (expert ascending, kept position
// ascending) so that the permutation is unique and reproducible.
//
// No slot is claimed with an atomic counter (that would make the order depend on scheduling).
// A block of 256 kept positions records, per expert, a 256-bit membership mask in LDS (the
// bitwise OR is order-free); a slot's rank inside the block is the population count of the mask
// bits below its position, per-block counts are scanned in block order, and the destination row
// is expert_offset + block_base + rank.

#include "common.h"
#include "tiles.h"

namespace {

constexpr int PB = FMOE_PERM_BLOCK;
constexpr int PW = PB / 32;  // mask words per expert

// ---- P1: per-block expert masks -> in-block ranks and per-block counts
__global__ __launch_bounds__(PB) void permute_count_kernel(
    const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ kept_idx, int n_cap,
    const int32_t* __restrict__ n_dev, int E, int Kmax, int32_t* __restrict__ slot_rank,
    int32_t* __restrict__ blk_count) {
  __shared__ uint32_t mask[FMOE_MAX_EXPERTS * PW];
  const int n = resolve_count(n_cap, n_dev);
  const int blk = blockIdx.x;
  for (int i = threadIdx.x; i < E * PW; i += PB) mask[i] = 0u;
  __syncthreads();
  const int lp = threadIdx.x;
  const int p = blk * PB + lp;
  int ex[FMOE_MAX_TOPK];
#pragma unroll
  for (int s = 0; s < FMOE_MAX_TOPK; ++s) ex[s] = -1;
  if (p < n) {
    const int t = kept_idx ? kept_idx[p] : p;
#pragma unroll
    for (int s = 0; s < FMOE_MAX_TOPK; ++s) {
      if (s < Kmax) {
        const int e = topk_idx[(size_t)t * Kmax + s];
        if (e >= 0 && e < E) {
          ex[s] = e;
          atomicOr(&mask[e * PW + (lp >> 5)], 1u << (lp & 31));
        }
      }
    }
  }
  __syncthreads();
  if (p < n) {
#pragma unroll
    for (int s = 0; s < FMOE_MAX_TOPK; ++s) {
      if (s < Kmax) {
        int rank = -1;
        if (ex[s] >= 0) {
          const uint32_t* m = &mask[ex[s] * PW];
          rank = __popc(m[lp >> 5] & ((1u << (lp & 31)) - 1u));
          for (int w = 0; w < (lp >> 5); ++w) rank += __popc(m[w]);
        }
        slot_rank[(size_t)p * Kmax + s] = rank;
      }
    }
  }
  for (int e = threadIdx.x; e < E; e += PB) {
    int c = 0;
#pragma unroll
    for (int w = 0; w < PW; ++w) c += __popc(mask[e * PW + w]);
    blk_count[(size_t)blk * E + e] = c;
  }
}

// ---- P2: one block; thread e scans its expert's per-block counts (turning them into block
// bases in place), then the per-expert totals are scanned into expert_offsets.
__global__ __launch_bounds__(256) void permute_scan_kernel(int n_cap, const int32_t* __restrict__ n_dev,
                                                           int E, int32_t* __restrict__ blk_count,
                                                           int32_t* __restrict__ expert_offsets,
                                                           fmoe_ffn_geom geom, int build, int n_shared,
                                                           int row_cap, fmoe_tile* __restrict__ tiles1,
                                                           fmoe_tile* __restrict__ tiles2,
                                                           int32_t* __restrict__ tile_count) {
  __shared__ int total[FMOE_MAX_EXPERTS];
  __shared__ __align__(8) int scratch[513];
  const int n = resolve_count(n_cap, n_dev);
  const int nblk = (n + PB - 1) / PB;
  const int e = threadIdx.x;
  if (e < E) {
    // SC blocks at a time: their counts are fetched together (independent loads), then turned into
    // bases -- one memory latency per SC blocks instead of one per block
    constexpr int SC = 16;
    int running = 0;
    for (int b0 = 0; b0 < nblk; b0 += SC) {
      int c[SC];
#pragma unroll
      for (int i = 0; i < SC; ++i) c[i] = (b0 + i < nblk) ? blk_count[(size_t)(b0 + i) * E + e] : 0;
#pragma unroll
      for (int i = 0; i < SC; ++i) {
        if (b0 + i < nblk) blk_count[(size_t)(b0 + i) * E + e] = running;
        running += c[i];
      }
    }
    total[e] = running;
  }
  __syncthreads();
  if (threadIdx.x < 64) {   // exclusive scan of the (at most 256) totals by one wavefront, four per lane
    const int lane = threadIdx.x;
    int c[4], sum = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int i = 4 * lane + q;
      c[q] = (i < E) ? total[i] : 0;
      sum += c[q];
    }
    int incl = sum;
#pragma unroll
    for (int sh = 1; sh < 64; sh <<= 1) {
      const int o = __shfl_up(incl, sh, 64);
      if (lane >= sh) incl += o;
    }
    int excl = incl - sum;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int i = 4 * lane + q;
      if (i < E) expert_offsets[i] = excl;
      excl += c[q];
    }
    if (lane == 63) expert_offsets[E] = incl;
  }
  if (build) {   // fused layer path: the grouped-GEMM work lists come out of the same scan
    __threadfence_block();
    __syncthreads();
    fmoe_build_tiles(expert_offsets, E, row_cap, n, n_shared, geom.bm, geom.tile_cap, geom.cols1,
                     geom.scols1, tiles1, tiles2, tile_count, scratch);
  }
}

// ---- P3: scatter
__global__ __launch_bounds__(PB) void permute_scatter_kernel(
    const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ kept_idx, int n_cap,
    const int32_t* __restrict__ n_dev, int E, int Kmax, const int32_t* __restrict__ slot_rank,
    const int32_t* __restrict__ blk_base, const int32_t* __restrict__ expert_offsets,
    int32_t* __restrict__ perm_src, int32_t* __restrict__ inv_perm) {
  const int n = resolve_count(n_cap, n_dev);
  const int blk = blockIdx.x;
  const int p = blk * PB + threadIdx.x;
  if (p >= n) return;
  const int t = kept_idx ? kept_idx[p] : p;
  for (int s = 0; s < Kmax; ++s) {
    const int e = topk_idx[(size_t)t * Kmax + s];
    int row = -1;
    if (e >= 0 && e < E) {
      row = expert_offsets[e] + blk_base[(size_t)blk * E + e] + slot_rank[(size_t)p * Kmax + s];
      perm_src[row] = p;
    }
    inv_perm[(size_t)p * Kmax + s] = row;
  }
}

}  // namespace

int launch_permute(const fmoe_ctx* ctx, const int32_t* topk_idx, const int32_t* kept_idx, int n_cap,
                   const int32_t* n_dev, int32_t* expert_offsets, int32_t* perm_src,
                   int32_t* inv_perm, void* ws, const fmoe_ws_layout& L, bool build_tiles,
                   hipStream_t stream) {
  char* base = static_cast<char*>(ws);
  int32_t* slot_rank = reinterpret_cast<int32_t*>(base + L.slot_rank);
  int32_t* blk_count = reinterpret_cast<int32_t*>(base + L.blk_count);
  const int E = ctx->cfg.n_experts, Kmax = ctx->kmax;
  const int nblk = (n_cap + PB - 1) / PB;
  if (nblk > 0 && Kmax > 0) {
    fmoe_prof_scope prof(ctx, SLOT_PERM_COUNT, stream);
    hipLaunchKernelGGL(permute_count_kernel, dim3(nblk), dim3(PB), 0, stream, topk_idx, kept_idx,
                       n_cap, n_dev, E, Kmax, slot_rank, blk_count);
  }
  {
    fmoe_prof_scope prof(ctx, SLOT_PERM_SCAN, stream);
    hipLaunchKernelGGL(permute_scan_kernel, dim3(1), dim3(256), 0, stream, (Kmax > 0) ? n_cap : 0,
                       (Kmax > 0) ? n_dev : nullptr, E, blk_count, expert_offsets,
                       fmoe_geom(ctx, n_cap), build_tiles ? 1 : 0, ctx->cfg.n_shared,
                       n_cap * Kmax, reinterpret_cast<fmoe_tile*>(base + L.tiles),
                       reinterpret_cast<fmoe_tile*>(base + L.tiles2),
                       reinterpret_cast<int32_t*>(base + L.tile_count));
  }
  if (nblk > 0 && Kmax > 0) {
    fmoe_prof_scope prof(ctx, SLOT_PERM_SCATTER, stream);
    hipLaunchKernelGGL(permute_scatter_kernel, dim3(nblk), dim3(PB), 0, stream, topk_idx, kept_idx,
                       n_cap, n_dev, E, Kmax, slot_rank, blk_count, expert_offsets, perm_src,
                       inv_perm);
  }
  FMOE_HIP_CHECK(hipGetLastError());
  return FMOE_OK;
}
