// Device-side construction of the grouped-GEMM work list, shared by the permutation scan (fused
// layer path) and the stand-alone expert-FFN entry point.
#pragma once

#include "common.h"

#if defined(__HIPCC__)
// Builds the tile list with one 256-thread block: routed experts first (ascending expert, then
// ascending rows, `bm` rows per tile), then the dense shared-expert group (group id E) over the
// n kept tokens if has_shared.  counts[0] = number of tiles.  Experts whose offsets are malformed
// (negative, decreasing or past row_cap) are skipped so that no tile can index outside the row
// buffers.  `scratch` is 257 ints of LDS.
__device__ __forceinline__ void fmoe_build_tiles(const int32_t* expert_offsets, int E, int row_cap,
                                                 int n, bool has_shared, int bm, int tile_cap,
                                                 fmoe_tile* tiles, int32_t* counts, int* scratch) {
  const int e = threadIdx.x;
  int r0 = 0, cnt = 0;
  if (e < E) {
    r0 = expert_offsets[e];
    const int r1 = expert_offsets[e + 1];
    cnt = r1 - r0;
    if (r0 < 0 || cnt < 0 || r1 > row_cap) cnt = 0;
  }
  const int nt = (cnt + bm - 1) / bm;
  __syncthreads();
  if (e < E) scratch[e + 1] = nt;
  if (e == 0) scratch[0] = 0;
  __syncthreads();
  if (threadIdx.x == 0)
    for (int i = 1; i <= E; ++i) scratch[i] += scratch[i - 1];
  __syncthreads();
  const int routed = scratch[E];
  if (e < E) {
    for (int j = 0; j < nt; ++j) {
      const int slot = scratch[e] + j;
      if (slot >= tile_cap) break;
      fmoe_tile t;
      t.group = e;
      t.row0 = r0 + j * bm;
      t.rows = (cnt - j * bm < bm) ? (cnt - j * bm) : bm;
      t.pad = 0;
      tiles[slot] = t;
    }
  }
  const int ns = has_shared ? (n + bm - 1) / bm : 0;
  for (int j = threadIdx.x; j < ns; j += blockDim.x) {
    const int slot = routed + j;
    if (slot >= tile_cap) break;
    fmoe_tile t;
    t.group = E;
    t.row0 = j * bm;
    t.rows = (n - j * bm < bm) ? (n - j * bm) : bm;
    t.pad = 0;
    tiles[slot] = t;
  }
  if (threadIdx.x == 0) {
    const int total = routed + ns;
    counts[0] = total < tile_cap ? total : tile_cap;
  }
}
#endif
