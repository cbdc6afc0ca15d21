// Device-side construction of the grouped-GEMM work lists, shared by the permutation scan (fused
// layer path) and the stand-alone expert-FFN entry point.
#pragma once

#include "common.h"

#if defined(__HIPCC__)
// Builds, with one 256-thread block, the two row-tile lists of the expert FFN (`bm` rows per tile):
//   list 1 (gate/up GEMM): the dense shared-expert group (group id E, all n kept tokens, hidden
//     dimension = the N_s experts concatenated) first, then the routed experts;
//   list 2 (down GEMM): one dense group per shared expert (group id E+s) first, then the routed
//     experts.
// Long items go first: the shared groups (every kept token), then the routed experts by
// descending row count (ties: ascending expert id), so that the short tiles are the ones left to
// fill the tail of the launch.  A launch gives every entry `cols1` column tiles; the shared group
// of list 1 may have more (`scols1`): its row tiles are then repeated with a column-tile offset in
// `col0`.  The row tiles of one group (one replica) are consecutive entries, cut into runs of at most
// FMOE_TILE_RUN row tiles (rt / nrt number a tile within its run): a run is the unit within which
// the GEMM kernel re-deals its workgroups column-major, and eight row tiles by eight column tiles
// is about what one XCD runs at a time.
// counts[0], counts[1] = number of entries in list 1 / list 2.  Experts whose offsets are malformed
// (negative, decreasing or past row_cap) are skipped so that no tile can index outside the row
// buffers.  `scratch` is 513 ints of LDS (8-byte aligned); bm is a power of two.
__device__ __forceinline__ void fmoe_build_tiles(const int32_t* expert_offsets, int E, int row_cap,
                                                 int n, int n_shared, int bm, int tile_cap, int cols1,
                                                 int scols1, fmoe_tile* tiles1, fmoe_tile* tiles2,
                                                 int32_t* counts, int* scratch) {
  const int e = threadIdx.x;
  const int sh = 31 - __clz(bm);   // bm is a power of two
  int r0 = 0, cnt = 0;
  if (e < E) {
    r0 = expert_offsets[e];
    const int r1 = expert_offsets[e + 1];
    cnt = r1 - r0;
    if (r0 < 0 || cnt < 0 || r1 > row_cap) cnt = 0;
  }
  __syncthreads();
  // order key: more rows first, then the lower expert id (rows < 2^24, ids < 2^8)
  const unsigned key = ((unsigned)cnt << 8) | (unsigned)(255 - (e & 255));
  if (e < 256) {
    scratch[2 * e] = (e < E) ? (int)key : 0;
    scratch[2 * e + 1] = (e < E) ? ((cnt + bm - 1) >> sh) : 0;
  }
  __syncthreads();
  // first tile slot of expert e = tiles of all experts ahead of it in that order
  int start = 0, routed = 0;
  if (e < E) {
#pragma unroll 8
    for (int o = 0; o < E; ++o) {
      const int2 kn = *reinterpret_cast<const int2*>(&scratch[2 * o]);
      routed += kn.y;
      start += ((unsigned)kn.x > key) ? kn.y : 0;
    }
    if (e == 0) scratch[512] = routed;
  }
  __syncthreads();
  routed = scratch[512];

  const int ns = (n_shared > 0) ? (n + bm - 1) / bm : 0;
  const int rep1 = (ns > 0 && cols1 > 0) ? (scols1 + cols1 - 1) / cols1 : 0;
  const int sh1 = ns * rep1, sh2 = ns * n_shared;
  for (int j = threadIdx.x; j < ns; j += blockDim.x) {
    fmoe_tile t;
    t.row0 = j * bm;
    t.rows = (n - j * bm < bm) ? (n - j * bm) : bm;
    t.rt = j % FMOE_TILE_RUN;
    t.nrt = (ns - (j - t.rt) < FMOE_TILE_RUN) ? (ns - (j - t.rt)) : FMOE_TILE_RUN;
    t.group = E;
    for (int c = 0; c < rep1; ++c) {   // replica-major: the row tiles of one replica are consecutive
      const int slot = c * ns + j;
      if (slot >= tile_cap) break;
      t.col0 = c * cols1;
      tiles1[slot] = t;
    }
    t.col0 = 0;
    for (int s = 0; s < n_shared; ++s) {
      const int slot = s * ns + j;
      if (slot >= tile_cap) break;
      t.group = E + s;
      tiles2[slot] = t;
    }
  }
  if (e < E) {
    const int nt = (cnt + bm - 1) >> sh;
    for (int j = 0; j < nt; ++j) {
      fmoe_tile t;
      t.group = e;
      t.row0 = r0 + j * bm;
      t.rows = (cnt - j * bm < bm) ? (cnt - j * bm) : bm;
      t.col0 = 0;
      t.rt = j % FMOE_TILE_RUN;
      t.nrt = (nt - (j - t.rt) < FMOE_TILE_RUN) ? (nt - (j - t.rt)) : FMOE_TILE_RUN;
      if (sh1 + start + j < tile_cap) tiles1[sh1 + start + j] = t;
      if (sh2 + start + j < tile_cap) tiles2[sh2 + start + j] = t;
    }
  }
  if (threadIdx.x == 0) {
    const int t1 = routed + sh1, t2 = routed + sh2;
    counts[0] = t1 < tile_cap ? t1 : tile_cap;
    counts[1] = t2 < tile_cap ? t2 : tile_cap;
  }
}
#endif
