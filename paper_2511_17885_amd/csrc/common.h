// Internal declarations shared by the library's translation units (host side + device helpers).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "fmoe.h"

#define FMOE_MAX_EXPERTS 256
#define FMOE_MAX_TOPK 16
#define FMOE_MAX_WINDOW 64
#define FMOE_PERM_BLOCK 256   // kept positions per block in the permutation kernels
#define FMOE_TILE_M 64        // rows per grouped-GEMM tile (tile list granularity)
#define FMOE_TILE_RUN 8       // row tiles per run of a group in the tile lists
#define FMOE_SEG_MIN_TILES 256   // tile entries from which each XCD takes a contiguous segment of the list
#define FMOE_ROUTE_TT2_MIN_TOKENS 16384  // tokens from which a router block takes two tiles of 16 tokens
#define FMOE_ROUTE_SHALLOW_MIN_TOKENS 4096  // tokens from which the router keeps two instead of four chunks in flight
#define FMOE_DENSE_MIN_ROWS 256  // routed-row capacity per expert from which the expert GEMMs take their dense shape

// ---- optional per-kernel timing (instrumentation; off by default)
enum fmoe_kernel_slot {
  SLOT_ROUTE = 0, SLOT_ORDINALS, SLOT_SCORES, SLOT_SELECT, SLOT_COMPACT, SLOT_DISPATCH,
  SLOT_PERM_COUNT, SLOT_PERM_SCAN, SLOT_PERM_SCATTER, SLOT_TILES, SLOT_GEMM1, SLOT_GEMM2,
  SLOT_COMBINE, SLOT_GEMM1_DENSE, SLOT_GEMM2_DENSE, SLOT_COUNT
};
struct fmoe_prof {
  bool on;
  hipEvent_t beg[SLOT_COUNT], end[SLOT_COUNT];
  bool used[SLOT_COUNT];
};

struct fmoe_ctx {
  fmoe_config cfg;
  int device;
  int kmax;
  const void* router_w;      // caller's [E,H] in dtype
  float* router_wp;          // private fp32 copy of router_w in the router kernel's operand order
  const float* router_bias;
  const void *w_gate, *w_up, *w_down;
  const void *ws_gate, *ws_up, *ws_down;
  // bf16 contexts: private copies of the expert weights in matrix-core operand order (ffn.hip)
  void *pk_gate_up, *pk_down, *pk_sgate_up, *pk_sdown;
  bool weights_set;
  int sel_strategy, sel_k_base;   // selection-strategy ablation (fmoe_set_selection); 0 = off
  unsigned long long sel_seed;
  int ffn_shape;                  // fmoe_set_ffn_shape: 0 by size, 1 weight-stream, 2 dense
  fmoe_prof* prof;           // nullptr unless fmoe_profile_enable was called
};

// Brackets one kernel launch with events when profiling is on (host-side cost only then).
struct fmoe_prof_scope {
  fmoe_prof* p; int slot; hipStream_t s;
  fmoe_prof_scope(const fmoe_ctx* ctx, int slot_, hipStream_t s_) : p(ctx->prof), slot(slot_), s(s_) {
    if (p && p->on) { (void)hipEventRecord(p->beg[slot], s); } else { p = nullptr; }
  }
  ~fmoe_prof_scope() {
    if (p) { (void)hipEventRecord(p->end[slot], s); p->used[slot] = true; }
  }
};

// ---- error reporting (api.cpp)
int fmoe_fail(int code, const char* fmt, ...);
#define FMOE_HIP_CHECK(expr)                                                              \
  do {                                                                                    \
    hipError_t _e = (expr);                                                               \
    if (_e != hipSuccess)                                                                 \
      return fmoe_fail(FMOE_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(_e));      \
  } while (0)

// ---- workspace layout: one carve-up used by every entry point
struct fmoe_ws_layout {
  size_t probs, topk_idx, topk_gate;            // layer_forward intermediates
  size_t vis_tok, vis_ord, seq_nv;              // prune
  size_t win_s, win_a, drop_from, keep_prefix;  // prune
  size_t compact_blk;                           // prune: kept tokens per block of the compaction
  size_t rank_c, win_merged, merged_before;     // prune with window merging
  size_t is_merged, vis_out, x_merged;          // layer_forward with window merging
  size_t slot_rank, blk_count;                  // permute
  size_t expert_offsets, perm_src, inv_perm;    // layer_forward intermediates
  size_t tiles, tiles2, tile_count;             // grouped GEMM tile lists (gate/up, down)
  size_t h, h_shared, y, y_shared;              // FFN intermediates
  size_t total;
};
fmoe_ws_layout fmoe_layout(const fmoe_ctx* ctx, int32_t max_tokens, int32_t max_seqs);

struct fmoe_tile {  // one M-tile of the grouped GEMM
  int32_t group;    // expert id
  int32_t row0;     // first row (in the permuted row space)
  int32_t rows;     // valid rows in the tile
  int32_t col0;     // first column tile this entry covers (shared group split over entries)
  int32_t rt;       // index of this row tile within its group's run of consecutive entries
  int32_t nrt;      // number of row tiles in that run
};

// launch geometry of the two grouped GEMMs for a call with capacity n_cap
struct fmoe_ffn_geom {
  int bm;              // rows per tile
  int cols1, scols1;   // column tiles per launch entry / of the shared group, gate-up GEMM
  int cols2, scols2;   // same, down GEMM
  int tile_cap;        // capacity of each tile list
};
fmoe_ffn_geom fmoe_geom(const fmoe_ctx* ctx, int n_cap);
size_t fmoe_packed_bytes(const fmoe_ctx* ctx, int which);   // 0 gate/up, 1 down, 2 shared gate/up, 3 shared down
int launch_pack_experts(fmoe_ctx* ctx, hipStream_t stream);

// ---- kernel launchers (each returns a fmoe_status; all work goes to `stream`)
size_t router_pack_floats(const fmoe_ctx* ctx);
int launch_pack_router(const fmoe_ctx* ctx, const void* router_w, float* wp, hipStream_t stream);

// Visual ordinals to be produced by extra blocks of the router's launch (Sec. 3.2 needs them before
// the window scores; they do not depend on the routing).  cu == nullptr: none.
struct fmoe_ordinals_job {
  const int32_t* cu;
  int B;
  int32_t *vis_ord, *vis_tok, *seq_nv;
};
// T_dev (nullable): device count of the tokens actually present (<= T, the capacity).
int launch_route(const fmoe_ctx* ctx, const void* x, const uint8_t* is_visual, int T, float* probs,
                 int32_t* topk_idx, float* topk_gate, const fmoe_ordinals_job& ord, hipStream_t stream,
                 const int32_t* T_dev = nullptr);

int launch_prune(const fmoe_ctx* ctx, const fmoe_prune_params* pp, const float* probs,
                 const uint8_t* is_visual, const int32_t* cu_seqlens, int B, int T,
                 const float* attn, int32_t* kept_idx, int32_t* new_cu_seqlens, float* scores_out,
                 uint8_t* is_visual_out, const void* x_in, void* x_merged, uint8_t* is_merged_out,
                 void* ws, const fmoe_ws_layout& L, hipStream_t stream, bool ordinals_ready = false);

// Small batches: window scores, then ONE block for drop order, compaction, permutation by expert and
// the grouped-GEMM tile lists (prune == false: every token is kept).  Expects the visual ordinals in
// the workspace (fmoe_ordinals_job) when pruning.  T_dev (nullable): device count of the tokens present;
// write_kept = false: permutation and tile lists only (kept_idx / new_cu_seqlens / is_visual_out untouched).
bool dispatch_small_fits(int T, int window, bool prune);
int launch_prune_dispatch_small(const fmoe_ctx* ctx, const fmoe_prune_params* pp, bool prune,
                                const float* probs, const uint8_t* is_visual, const int32_t* cu_seqlens,
                                int B, int T, const float* attn, const int32_t* topk_idx,
                                int32_t* kept_idx, int32_t* new_cu_seqlens, uint8_t* is_visual_out,
                                int32_t* expert_offsets, int32_t* perm_src, int32_t* inv_perm, void* ws,
                                const fmoe_ws_layout& L, hipStream_t stream, const int32_t* T_dev = nullptr,
                                bool write_kept = true);

int launch_identity_kept(const uint8_t* is_visual, const int32_t* cu_seqlens, int B, int T,
                         int32_t* kept_idx, int32_t* new_cu_seqlens, uint8_t* is_visual_out,
                         hipStream_t stream);

// build_tiles: also write the grouped-GEMM tile lists (geometry from fmoe_geom(ctx, n_cap))
int launch_permute(const fmoe_ctx* ctx, const int32_t* topk_idx, const int32_t* kept_idx, int n_cap,
                   const int32_t* n_dev, int32_t* expert_offsets, int32_t* perm_src,
                   int32_t* inv_perm, void* ws, const fmoe_ws_layout& L, bool build_tiles,
                   hipStream_t stream);



int launch_expert_ffn(const fmoe_ctx* ctx, const void* x, const int32_t* kept_idx, int n_cap,
                      const int32_t* n_dev, const int32_t* expert_offsets, const int32_t* perm_src,
                      void* y, void* y_shared, void* ws, const fmoe_ws_layout& L, bool tiles_ready,
                      hipStream_t stream);

int launch_combine(const fmoe_ctx* ctx, const void* y, const void* y_shared, const int32_t* inv_perm,
                   const float* topk_gate, const int32_t* kept_idx, int n_cap, const int32_t* n_dev,
                   const void* residual, void* out, hipStream_t stream);

// ---- diagnostics (diag.hip)
int launch_adjacent_similarity(const float* probs, const uint8_t* is_visual, const int32_t* cu, int B, int T,
                               int E, float* pair_sim, float* mean, int32_t* count, hipStream_t stream);
int launch_magnitude_stability(const fmoe_ctx* ctx, const void* y, int M, const int32_t* M_dev,
                               const int32_t* perm_src, const int32_t* kept_idx, const uint8_t* is_visual,
                               float* row_norm, float* stats, hipStream_t stream);
int launch_row_cosine(const fmoe_ctx* ctx, const void* a, const void* b, int n, const int32_t* n_dev, float* out,
                      hipStream_t stream);
int launch_gate_cosine(const float* gates, int T, int K, int m, float* out, hipStream_t stream);

// ---- device helpers
#if defined(__HIPCC__)
typedef uint16_t bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even; inputs are finite in this library's data paths
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return bf16_to_f32(v); }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return f32_to_bf16(v); }

// One rounding from fp64 to the storage type.  bf16 goes through an fp32 value rounded to odd (the
// truncated value with a sticky last bit), from which the nearest-even rounding to 8 significant
// bits is the same as from the double itself.
template <typename T> __device__ __forceinline__ T from_f64(double v);
template <> __device__ __forceinline__ float from_f64<float>(double v) { return (float)v; }
template <> __device__ __forceinline__ bf16_t from_f64<bf16_t>(double v) {
  const float f = (float)v;
  const double back = (double)f;
  uint32_t u = __float_as_uint(f);
  if (back != v) {
    if (fabs(back) > fabs(v)) u -= 1u;   // step back towards zero: the truncated value
    u |= 1u;
  }
  return f32_to_bf16(__uint_as_float(u));
}

// number of valid entries: the device-side count if given (clamped to the capacity), else cap
__device__ __forceinline__ int resolve_count(int cap, const int32_t* n_dev) {
  if (n_dev == nullptr) return cap;
  int n = *n_dev;
  return n < 0 ? 0 : (n > cap ? cap : n);
}
#endif
