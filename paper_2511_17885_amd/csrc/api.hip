// C-ABI entry points: argument validation, workspace carve-up, kernel sequencing.
// No entry point other than fmoe_set_weights (private router copy; packed expert weights of bf16
// contexts) allocates device memory, and none synchronises with the host.

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>

#include "common.h"

namespace {

thread_local char g_err[512] = "";

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }
inline size_t elem_size(const fmoe_ctx* c) { return c->cfg.dtype == FMOE_BF16 ? 2 : 4; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_config(const fmoe_config& c) {
  if (c.d_model <= 0 || c.n_experts <= 0 || c.d_ffn <= 0 || c.n_shared < 0)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "config: sizes must be positive (d_model %d, n_experts %d, d_ffn %d, n_shared %d)",
                     c.d_model, c.n_experts, c.d_ffn, c.n_shared);
  if (c.n_shared > 0 && c.d_ffn_shared <= 0)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "config: d_ffn_shared must be positive when n_shared > 0");
  if (c.dtype != FMOE_F32 && c.dtype != FMOE_BF16)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "config: dtype %d is neither FMOE_F32 nor FMOE_BF16", c.dtype);
  if (c.k_text < 0 || c.k_visual < 0 || c.k_text > c.n_experts || c.k_visual > c.n_experts)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "config: need 0 <= k <= n_experts (k_text %d, k_visual %d, E %d)",
                     c.k_text, c.k_visual, c.n_experts);
  if (c.n_experts > FMOE_MAX_EXPERTS)
    return fmoe_fail(FMOE_ERR_UNSUPPORTED, "config: n_experts %d > %d", c.n_experts, FMOE_MAX_EXPERTS);
  if (c.k_text > FMOE_MAX_TOPK || c.k_visual > FMOE_MAX_TOPK)
    return fmoe_fail(FMOE_ERR_UNSUPPORTED, "config: top-k above %d", FMOE_MAX_TOPK);
  if (c.d_model % 8 || c.d_ffn % 8 || (c.n_shared > 0 && c.d_ffn_shared % 8))
    return fmoe_fail(FMOE_ERR_UNSUPPORTED, "config: d_model, d_ffn and d_ffn_shared must be multiples of 8");
  return FMOE_OK;
}

int check_ctx(const fmoe_ctx* ctx, bool need_weights) {
  if (!ctx) return fmoe_fail(FMOE_ERR_NULL_PTR, "ctx is NULL");
  if (need_weights && !ctx->weights_set)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_set_weights has not been called on this context");
  return FMOE_OK;
}

int check_tokens(int32_t T) {
  if (T < 0) return fmoe_fail(FMOE_ERR_INVALID_ARG, "token count %d is negative", T);
  if (T >= (1 << 24)) return fmoe_fail(FMOE_ERR_UNSUPPORTED, "token count %d >= 2^24", T);
  return FMOE_OK;
}

int check_prune(const fmoe_prune_params* p) {
  if (!(p->retention > 0.0f) || p->retention > 1.0f)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "prune: retention %g outside (0,1]", (double)p->retention);
  if (p->window < 1) return fmoe_fail(FMOE_ERR_INVALID_ARG, "prune: window %d < 1", p->window);
  if (p->window > FMOE_MAX_WINDOW)
    return fmoe_fail(FMOE_ERR_UNSUPPORTED, "prune: window %d > %d", p->window, FMOE_MAX_WINDOW);
  if (!(p->alpha >= 0.0f) || p->alpha > 1.0f)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "prune: alpha %g outside [0,1]", (double)p->alpha);
  if (p->merge_mode != 0 && p->merge_mode != 1)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "prune: merge_mode %d is neither 0 (MLERP) nor 1 (mean)", p->merge_mode);
  if (!(p->gamma >= 0.0f) || p->gamma >= 1.0f)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "prune: gamma %g outside [0,1)", (double)p->gamma);
  if (p->sim_mode != 0 && p->sim_mode != 1)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "prune: sim_mode %d", p->sim_mode);
  if (p->prune_mode < 0 || p->prune_mode > 2)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "prune: prune_mode %d", p->prune_mode);
  return FMOE_OK;
}

// bf16 expert GEMMs address activation rows with 32-bit byte offsets into one buffer descriptor: the
// layer input of n tokens and the hidden buffers of n tokens' rows must each stay below 4 GiB.
int check_ffn_extent(const fmoe_ctx* ctx, int32_t n, const char* who) {
  if (ctx->cfg.dtype != FMOE_BF16) return FMOE_OK;
  const fmoe_config& c = ctx->cfg;
  const size_t lim = 0xffffffffull;
  const size_t kmax = ctx->kmax > 0 ? (size_t)ctx->kmax : 0;
  if ((size_t)n * c.d_model * 2 > lim)
    return fmoe_fail(FMOE_ERR_UNSUPPORTED, "%s: an activation tensor of %d tokens exceeds 4 GiB", who, n);
  if ((size_t)n * kmax * c.d_ffn * 2 > lim || (size_t)n * c.n_shared * c.d_ffn_shared * 2 > lim)
    return fmoe_fail(FMOE_ERR_UNSUPPORTED, "%s: a hidden buffer of %d tokens' rows exceeds 4 GiB", who, n);
  return FMOE_OK;
}

int check_ws(const fmoe_ctx* ctx, const void* ws, size_t ws_bytes, int32_t tokens, int32_t seqs) {
  if (!ws) return fmoe_fail(FMOE_ERR_WORKSPACE, "workspace is NULL");
  if (reinterpret_cast<uintptr_t>(ws) & 255u)
    return fmoe_fail(FMOE_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  const size_t need = fmoe_layout(ctx, tokens, seqs).total;
  if (ws_bytes < need)
    return fmoe_fail(FMOE_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed for %d tokens / %d sequences",
                     ws_bytes, need, tokens, seqs);
  return FMOE_OK;
}

}  // namespace

int fmoe_fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

fmoe_ws_layout fmoe_layout(const fmoe_ctx* ctx, int32_t max_tokens, int32_t max_seqs) {
  const fmoe_config& c = ctx->cfg;
  const size_t T = max_tokens > 0 ? (size_t)max_tokens : 1;
  const size_t B = max_seqs > 0 ? (size_t)max_seqs : 1;
  const size_t K = ctx->kmax > 0 ? (size_t)ctx->kmax : 1;
  const size_t E = (size_t)c.n_experts;
  const size_t es = elem_size(ctx);
  const size_t rows = T * K;
  fmoe_ws_layout L{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  L.probs = take(T * E * 4);
  L.topk_idx = take(rows * 4);
  L.topk_gate = take(rows * 4);
  L.vis_tok = take(T * 4);
  L.vis_ord = take(T * 4);
  L.seq_nv = take(B * 4);
  L.win_s = take(T * 4);
  L.win_a = take(T * 4);
  L.drop_from = take(T * 4);
  L.keep_prefix = take((T + 1) * 4);
  L.compact_blk = take((T / 1024 + 2) * 4);
  L.rank_c = take(T * 4);
  L.win_merged = take(T * 4);
  L.merged_before = take(T * 4);
  L.is_merged = take(T);
  L.vis_out = take(T);
  L.x_merged = take(T * (size_t)c.d_model * es);
  L.slot_rank = take(rows * 4);
  L.blk_count = take(((T + FMOE_PERM_BLOCK - 1) / FMOE_PERM_BLOCK) * E * 4);
  L.expert_offsets = take((E + 1) * 4);
  L.perm_src = take(rows * 4);
  L.inv_perm = take(rows * 4);
  const size_t tile_cap = (size_t)fmoe_geom(ctx, (int)T).tile_cap;
  L.tiles = take(tile_cap * sizeof(fmoe_tile));
  L.tiles2 = take(tile_cap * sizeof(fmoe_tile));
  L.tile_count = take(16);
  L.h = take(rows * (size_t)c.d_ffn * es);
  L.h_shared = take(c.n_shared > 0 ? T * (size_t)c.n_shared * c.d_ffn_shared * es : 0);
  L.y = take(rows * (size_t)c.d_model * es);
  L.y_shared = take(c.n_shared > 0 ? (size_t)c.n_shared * T * (size_t)c.d_model * es : 0);
  L.total = off;
  return L;
}

extern "C" {

const char* fmoe_version(void) { return "fmoe 0.1 (gfx950)"; }

const char* fmoe_last_error(void) { return g_err; }

int fmoe_create(fmoe_ctx** out_ctx, const fmoe_config* config, int device) {
  if (!out_ctx || !config) return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_create: NULL argument");
  *out_ctx = nullptr;
  int rc = check_config(*config);
  if (rc != FMOE_OK) return rc;
  if (device < 0) return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_create: device %d", device);
  fmoe_ctx* ctx = new (std::nothrow) fmoe_ctx();
  if (!ctx) return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_create: out of host memory");
  std::memset(ctx, 0, sizeof(*ctx));
  ctx->cfg = *config;
  ctx->device = device;
  ctx->kmax = config->k_text > config->k_visual ? config->k_text : config->k_visual;
  *out_ctx = ctx;
  return FMOE_OK;
}

void fmoe_destroy(fmoe_ctx* ctx) {
  if (!ctx) return;
  if (ctx->prof) {
    for (int i = 0; i < SLOT_COUNT; ++i) {
      (void)hipEventDestroy(ctx->prof->beg[i]);
      (void)hipEventDestroy(ctx->prof->end[i]);
    }
    delete ctx->prof;
  }
  if (ctx->router_wp) (void)hipFree(ctx->router_wp);
  void* packed[4] = {ctx->pk_gate_up, ctx->pk_down, ctx->pk_sgate_up, ctx->pk_sdown};
  for (void* p : packed)
    if (p) (void)hipFree(p);
  delete ctx;
}

int fmoe_set_topk(fmoe_ctx* ctx, int32_t k_text, int32_t k_visual) {
  int rc = check_ctx(ctx, false);
  if (rc != FMOE_OK) return rc;
  fmoe_config c = ctx->cfg;
  c.k_text = k_text;
  c.k_visual = k_visual;
  rc = check_config(c);
  if (rc != FMOE_OK) return rc;
  ctx->cfg = c;
  ctx->kmax = k_text > k_visual ? k_text : k_visual;
  return FMOE_OK;
}

int fmoe_set_selection(fmoe_ctx* ctx, int32_t strategy, int32_t k_base, uint64_t seed) {
  int rc = check_ctx(ctx, false);
  if (rc != FMOE_OK) return rc;
  if (strategy < 0 || strategy > 2)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_set_selection: strategy %d is not 0 (TopK), 1 (RandomK) or 2 (MinK)", strategy);
  if (k_base < 0 || k_base > ctx->cfg.n_experts || k_base > FMOE_MAX_TOPK)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_set_selection: k_base %d outside [0, min(E, %d)]", k_base, FMOE_MAX_TOPK);
  ctx->sel_strategy = strategy;
  ctx->sel_k_base = k_base;
  ctx->sel_seed = seed;
  return FMOE_OK;
}

int fmoe_set_ffn_shape(fmoe_ctx* ctx, int32_t shape) {
  int rc = check_ctx(ctx, false);
  if (rc != FMOE_OK) return rc;
  if (shape < 0 || shape > 2)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_set_ffn_shape: shape %d is not 0 (by size), 1 (weight-stream) or 2 (dense)", shape);
  ctx->ffn_shape = shape;
  return FMOE_OK;
}

int fmoe_set_weights(fmoe_ctx* ctx, const void* router_w, const float* router_bias,
                     const void* w_gate, const void* w_up, const void* w_down, const void* ws_gate,
                     const void* ws_up, const void* ws_down, void* stream) {
  int rc = check_ctx(ctx, false);
  if (rc != FMOE_OK) return rc;
  if (!router_w || !w_gate || !w_up || !w_down)
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_set_weights: router_w / w_gate / w_up / w_down must not be NULL");
  const bool has_shared = ctx->cfg.n_shared > 0;
  if (has_shared && (!ws_gate || !ws_up || !ws_down))
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_set_weights: shared-expert weights missing (n_shared = %d)",
                     ctx->cfg.n_shared);
  if (!has_shared && (ws_gate || ws_up || ws_down))
    return fmoe_fail(FMOE_ERR_BAD_SHAPE, "fmoe_set_weights: shared-expert weights given but n_shared = 0");
  const void* ptrs[] = {router_w, router_bias, w_gate, w_up, w_down, ws_gate, ws_up, ws_down};
  for (const void* p : ptrs)
    if (p && !aligned16(p)) return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_set_weights: pointer %p not 16-byte aligned", p);
  ctx->weights_set = false;
  ctx->router_w = router_w;
  if (!ctx->router_wp) {
    FMOE_HIP_CHECK(hipSetDevice(ctx->device));
    FMOE_HIP_CHECK(hipMalloc(reinterpret_cast<void**>(&ctx->router_wp), router_pack_floats(ctx) * sizeof(float)));
  }
  rc = launch_pack_router(ctx, router_w, ctx->router_wp, static_cast<hipStream_t>(stream));
  if (rc != FMOE_OK) return rc;
  ctx->router_bias = router_bias;
  ctx->w_gate = w_gate; ctx->w_up = w_up; ctx->w_down = w_down;
  ctx->ws_gate = ws_gate; ctx->ws_up = ws_up; ctx->ws_down = ws_down;
  if (ctx->cfg.dtype == FMOE_BF16) {
    void** slots[4] = {&ctx->pk_gate_up, &ctx->pk_down, &ctx->pk_sgate_up, &ctx->pk_sdown};
    for (int i = 0; i < 4; ++i) {
      const size_t bytes = fmoe_packed_bytes(ctx, i);
      if (bytes && !*slots[i]) FMOE_HIP_CHECK(hipMalloc(slots[i], bytes));
    }
    if ((rc = launch_pack_experts(ctx, static_cast<hipStream_t>(stream))) != FMOE_OK) return rc;
  }
  ctx->weights_set = true;
  return FMOE_OK;
}

size_t fmoe_workspace_bytes(const fmoe_ctx* ctx, int32_t max_tokens, int32_t max_seqs) {
  if (!ctx) return 0;
  return fmoe_layout(ctx, max_tokens, max_seqs).total;
}

int fmoe_route(fmoe_ctx* ctx, const void* x, const uint8_t* is_visual, int32_t T, float* probs,
               int32_t* topk_idx, float* topk_gate, void* stream) {
  int rc = check_ctx(ctx, true);
  if (rc != FMOE_OK) return rc;
  if ((rc = check_tokens(T)) != FMOE_OK) return rc;
  if (T == 0) return FMOE_OK;
  if (!x || !is_visual) return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_route: x / is_visual is NULL");
  if (ctx->kmax > 0 && (!topk_idx || !topk_gate))
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_route: topk_idx / topk_gate is NULL");
  if (!aligned16(x)) return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_route: x not 16-byte aligned");
  return launch_route(ctx, x, is_visual, T, probs, topk_idx, topk_gate, fmoe_ordinals_job{},
                      static_cast<hipStream_t>(stream));
}

int fmoe_prune(fmoe_ctx* ctx, const fmoe_prune_params* params, const float* probs,
               const uint8_t* is_visual, const int32_t* cu_seqlens, int32_t B, int32_t T,
               const float* attn_importance, const void* x_in, int32_t* kept_idx,
               int32_t* new_cu_seqlens, float* scores, void* x_merged, uint8_t* is_merged, void* ws,
               size_t ws_bytes, void* stream) {
  int rc = check_ctx(ctx, false);
  if (rc != FMOE_OK) return rc;
  if (!params) return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_prune: params is NULL");
  if ((rc = check_prune(params)) != FMOE_OK) return rc;
  if ((rc = check_tokens(T)) != FMOE_OK) return rc;
  if (B < 0) return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_prune: B %d is negative", B);
  if (T > 0 && B == 0) return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_prune: %d tokens but no sequence", T);
  if (!cu_seqlens || !new_cu_seqlens) return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_prune: cu_seqlens / new_cu_seqlens is NULL");
  if (T > 0 && (!probs || !is_visual || !kept_idx))
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_prune: probs / is_visual / kept_idx is NULL");
  const bool merging = params->gamma > 0.0f;
  if (merging && T > 0 && (!x_in || !x_merged))
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_prune: gamma > 0 needs x_in and x_merged");
  if (!merging && (x_in || x_merged || is_merged))
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_prune: x_in / x_merged / is_merged belong to window merging (gamma > 0) and must be NULL without it");
  if (!aligned16(x_in) || !aligned16(x_merged))
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_prune: x_in / x_merged not 16-byte aligned");
  if ((rc = check_ws(ctx, ws, ws_bytes, T, B)) != FMOE_OK) return rc;
  const fmoe_ws_layout L = fmoe_layout(ctx, T, B);
  return launch_prune(ctx, params, probs, is_visual, cu_seqlens, B, T, attn_importance, kept_idx,
                      new_cu_seqlens, scores, nullptr, x_in, x_merged, is_merged, ws, L,
                      static_cast<hipStream_t>(stream));
}

int fmoe_permute(fmoe_ctx* ctx, const int32_t* topk_idx, const int32_t* kept_idx, int32_t n_kept,
                 const int32_t* n_kept_dev, int32_t* expert_offsets, int32_t* perm_src,
                 int32_t* inv_perm, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_ctx(ctx, false);
  if (rc != FMOE_OK) return rc;
  if ((rc = check_tokens(n_kept)) != FMOE_OK) return rc;
  if (!expert_offsets) return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_permute: expert_offsets is NULL");
  if (n_kept > 0 && ctx->kmax > 0 && (!topk_idx || !perm_src || !inv_perm))
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_permute: topk_idx / perm_src / inv_perm is NULL");
  if ((rc = check_ws(ctx, ws, ws_bytes, n_kept, 1)) != FMOE_OK) return rc;
  const fmoe_ws_layout L = fmoe_layout(ctx, n_kept, 1);
  return launch_permute(ctx, topk_idx, kept_idx, n_kept, n_kept_dev, expert_offsets, perm_src,
                        inv_perm, ws, L, false, static_cast<hipStream_t>(stream));
}

int fmoe_expert_ffn(fmoe_ctx* ctx, const void* x, const int32_t* kept_idx, int32_t n_kept,
                    const int32_t* n_kept_dev, const int32_t* expert_offsets,
                    const int32_t* perm_src, void* y, void* y_shared, void* ws, size_t ws_bytes,
                    void* stream) {
  int rc = check_ctx(ctx, false);
  if (rc != FMOE_OK) return rc;
  if ((rc = check_tokens(n_kept)) != FMOE_OK) return rc;
  if ((rc = check_ffn_extent(ctx, n_kept, "fmoe_expert_ffn")) != FMOE_OK) return rc;
  if ((rc = check_ctx(ctx, true)) != FMOE_OK) return rc;
  if (n_kept == 0) return FMOE_OK;
  if (!x) return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_expert_ffn: x is NULL");
  if (ctx->kmax > 0 && (!expert_offsets || !perm_src || !y))
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_expert_ffn: expert_offsets / perm_src / y is NULL");
  if (ctx->cfg.n_shared > 0 && !y_shared)
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_expert_ffn: y_shared is NULL but n_shared = %d", ctx->cfg.n_shared);
  if (!aligned16(x) || !aligned16(y) || !aligned16(y_shared))
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_expert_ffn: x / y / y_shared not 16-byte aligned");
  if ((rc = check_ws(ctx, ws, ws_bytes, n_kept, 1)) != FMOE_OK) return rc;
  const fmoe_ws_layout L = fmoe_layout(ctx, n_kept, 1);
  return launch_expert_ffn(ctx, x, kept_idx, n_kept, n_kept_dev, expert_offsets, perm_src, y,
                           ctx->cfg.n_shared > 0 ? y_shared : nullptr, ws, L, false,
                           static_cast<hipStream_t>(stream));
}

int fmoe_combine(fmoe_ctx* ctx, const void* y, const void* y_shared, const int32_t* inv_perm,
                 const float* topk_gate, const int32_t* kept_idx, int32_t n_kept,
                 const int32_t* n_kept_dev, const void* residual, void* out, void* stream) {
  int rc = check_ctx(ctx, false);
  if (rc != FMOE_OK) return rc;
  if ((rc = check_tokens(n_kept)) != FMOE_OK) return rc;
  if (n_kept == 0) return FMOE_OK;
  if (!out) return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_combine: out is NULL");
  if (ctx->kmax > 0 && (!y || !inv_perm || !topk_gate))
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_combine: y / inv_perm / topk_gate is NULL");
  if (ctx->cfg.n_shared > 0 && !y_shared)
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_combine: y_shared is NULL but n_shared = %d", ctx->cfg.n_shared);
  if (!aligned16(y) || !aligned16(y_shared) || !aligned16(residual) || !aligned16(out))
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_combine: tensor pointers must be 16-byte aligned");
  return launch_combine(ctx, y, ctx->cfg.n_shared > 0 ? y_shared : nullptr, inv_perm, topk_gate,
                        kept_idx, n_kept, n_kept_dev, residual, out, static_cast<hipStream_t>(stream));
}

int fmoe_layer_forward(fmoe_ctx* ctx, const fmoe_prune_params* params, const void* x,
                       const uint8_t* is_visual, const int32_t* cu_seqlens, int32_t B, int32_t T,
                       const float* attn_importance, int add_residual, void* out,
                       int32_t* kept_idx, int32_t* new_cu_seqlens, uint8_t* is_visual_out,
                       void* ws, size_t ws_bytes, void* stream) {
  int rc = check_ctx(ctx, false);
  if (rc != FMOE_OK) return rc;
  if ((rc = check_tokens(T)) != FMOE_OK) return rc;
  if ((rc = check_ffn_extent(ctx, T, "fmoe_layer_forward")) != FMOE_OK) return rc;
  if ((rc = check_ctx(ctx, true)) != FMOE_OK) return rc;
  if (B < 0) return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_layer_forward: B %d is negative", B);
  if (T > 0 && B == 0) return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_layer_forward: %d tokens but no sequence", T);
  if (!cu_seqlens || !new_cu_seqlens)
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_layer_forward: cu_seqlens / new_cu_seqlens is NULL");
  if (T > 0 && (!x || !is_visual || !out || !kept_idx))
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_layer_forward: x / is_visual / out / kept_idx is NULL");
  if (!aligned16(x) || !aligned16(out))
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_layer_forward: x / out not 16-byte aligned");
  const bool do_prune = params && params->prune_mode != 0 && params->retention < 1.0f;
  if (params && (rc = check_prune(params)) != FMOE_OK) return rc;
  if ((rc = check_ws(ctx, ws, ws_bytes, T, B)) != FMOE_OK) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const fmoe_ws_layout L = fmoe_layout(ctx, T, B);
  char* base = static_cast<char*>(ws);
  float* probs = reinterpret_cast<float*>(base + L.probs);
  int32_t* topk_idx = reinterpret_cast<int32_t*>(base + L.topk_idx);
  float* topk_gate = reinterpret_cast<float*>(base + L.topk_gate);
  int32_t* expert_offsets = reinterpret_cast<int32_t*>(base + L.expert_offsets);
  int32_t* perm_src = reinterpret_cast<int32_t*>(base + L.perm_src);
  int32_t* inv_perm = reinterpret_cast<int32_t*>(base + L.inv_perm);
  void* y = base + L.y;
  void* y_shared = ctx->cfg.n_shared > 0 ? base + L.y_shared : nullptr;

  const bool merging = do_prune && params->gamma > 0.0f;
  const bool merge_after = merging && params->prune_mode == 2;
  const bool small = !merging && T > 0 && dispatch_small_fits(T, do_prune ? params->window : 1, do_prune);
  // with merging the pruning decisions take the general kernels, but a small batch still gets its
  // permutation and tile lists from the single-workgroup kernel
  const bool small_merge = merging && T > 0 && dispatch_small_fits(T, 1, false);
  // whenever the layer prunes, the router's launch carries the per-sequence ordinal blocks
  fmoe_ordinals_job ord{};
  if (do_prune && T > 0)
    ord = fmoe_ordinals_job{cu_seqlens, B, reinterpret_cast<int32_t*>(base + L.vis_ord),
                            reinterpret_cast<int32_t*>(base + L.vis_tok),
                            reinterpret_cast<int32_t*>(base + L.seq_nv)};
  if ((rc = launch_route(ctx, x, is_visual, T, do_prune ? probs : nullptr, topk_idx, topk_gate, ord, s)) != FMOE_OK)
    return rc;
  const int32_t* kept = nullptr;
  const int32_t* n_dev = nullptr;
  if (small) {
    // a few thousand tokens: scores, then one block for the whole prune/permute chain
    if ((rc = launch_prune_dispatch_small(ctx, params, do_prune, probs, is_visual, cu_seqlens, B, T,
                                          attn_importance, topk_idx, kept_idx, new_cu_seqlens,
                                          is_visual_out, expert_offsets, perm_src, inv_perm, ws, L, s)) != FMOE_OK)
      return rc;
    if (do_prune) {
      kept = kept_idx;
      n_dev = new_cu_seqlens + B;
    }
    if ((rc = launch_expert_ffn(ctx, x, kept, T, n_dev, expert_offsets, perm_src, y, y_shared, ws, L, true, s)) != FMOE_OK)
      return rc;
    return launch_combine(ctx, y, y_shared, inv_perm, topk_gate, kept, T, n_dev, add_residual ? x : nullptr,
                          out, s);
  }
  if (merge_after) {
    // Window merging after the layer (Sec. 3.2.3 applied to the layer's output, the tensor that is
    // compacted here): a merged token is built from the output rows of all tokens of its window, so
    // the experts run on every token; the windows are then scored on this layer's probabilities and
    // the output rows are compacted, merged windows replaced by their merged row (Eq.16-18).
    if (T == 0)
      return launch_identity_kept(is_visual, cu_seqlens, B, T, kept_idx, new_cu_seqlens, is_visual_out, s);
    void* full = base + L.x_merged;   // [T,d]: the layer's output before compaction
    if ((rc = launch_permute(ctx, topk_idx, nullptr, T, nullptr, expert_offsets, perm_src, inv_perm, ws, L, true, s)) != FMOE_OK)
      return rc;
    if ((rc = launch_expert_ffn(ctx, x, nullptr, T, nullptr, expert_offsets, perm_src, y, y_shared, ws, L, true, s)) != FMOE_OK)
      return rc;
    if ((rc = launch_combine(ctx, y, y_shared, inv_perm, topk_gate, nullptr, T, nullptr, add_residual ? x : nullptr,
                             full, s)) != FMOE_OK)
      return rc;
    return launch_prune(ctx, params, probs, is_visual, cu_seqlens, B, T, attn_importance, kept_idx,
                        new_cu_seqlens, nullptr, is_visual_out, full, out, nullptr, ws, L, s, true);
  }
  if (merging) {
    // Window merging changes the layer input: the kept rows are gathered into a compact tensor (merged
    // windows replaced by their merged token, Eq.16-18), every kept token is routed again on it (only
    // the merged ones can come out differently) and the rest of the layer runs on that tensor.
    if (T == 0)
      return launch_identity_kept(is_visual, cu_seqlens, B, T, kept_idx, new_cu_seqlens, is_visual_out, s);
    void* xm = base + L.x_merged;
    uint8_t* vis_m = is_visual_out ? is_visual_out : reinterpret_cast<uint8_t*>(base + L.vis_out);
    if ((rc = launch_prune(ctx, params, probs, is_visual, cu_seqlens, B, T, attn_importance, kept_idx,
                           new_cu_seqlens, nullptr, vis_m, x, xm, nullptr, ws, L, s, true)) != FMOE_OK)
      return rc;
    n_dev = new_cu_seqlens + B;
    if ((rc = launch_route(ctx, xm, vis_m, T, nullptr, topk_idx, topk_gate, fmoe_ordinals_job{}, s, n_dev)) != FMOE_OK)
      return rc;
    if (small_merge)
      rc = launch_prune_dispatch_small(ctx, params, false, nullptr, vis_m, new_cu_seqlens, B, T, nullptr, topk_idx,
                                       kept_idx, new_cu_seqlens, nullptr, expert_offsets, perm_src, inv_perm,
                                       ws, L, s, n_dev, false);
    else
      rc = launch_permute(ctx, topk_idx, nullptr, T, n_dev, expert_offsets, perm_src, inv_perm, ws, L, true, s);
    if (rc != FMOE_OK) return rc;
    if ((rc = launch_expert_ffn(ctx, xm, nullptr, T, n_dev, expert_offsets, perm_src, y, y_shared, ws, L, true, s)) != FMOE_OK)
      return rc;
    return launch_combine(ctx, y, y_shared, inv_perm, topk_gate, nullptr, T, n_dev, add_residual ? xm : nullptr,
                          out, s);
  }
  if (do_prune) {
    rc = launch_prune(ctx, params, probs, is_visual, cu_seqlens, B, T, attn_importance, kept_idx,
                      new_cu_seqlens, nullptr, is_visual_out, nullptr, nullptr, nullptr, ws, L, s, true);
    kept = kept_idx;
    n_dev = new_cu_seqlens + B;
  } else {
    rc = launch_identity_kept(is_visual, cu_seqlens, B, T, kept_idx, new_cu_seqlens, is_visual_out, s);
  }
  if (rc != FMOE_OK) return rc;
  if (T == 0) return FMOE_OK;
  if ((rc = launch_permute(ctx, topk_idx, kept, T, n_dev, expert_offsets, perm_src, inv_perm, ws, L, true, s)) != FMOE_OK)
    return rc;
  if ((rc = launch_expert_ffn(ctx, x, kept, T, n_dev, expert_offsets, perm_src, y, y_shared, ws, L, true, s)) != FMOE_OK)
    return rc;
  return launch_combine(ctx, y, y_shared, inv_perm, topk_gate, kept, T, n_dev, add_residual ? x : nullptr,
                        out, s);
}

int fmoe_adjacent_similarity(fmoe_ctx* ctx, const float* probs, const uint8_t* is_visual,
                             const int32_t* cu_seqlens, int32_t B, int32_t T, float* pair_sim, float* mean,
                             int32_t* count, void* stream) {
  int rc = check_ctx(ctx, false);
  if (rc != FMOE_OK) return rc;
  if ((rc = check_tokens(T)) != FMOE_OK) return rc;
  if (B < 0) return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_adjacent_similarity: B %d is negative", B);
  if (!cu_seqlens || !mean || !count)
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_adjacent_similarity: cu_seqlens / mean / count is NULL");
  if (T > 0 && (!probs || !is_visual || !pair_sim))
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_adjacent_similarity: probs / is_visual / pair_sim is NULL");
  if (T > 0 && B == 0)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_adjacent_similarity: %d tokens but no sequence", T);
  return launch_adjacent_similarity(probs, is_visual, cu_seqlens, B, T, ctx->cfg.n_experts, pair_sim, mean,
                                    count, static_cast<hipStream_t>(stream));
}

int fmoe_magnitude_stability(fmoe_ctx* ctx, const void* y, int32_t M, const int32_t* M_dev,
                             const int32_t* perm_src, const int32_t* kept_idx, const uint8_t* is_visual,
                             float* row_norm, float* stats, void* stream) {
  int rc = check_ctx(ctx, false);
  if (rc != FMOE_OK) return rc;
  if (M < 0) return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_magnitude_stability: M %d is negative", M);
  if (!stats) return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_magnitude_stability: stats is NULL");
  if (M > 0 && (!y || !perm_src || !is_visual || !row_norm))
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_magnitude_stability: y / perm_src / is_visual / row_norm is NULL");
  return launch_magnitude_stability(ctx, y, M, M_dev, perm_src, kept_idx, is_visual, row_norm, stats,
                                    static_cast<hipStream_t>(stream));
}

int fmoe_row_cosine(fmoe_ctx* ctx, const void* a, const void* b, int32_t n, const int32_t* n_dev, float* out,
                    void* stream) {
  int rc = check_ctx(ctx, false);
  if (rc != FMOE_OK) return rc;
  if ((rc = check_tokens(n)) != FMOE_OK) return rc;
  if (n > 0 && (!a || !b || !out)) return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_row_cosine: a / b / out is NULL");
  return launch_row_cosine(ctx, a, b, n, n_dev, out, static_cast<hipStream_t>(stream));
}

int fmoe_gate_cosine(fmoe_ctx* ctx, const float* gates, int32_t T, int32_t K, int32_t m, float* out,
                     void* stream) {
  int rc = check_ctx(ctx, false);
  if (rc != FMOE_OK) return rc;
  if ((rc = check_tokens(T)) != FMOE_OK) return rc;
  if (K < 1 || m < 0 || m > K)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_gate_cosine: need K >= 1 and 0 <= m <= K (K %d, m %d)", K, m);
  if (T > 0 && (!gates || !out)) return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_gate_cosine: gates / out is NULL");
  return launch_gate_cosine(gates, T, K, m, out, static_cast<hipStream_t>(stream));
}

int fmoe_flops_ratios(const fmoe_flops_model* m, double* ratios) {
  if (!m || !ratios) return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_flops_ratios: model / ratios is NULL");
  if (m->n_layers < 1 || m->n_dense < 0 || m->n_dense > m->n_layers)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_flops_ratios: need n_layers >= 1 and 0 <= n_dense <= n_layers (%d, %d)",
                     m->n_layers, m->n_dense);
  if (!(m->H > 0.0) || !(m->S_m > 0.0) || !(m->E > 0.0) || !(m->K > 0.0) || !(m->K_v >= 0.0) || !(m->L_v > 0.0) ||
      (m->n_dense > 0 && !(m->S > 0.0)))
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_flops_ratios: H, S_m, E, K, L_v (and S with dense layers) must be positive, K_v >= 0");
  if (!(m->beta > 0.0 && m->beta <= 1.0))
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_flops_ratios: beta %g is not in (0,1]", m->beta);
  if (m->l_v < 0 || m->l_v > m->n_layers)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_flops_ratios: l_v %d is not in 0..%d", m->l_v, m->n_layers);
  if (m->n_prune < 0 || m->n_prune > 8)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_flops_ratios: n_prune %d is not in 0..8", m->n_prune);
  for (int s = 0; s < m->n_prune; ++s)
    if (m->prune_layers[s] < 0 || m->prune_layers[s] >= m->n_layers || (s > 0 && m->prune_layers[s] <= m->prune_layers[s - 1]))
      return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_flops_ratios: prune layers must ascend inside 0..%d", m->n_layers - 1);
  // one pass over the layers, each priced at the vision length and the expert count in force there
  const double H = m->H;
  auto attention = [&](double x) { return 4.0 * x * x * H + 8.0 * x * H * H; };
  auto ffn = [&](int layer, double x, double k) {
    return layer < m->n_dense ? 6.0 * x * H * m->S : 2.0 * x * H * m->E + 6.0 * x * H * m->S_m * k;
  };
  double base = 0.0, pruned = 0.0, reduced = 0.0, both = 0.0, x = m->L_v;
  int stage = 0;
  for (int i = 0; i < m->n_layers; ++i) {
    const double k = i >= m->l_v ? m->K_v : m->K;
    base += attention(m->L_v) + ffn(i, m->L_v, m->K);
    pruned += attention(x) + ffn(i, x, m->K);
    reduced += attention(m->L_v) + ffn(i, m->L_v, k);
    both += attention(x) + ffn(i, x, k);
    if (stage < m->n_prune && m->prune_layers[stage] == i) {   // acts on the layers after this one
      x *= m->beta;
      ++stage;
    }
  }
  ratios[0] = pruned / base;
  ratios[1] = reduced / base;
  ratios[2] = both / base;
  return FMOE_OK;
}

int fmoe_profile_slots(void) { return SLOT_COUNT; }

const char* fmoe_profile_name(int slot) {
  // kernel symbols (the two expert GEMMs: bf16 symbol; fp32 contexts run grouped_gemm_kernel)
  static const char* names[SLOT_COUNT] = {
      "route_kernel", "seq_ordinals_kernel", "window_score_kernel", "select_kernel", "compact_flag_kernel+compact_write_kernel",
      "prune_dispatch_small_kernel", "permute_count_kernel", "permute_scan_kernel",
      "permute_scatter_kernel", "build_tiles_kernel", "ffn_stream_kernel<true>",
      "ffn_stream_kernel<false>", "combine_kernel", "ffn_dense_kernel<true>", "ffn_dense_kernel<false>"};
  return (slot >= 0 && slot < SLOT_COUNT) ? names[slot] : "";
}

int fmoe_profile_enable(fmoe_ctx* ctx, int enable) {
  int rc = check_ctx(ctx, false);
  if (rc != FMOE_OK) return rc;
  if (enable && !ctx->prof) {
    fmoe_prof* p = new (std::nothrow) fmoe_prof();
    if (!p) return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_profile_enable: out of host memory");
    std::memset(p, 0, sizeof(*p));
    for (int i = 0; i < SLOT_COUNT; ++i) {
      FMOE_HIP_CHECK(hipEventCreate(&p->beg[i]));
      FMOE_HIP_CHECK(hipEventCreate(&p->end[i]));
    }
    ctx->prof = p;
  }
  if (ctx->prof) ctx->prof->on = enable != 0;
  return FMOE_OK;
}

int fmoe_profile_read(fmoe_ctx* ctx, float* ms) {
  int rc = check_ctx(ctx, false);
  if (rc != FMOE_OK) return rc;
  if (!ms) return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_profile_read: ms is NULL");
  if (!ctx->prof) return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_profile_read: profiling was never enabled");
  for (int i = 0; i < SLOT_COUNT; ++i) {
    ms[i] = -1.0f;
    if (!ctx->prof->used[i]) continue;
    FMOE_HIP_CHECK(hipEventSynchronize(ctx->prof->end[i]));
    FMOE_HIP_CHECK(hipEventElapsedTime(&ms[i], ctx->prof->beg[i], ctx->prof->end[i]));
    ctx->prof->used[i] = false;
  }
  return FMOE_OK;
}

}  // extern "C"
