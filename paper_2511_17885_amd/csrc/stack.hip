// The layer stack: x <- x + MoE_l(x) with the per-layer expert activation of Sec. 3.1 (reduced K_v
// from layer l_v on) and pruning stages at chosen layers (Sec. 3.2; App. D: several stages of equal
// per-stage ratio).  Host-side sequencing of fmoe_layer_forward calls plus two tiny kernels for the
// index bookkeeping; the token counts after a stage follow on the host from the exact budget rule of
// Sec. 3.2.3, so nothing is read back from the device.

#include <cmath>
#include <vector>

#include "common.h"

namespace {

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

// eta = floor(r*N_v + 1/2) in fp64 with r at fp32 precision, clamped to [min(1,N_v), N_v]
// (Sec. 3.2.3; the same expression as the kernels' token_budget)
inline int32_t host_token_budget(int32_t nv, float retention) {
  int32_t eta = (int32_t)std::floor((double)retention * (double)nv + 0.5);
  eta = eta > nv ? nv : eta;
  const int32_t lo = nv < 1 ? nv : 1;
  return eta < lo ? lo : eta;
}

inline bool stage_active(const fmoe_prune_params& p) { return p.prune_mode != 0 && p.retention < 1.0f; }

// Positions in the input batch of the tokens a stage kept: total_out[p] = total_in[kept[p]]
// (total_in == nullptr: the stage saw the input batch itself).
__global__ void compose_kept_kernel(const int32_t* __restrict__ kept, const int32_t* __restrict__ total_in,
                                    int n_cap, const int32_t* __restrict__ n_dev, int t_in,
                                    int32_t* __restrict__ total_out) {
  const int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= resolve_count(n_cap, n_dev)) return;
  int k = kept[p];
  k = k < 0 ? 0 : (k >= t_in ? t_in - 1 : k);
  total_out[p] = total_in ? total_in[k] : k;
}

// The stack's index outputs: kept_idx (identity when no stage ran), sequence bounds, modality mask.
__global__ void stack_finish_kernel(const int32_t* __restrict__ total, const int32_t* __restrict__ cu,
                                    const uint8_t* __restrict__ vis, int n, int B,
                                    int32_t* __restrict__ kept_out, int32_t* __restrict__ cu_out,
                                    uint8_t* __restrict__ vis_out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    kept_out[i] = total ? total[i] : i;
    if (vis_out != nullptr) vis_out[i] = vis[i];
  }
  if (i <= B && cu_out != cu) cu_out[i] = cu[i];
}

struct stack_layout {
  size_t xa, xb;          // activation ping-pong [T, d]
  size_t vis_a, vis_b;    // modality masks
  size_t cu_a, cu_b;      // sequence bounds
  size_t kept;            // a layer's kept_idx
  size_t tot_a, tot_b;    // composed positions in the input batch
  size_t layer_ws;        // workspace handed to the layers
  size_t total;
};

int check_stack(fmoe_ctx* const* layers, const fmoe_layer_plan* plan, int32_t n_layers) {
  if (!layers || !plan) return fmoe_fail(FMOE_ERR_NULL_PTR, "stack: layers / plan is NULL");
  if (n_layers < 1) return fmoe_fail(FMOE_ERR_INVALID_ARG, "stack: n_layers %d < 1", n_layers);
  for (int l = 0; l < n_layers; ++l) {
    if (!layers[l]) return fmoe_fail(FMOE_ERR_NULL_PTR, "stack: layers[%d] is NULL", l);
    const fmoe_config& c = layers[l]->cfg;
    const fmoe_config& c0 = layers[0]->cfg;
    if (c.d_model != c0.d_model || c.dtype != c0.dtype || layers[l]->device != layers[0]->device)
      return fmoe_fail(FMOE_ERR_BAD_SHAPE, "stack: layer %d differs from layer 0 in d_model, dtype or device", l);
    if (plan[l].k_text < 0 || plan[l].k_visual < 0 || plan[l].k_text > c.n_experts || plan[l].k_visual > c.n_experts)
      return fmoe_fail(FMOE_ERR_INVALID_ARG, "stack: plan[%d] needs 0 <= k <= n_experts (k_text %d, k_visual %d)", l,
                       plan[l].k_text, plan[l].k_visual);
    if (plan[l].k_text > FMOE_MAX_TOPK || plan[l].k_visual > FMOE_MAX_TOPK)
      return fmoe_fail(FMOE_ERR_UNSUPPORTED, "stack: plan[%d] top-k above %d", l, FMOE_MAX_TOPK);
  }
  return FMOE_OK;
}

// Largest per-layer workspace over the plan: layer l is sized for the tokens that can reach it (the
// capacity T; stages only shrink the batch) and for its own Kmax.
size_t max_layer_ws(fmoe_ctx* const* layers, const fmoe_layer_plan* plan, int32_t n_layers, int32_t T, int32_t B) {
  size_t need = 0;
  for (int l = 0; l < n_layers; ++l) {
    fmoe_ctx probe = *layers[l];   // host-side copy: only cfg / kmax are read by the layout
    probe.cfg.k_text = plan[l].k_text;
    probe.cfg.k_visual = plan[l].k_visual;
    probe.kmax = plan[l].k_text > plan[l].k_visual ? plan[l].k_text : plan[l].k_visual;
    const size_t b = fmoe_layout(&probe, T, B).total;
    need = b > need ? b : need;
  }
  return need;
}

stack_layout make_stack_layout(fmoe_ctx* const* layers, const fmoe_layer_plan* plan, int32_t n_layers, int32_t T,
                               int32_t B) {
  const size_t Tc = T > 0 ? (size_t)T : 1, Bc = B > 0 ? (size_t)B : 1;
  const size_t es = layers[0]->cfg.dtype == FMOE_BF16 ? 2 : 4;
  const size_t row = (size_t)layers[0]->cfg.d_model * es;
  stack_layout L{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  L.xa = take(Tc * row);
  L.xb = take(Tc * row);
  L.vis_a = take(Tc);
  L.vis_b = take(Tc);
  L.cu_a = take((Bc + 1) * 4);
  L.cu_b = take((Bc + 1) * 4);
  L.kept = take(Tc * 4);
  L.tot_a = take(Tc * 4);
  L.tot_b = take(Tc * 4);
  L.layer_ws = take(max_layer_ws(layers, plan, n_layers, T, B));
  L.total = off;
  return L;
}

}  // namespace

extern "C" {

int fmoe_kept_counts(const int32_t* visual_lens, int32_t B, float retention, int32_t* kept_visual_lens) {
  if (B < 0) return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_kept_counts: B %d is negative", B);
  if (B > 0 && (!visual_lens || !kept_visual_lens))
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_kept_counts: visual_lens / kept_visual_lens is NULL");
  if (!(retention > 0.0f) || retention > 1.0f)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_kept_counts: retention %g outside (0,1]", (double)retention);
  for (int b = 0; b < B; ++b)
    if (visual_lens[b] < 0)
      return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_kept_counts: visual_lens[%d] = %d is negative", b, visual_lens[b]);
  for (int b = 0; b < B; ++b) kept_visual_lens[b] = host_token_budget(visual_lens[b], retention);
  return FMOE_OK;
}

int fmoe_stage_retention(float retention, int32_t stages, float* beta) {
  if (!beta) return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_stage_retention: beta is NULL");
  if (!(retention > 0.0f) || retention > 1.0f)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_stage_retention: retention %g outside (0,1]", (double)retention);
  if (stages < 1) return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_stage_retention: stages %d < 1", stages);
  *beta = (float)std::pow((double)retention, 1.0 / (double)stages);
  return FMOE_OK;
}

int fmoe_stack_plan(int32_t n_layers, int32_t K, int32_t K_v, int32_t l_v, const int32_t* prune_layers,
                    int32_t n_stages, const fmoe_prune_params* stage, fmoe_layer_plan* plan) {
  if (!plan) return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_stack_plan: plan is NULL");
  if (n_layers < 1) return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_stack_plan: n_layers %d < 1", n_layers);
  if (K < 0 || K_v < 0) return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_stack_plan: K %d / K_v %d is negative", K, K_v);
  if (l_v < 0 || l_v > n_layers)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_stack_plan: l_v %d is not in 0..%d", l_v, n_layers);
  if (n_stages < 0 || n_stages > n_layers)
    return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_stack_plan: n_stages %d is not in 0..%d", n_stages, n_layers);
  if (n_stages > 0 && (!prune_layers || !stage))
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_stack_plan: prune_layers / stage is NULL with %d stages", n_stages);
  for (int s = 0; s < n_stages; ++s)
    if (prune_layers[s] < 0 || prune_layers[s] >= n_layers || (s > 0 && prune_layers[s] <= prune_layers[s - 1]))
      return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_stack_plan: prune layers must ascend inside 0..%d", n_layers - 1);
  float beta = 1.0f;
  if (n_stages > 0) {
    const int rc = fmoe_stage_retention(stage->retention, n_stages, &beta);
    if (rc != FMOE_OK) return rc;
  }
  int s = 0;
  for (int l = 0; l < n_layers; ++l) {
    plan[l].k_text = K;
    plan[l].k_visual = l >= l_v ? K_v : K;
    fmoe_prune_params none{};
    none.retention = 1.0f; none.window = 1; none.alpha = 1.0f;
    plan[l].prune = none;
    if (s < n_stages && prune_layers[s] == l) {
      plan[l].prune = *stage;
      plan[l].prune.retention = beta;
      ++s;
    }
  }
  return FMOE_OK;
}

size_t fmoe_stack_workspace_bytes(fmoe_ctx* const* layers, const fmoe_layer_plan* plan, int32_t n_layers,
                                  int32_t max_tokens, int32_t max_seqs) {
  if (check_stack(layers, plan, n_layers) != FMOE_OK) return 0;
  return make_stack_layout(layers, plan, n_layers, max_tokens, max_seqs).total;
}

int fmoe_stack_forward(fmoe_ctx* const* layers, const fmoe_layer_plan* plan, int32_t n_layers,
                       const void* x, const uint8_t* is_visual, const int32_t* cu_seqlens,
                       const int32_t* visual_lens, const int32_t* text_lens, int32_t B, int32_t T,
                       const float* const* attn, void* out, int32_t* kept_idx, int32_t* new_cu_seqlens,
                       uint8_t* is_visual_out, int32_t* n_out, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_stack(layers, plan, n_layers);
  if (rc != FMOE_OK) return rc;
  if (T < 0 || B < 0) return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_stack_forward: T %d / B %d is negative", T, B);
  if (!cu_seqlens || !new_cu_seqlens)
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_stack_forward: cu_seqlens / new_cu_seqlens is NULL");
  if (T > 0 && (!x || !is_visual || !out || !kept_idx))
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_stack_forward: x / is_visual / out / kept_idx is NULL");
  if (B > 0 && (!visual_lens || !text_lens))
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_stack_forward: visual_lens / text_lens is NULL");
  std::vector<int32_t> nv(visual_lens, visual_lens + B);
  long long sum = 0, text = 0;
  for (int b = 0; b < B; ++b) {
    if (visual_lens[b] < 0 || text_lens[b] < 0)
      return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_stack_forward: negative length in sequence %d", b);
    sum += (long long)visual_lens[b] + text_lens[b];
    text += text_lens[b];
  }
  if (sum != T)
    return fmoe_fail(FMOE_ERR_BAD_SHAPE, "fmoe_stack_forward: visual_lens + text_lens add up to %lld tokens, T = %d", sum, T);
  if (!ws) return fmoe_fail(FMOE_ERR_WORKSPACE, "workspace is NULL");
  if (reinterpret_cast<uintptr_t>(ws) & 255u) return fmoe_fail(FMOE_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  const stack_layout L = make_stack_layout(layers, plan, n_layers, T, B);
  if (ws_bytes < L.total)
    return fmoe_fail(FMOE_ERR_WORKSPACE, "stack workspace has %zu bytes, %zu needed for %d tokens / %d sequences / %d layers",
                     ws_bytes, L.total, T, B, n_layers);
  hipStream_t s = static_cast<hipStream_t>(stream);
  char* base = static_cast<char*>(ws);
  void* xbuf[2] = {base + L.xa, base + L.xb};
  uint8_t* vbuf[2] = {reinterpret_cast<uint8_t*>(base + L.vis_a), reinterpret_cast<uint8_t*>(base + L.vis_b)};
  int32_t* cbuf[2] = {reinterpret_cast<int32_t*>(base + L.cu_a), reinterpret_cast<int32_t*>(base + L.cu_b)};
  int32_t* tbuf[2] = {reinterpret_cast<int32_t*>(base + L.tot_a), reinterpret_cast<int32_t*>(base + L.tot_b)};
  int32_t* layer_kept = reinterpret_cast<int32_t*>(base + L.kept);
  const size_t layer_ws_bytes = L.total - L.layer_ws;

  const void* cur_x = x;
  const uint8_t* cur_vis = is_visual;
  const int32_t* cur_cu = cu_seqlens;
  const int32_t* cur_total = nullptr;   // nullptr: rows are still the input batch's tokens
  int cur_T = T;
  int xi = 0, vi = 0, ci = 0, ti = 0;
  for (int l = 0; l < n_layers; ++l) {
    fmoe_ctx* ctx = layers[l];
    if ((rc = fmoe_set_topk(ctx, plan[l].k_text, plan[l].k_visual)) != FMOE_OK) return rc;
    const bool stage = stage_active(plan[l].prune);
    void* dst = (l == n_layers - 1) ? out : xbuf[xi];
    int32_t* cu_dst = cbuf[ci];
    uint8_t* vis_dst = stage ? vbuf[vi] : nullptr;
    rc = fmoe_layer_forward(ctx, stage ? &plan[l].prune : nullptr, cur_x, cur_vis, cur_cu, B, cur_T,
                            (stage && attn) ? attn[l] : nullptr, 1, dst, layer_kept, cu_dst, vis_dst,
                            base + L.layer_ws, layer_ws_bytes, stream);
    if (rc != FMOE_OK) return rc;
    cur_x = dst;
    if (l != n_layers - 1) xi ^= 1;
    if (stage) {
      int next_T = (int)text;
      for (int b = 0; b < B; ++b) {
        nv[b] = host_token_budget(nv[b], plan[l].prune.retention);
        next_T += nv[b];
      }
      if (next_T > 0) {
        hipLaunchKernelGGL(compose_kept_kernel, dim3((next_T + 255) / 256), dim3(256), 0, s, layer_kept, cur_total,
                           next_T, cu_dst + B, cur_T, tbuf[ti]);
        FMOE_HIP_CHECK(hipGetLastError());
      }
      cur_total = tbuf[ti];
      ti ^= 1;
      cur_vis = vis_dst;
      vi ^= 1;
      cur_cu = cu_dst;
      ci ^= 1;
      cur_T = next_T;
    }
  }
  const int n_fin = cur_T > B + 1 ? cur_T : B + 1;
  hipLaunchKernelGGL(stack_finish_kernel, dim3((n_fin + 255) / 256), dim3(256), 0, s, cur_total, cur_cu, cur_vis,
                     cur_T, B, kept_idx, new_cu_seqlens, is_visual_out);
  FMOE_HIP_CHECK(hipGetLastError());
  if (n_out) *n_out = cur_T;
  return FMOE_OK;
}

}  // extern "C"
