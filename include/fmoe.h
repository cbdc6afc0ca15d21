/* fmoe.h -- C ABI of the MI355X (gfx950) MoE-layer prefill library.
 *
 * The library computes one Mixture-of-Experts layer forward over a packed batch of
 * [visual tokens, text tokens] sequences with the two FastMMoE mechanisms in it:
 * modality-dependent top-k routing with gate renormalisation (paper Sec. 3.1) and routing-aware
 * sliding-window visual-token pruning (paper Sec. 3.2).  Symbols follow the paper: H = d_model,
 * E = routed experts, S_m = d_ffn, K = k_text, K_v = k_visual, N_s = n_shared, W = window.
 *
 * Conventions
 *  - Plain C; every function returns FMOE_OK (0) or a negative fmoe_status; nothing throws or
 *    aborts.  fmoe_last_error() gives a thread-local message for the last failure.
 *  - Every tensor pointer is a DEVICE pointer on the context's GPU unless marked [host].
 *    Tensors are row-major, contiguous, 16-byte aligned, and stay owned by the caller; the
 *    library only borrows them for the duration of the enqueued work.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *    enqueued asynchronously on it; no call synchronises with the host and no hot call
 *    (route / prune / permute / expert_ffn / combine / layer_forward) allocates memory.
 *    Scratch comes from a caller-provided workspace sized by fmoe_workspace_bytes().  A hot call
 *    is a sequence of kernel launches and nothing else (no memset, no copy), so it can be
 *    captured into a HIP graph on `stream` and replayed.
 *  - Data-dependent counts (tokens kept, rows per expert) stay on the device:
 *    new_cu_seqlens[B] holds the number of kept tokens T'; expert_offsets[E] holds the number
 *    of routed rows M.
 *  - "dtype" is the storage type of activations and weights (fp32 or bf16); accumulation is
 *    always fp32.  Router probabilities, gates and window scores are fp32 in a fixed
 *    operation order so that expert ids, the permutation and the kept-token set are
 *    reproducible bit for bit.
 *  - Shape limits: 1 <= E <= 256, Kmax = max(k_text,k_visual) <= 16 and <= E,
 *    d_model % 8 == 0, d_ffn % 8 == 0, d_ffn_shared % 8 == 0, T < 2^24, window <= 64.
 *    Anything else returns FMOE_ERR_UNSUPPORTED.
 */
#ifndef FMOE_H_
#define FMOE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FMOE_OK = 0,
  FMOE_ERR_INVALID_ARG = -1, /* value out of its documented range                  */
  FMOE_ERR_NULL_PTR = -2,    /* a required pointer is NULL                         */
  FMOE_ERR_BAD_SHAPE = -3,   /* sizes inconsistent with the context's config       */
  FMOE_ERR_WORKSPACE = -4,   /* workspace missing, misaligned or too small         */
  FMOE_ERR_UNSUPPORTED = -5, /* valid request outside the implemented shape limits */
  FMOE_ERR_HIP = -6          /* a HIP runtime call failed (launch, attribute, ...) */
} fmoe_status;

typedef enum { FMOE_F32 = 0, FMOE_BF16 = 1 } fmoe_dtype;

typedef struct {
  int32_t d_model;      /* H                                                    */
  int32_t n_experts;    /* E, routed (non-shared) experts                       */
  int32_t d_ffn;        /* S_m, intermediate size of one routed expert          */
  int32_t n_shared;     /* N_s >= 0 always-on shared experts (Eq.4, first sum)  */
  int32_t d_ffn_shared; /* intermediate size of one shared expert               */
  int32_t k_text;       /* K: experts per text token                            */
  int32_t k_visual;     /* K_v: experts per visual token (0 allowed)            */
  int32_t renormalize;  /* 1: gates divided by the sum over the kept experts    */
  int32_t dtype;        /* fmoe_dtype of activations and weights                */
} fmoe_config;

typedef struct {
  float retention;    /* r in (0,1]: keep round(r*N_v) visual tokens per sequence; 1 = off */
  int32_t window;     /* W >= 1 consecutive visual tokens per window (Sec. 3.2.2)          */
  float alpha;        /* weight of routing similarity in the redundancy score (Eq.13)      */
  float gamma;        /* merge rate in [0,1) (Eq.14): at most floor(eta*gamma) windows merged; 0 = off */
  int32_t sim_mode;   /* 0: similarity to the window mean (Eq.9-10); 1: all pairs (Eq.8)   */
  int32_t prune_mode; /* 0: none; 1: before the experts; 2: after the layer.  Without merging the two give
                         the same result (see fmoe_layer_forward); with gamma > 0 mode 1 merges the
                         layer input, mode 2 the layer output                                      */
  int32_t merge_mode; /* merged token: 0 = MLERP (Eq.16-18: mean rescaled to the largest token norm),
                         1 = plain mean (the alternative of the merge-method ablation, Sec. 4)  */
} fmoe_prune_params;

/* Model description for the theoretical FLOPs ratios of App. E (batch size 1, vision tokens only, as in
 * the appendix).  Layers are indexed from 0; the first n_dense layers carry a dense MLP of intermediate
 * size S instead of the experts (DeepSeek-VL2: 1, InternVL3.5: 0).  K and K_v count every active expert
 * of a token, shared ones included (the printed DeepSeek-VL2 savings come out with K = 6 + 2 and
 * K_v = 2 + 2).  Pruning after layer prune_layers[s] multiplies the vision length by beta, so layer i
 * sees L_v * beta^(number of prune layers below i); lengths stay real numbers, as in the appendix. */
typedef struct {
  int32_t n_layers;        /* transformer layers                                                  */
  int32_t n_dense;         /* leading layers with a dense MLP instead of the MoE FFN              */
  double H;                /* hidden size                                                         */
  double S;                /* intermediate size of the dense MLP (unused when n_dense = 0)        */
  double S_m;              /* intermediate size of one expert                                     */
  double E;                /* routed experts (the router term 2*L*H*E)                            */
  double K;                /* active experts per token                                            */
  double K_v;              /* active experts per vision token in layers >= l_v                    */
  int32_t l_v;             /* first layer with reduced activation, 0 .. n_layers (n_layers: none) */
  int32_t n_prune;         /* pruning stages, 0 .. 8                                              */
  int32_t prune_layers[8]; /* ascending layer indices; the stage acts on the layers after it      */
  double beta;             /* per-stage retention in (0,1]                                        */
  double L_v;              /* vision tokens before pruning                                        */
} fmoe_flops_model;

typedef struct fmoe_ctx fmoe_ctx;

/* Library version string, static storage. */
const char* fmoe_version(void);

/* Message for the calling thread's most recent failure ("" if none). [host] */
const char* fmoe_last_error(void);

/* Create a context for one layer shape on GPU `device`.  Validates the config against the
 * shape limits.  The context holds only host-side state and borrowed weight pointers. */
int fmoe_create(fmoe_ctx** out_ctx, const fmoe_config* config, int device);
void fmoe_destroy(fmoe_ctx* ctx);

/* Change K and K_v of an existing context (the per-layer l_v switch of Sec. 3.1).
 * Kmax = max(k_text,k_visual) changes with it, and so do the [*,Kmax] tensor shapes. */
int fmoe_set_topk(fmoe_ctx* ctx, int32_t k_text, int32_t k_visual);

/* Expert selection strategy for tokens with reduced activation (the ablation of Sec. 4, "Selection
 * Strategy for Expert Activation Reduction").  A token whose k (k_text or k_visual) is below k_base
 * first lists its k_base highest-probability experts (ties: lower index) and keeps k of them:
 * strategy 0 = the k highest (TopK: the method itself, the default), 1 = k at random (RandomK),
 * 2 = the k lowest (MinK).  The kept experts stay in list order and the gates are renormalised over
 * them (Eq.5).  RandomK is reproducible: candidate position r of token t (its index in the routed
 * batch) gets the key SplitMix64(seed) output number 16 t + r + 1 and the k smallest keys win.
 * Tokens with k >= k_base are routed as usual.  Affects fmoe_route and fmoe_layer_forward.
 * FMOE_ERR_INVALID_ARG unless 0 <= strategy <= 2 and 0 <= k_base <= min(E, 16). */
int fmoe_set_selection(fmoe_ctx* ctx, int32_t strategy, int32_t k_base, uint64_t seed);

/* Tuning knob of the bf16 expert GEMMs (Eq.4).  The kernel has two shapes: the weight-stream shape (a
 * workgroup = 128 rows x 4 column blocks) for calls that route few rows per expert, and the dense
 * shape (128 rows x 8 column blocks, half the on-chip traffic per flop) from a capacity of 256 routed
 * rows per expert (T * Kmax / E) on.  Both add the products of a dot product in ascending k, so their
 * outputs are bit-identical.  shape 0 = choose by that rule (default), 1 = always weight-stream,
 * 2 = always dense; anything else is FMOE_ERR_INVALID_ARG.  No effect on fp32 contexts. */
int fmoe_set_ffn_shape(fmoe_ctx* ctx, int32_t shape);

/* Register the layer's weights (Eq.1, Eq.4).  Pointers are borrowed until the next call or
 * fmoe_destroy.  router_w [E,H] dtype; router_bias [E] fp32 or NULL (added to the logits
 * before the softmax); w_gate, w_up [E,S_m,H]; w_down [E,H,S_m]; ws_gate, ws_up
 * [N_s,S_s,H]; ws_down [N_s,H,S_s] (NULL iff N_s == 0).  An expert is the three-matrix gated
 * FFN  y = W_down (silu(W_gate x) * (W_up x))  without biases (flop model of App. E).
 * Device allocations (the only ones the library makes; made on the first call, reused by later calls
 * on the same context, freed by fmoe_destroy):
 *  - a private fp32 copy of the router matrix in the router kernel's operand order (E*H*4 bytes
 *    rounded up to 16x16 blocks and whole 128-wide k chunks);
 *  - bf16 contexts only: private copies of all expert weights (routed and shared) in matrix-core
 *    operand order, the same total size as the originals up to zero padding of the reduction
 *    length to 64 and of the output columns to 64 (gate/up) / 128 (down).  The expert GEMMs of a
 *    bf16 context read ONLY these copies: the caller's expert tensors may be freed or changed after
 *    the call returns and the stream has drained, and a later change to them has no effect until
 *    fmoe_set_weights is called again.  A bf16 layer therefore holds its expert weights twice while
 *    the caller keeps the originals.
 * fp32 contexts keep borrowing w_gate .. ws_down until the next call or fmoe_destroy. */
int fmoe_set_weights(fmoe_ctx* ctx, const void* router_w, const float* router_bias,
                     const void* w_gate, const void* w_up, const void* w_down,
                     const void* ws_gate, const void* ws_up, const void* ws_down, void* stream);

/* Bytes of workspace that any hot call needs for up to max_tokens tokens in up to max_seqs
 * sequences with this context (for the Kmax current at the time of the call). [host] */
size_t fmoe_workspace_bytes(const fmoe_ctx* ctx, int32_t max_tokens, int32_t max_seqs);

/* Eq.1-3 and Eq.5: router logits, softmax, modality-dependent top-k, gates.
 * x [T,H] dtype; is_visual [T] (non-zero = visual token).
 * probs [T,E] fp32 or NULL: softmax probabilities of every token.
 * topk_idx [T,Kmax] int32: the k experts with the highest probability, ordered by
 * (probability descending, expert index ascending) -- ties go to the lower index -- padded
 * with -1 (k = k_visual for visual tokens, k_text otherwise).
 * topk_gate [T,Kmax] fp32: P_j / sum of the listed P (or P_j if renormalize == 0), pad 0. */
int fmoe_route(fmoe_ctx* ctx, const void* x, const uint8_t* is_visual, int32_t T, float* probs,
               int32_t* topk_idx, float* topk_gate, void* stream);

/* Sec. 3.2: window redundancy scores, budget, drop, compaction -- per sequence.
 * probs [T,E] fp32 from fmoe_route; cu_seqlens [B+1] int32 (cu[0] = 0, cu[B] = T; T > 0 with
 * B == 0 is FMOE_ERR_INVALID_ARG; should cu[B] be below T on the device, the tokens past it are in
 * no sequence: they are never pruned and lie beyond new_cu_seqlens[B]).
 * attn_importance [T] fp32 or NULL: per-token attention importance (Eq.7); when given, windows
 * are dropped in the order (normalised window attention ascending, score descending, index
 * ascending), otherwise (score descending, index ascending).
 * Visual tokens of a sequence, in position order, are cut into windows of W (the last may be
 * shorter; a one-token window scores exactly 1).  eta = floor(r*N_v + 1/2) visual tokens
 * survive (at least 1 if N_v > 0): whole windows are dropped in order while they fit and the
 * next window loses its last tokens.  Text tokens always survive.
 * kept_idx [T capacity] int32: ascending global indices of surviving tokens (first T' valid).
 * new_cu_seqlens [B+1] int32: per-sequence boundaries after pruning; new_cu_seqlens[B] = T'.
 * scores [T capacity] fp32 or NULL: the score C of window i of sequence b at
 * scores[cu_seqlens[b] + i].
 * Window merging (Sec. 3.2.3, Eq.14-18), params->gamma > 0: before the drop walk at most
 * floor(eta*gamma) windows are merged, taken in the order (score descending, index ascending); a
 * window of w >= 2 tokens is merged while the w-1 tokens this removes fit in the budget; the drop walk
 * then runs over the remaining windows with the budget that is left, so exactly eta visual tokens
 * survive as before.  A merged window is represented by ONE token at the position of its first
 * token: the mean of its rows rescaled to the largest row norm of the window.
 * x_in [T,H] dtype: the tensor whose rows are merged (the layer input); x_merged [T capacity, H] dtype:
 * row p = x_in[kept_idx[p]], or the merged token if position p is one; is_merged [T capacity] u8 or
 * NULL: 1 for merged positions.  All three must be NULL when gamma == 0; x_in and x_merged are
 * required when gamma > 0.  The caller routes the merged rows again (fmoe_layer_forward does). */
int fmoe_prune(fmoe_ctx* ctx, const fmoe_prune_params* params, const float* probs,
               const uint8_t* is_visual, const int32_t* cu_seqlens, int32_t B, int32_t T,
               const float* attn_importance, const void* x_in, int32_t* kept_idx,
               int32_t* new_cu_seqlens, float* scores, void* x_merged, uint8_t* is_merged, void* ws,
               size_t ws_bytes, void* stream);

/* Dispatch order (the paper leaves it to the framework): the rows are all (kept position p,
 * slot s) pairs with topk_idx >= 0, sorted by (expert ascending, p ascending).
 * kept_idx [n_kept] or NULL (= all tokens, p == t).  n_kept_dev: optional device int32 that
 * overrides n_kept (which then is only the capacity) -- pass new_cu_seqlens + B.
 * expert_offsets [E+1] int32: exclusive scan of rows per expert; expert_offsets[E] = M.
 * perm_src [n_kept*Kmax capacity] int32: row -> kept position p.
 * inv_perm [n_kept,Kmax] int32: (p,s) -> row, or -1. */
int fmoe_permute(fmoe_ctx* ctx, const int32_t* topk_idx, const int32_t* kept_idx, int32_t n_kept,
                 const int32_t* n_kept_dev, int32_t* expert_offsets, int32_t* perm_src,
                 int32_t* inv_perm, void* ws, size_t ws_bytes, void* stream);

/* fmoe_permute for callers that cannot allocate device memory or bring a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels
 * and bit-identical results; the scratch of the kernels (4.25 MiB) is a static device array that each
 * GPU running the library holds until the process ends.  The call allocates nothing and is kernel
 * launches only.  Limits: n_kept <= 65536 and n_kept * Kmax <= 2^20, else FMOE_ERR_UNSUPPORTED (use
 * fmoe_permute).  All calls on one GPU share the array: calls that overlap on one GPU (different
 * streams or threads) race and must be serialised by the caller; nothing has to be cleared between
 * calls (every scratch entry a call reads it has written itself).  The context's GPU must be the
 * current device, as for every other hot call. */
int fmoe_permute_noalloc(fmoe_ctx* ctx, const int32_t* topk_idx, const int32_t* kept_idx, int32_t n_kept,
                         const int32_t* n_kept_dev, int32_t* expert_offsets, int32_t* perm_src,
                         int32_t* inv_perm, void* stream);

/* The expert FFNs of Eq.4 as a grouped GEMM: for every row r of expert e,
 * y[r] = FFN_e(x[token(perm_src[r])]); the activation silu(.)*(.) is rounded to dtype between
 * the two products.  y [n_kept*Kmax capacity, H] dtype.  y_shared [N_s, n_kept, H] dtype or NULL
 * iff N_s == 0: the output of shared expert i for kept position p at (i*n_kept + p)*H.
 * bf16: rows of x are addressed with 32-bit byte offsets, so every token index in kept_idx must
 * lie within the first 4 GiB of x (2^32 / (2*H) tokens); hidden buffers beyond 4 GiB are
 * refused with FMOE_ERR_UNSUPPORTED. */
int fmoe_expert_ffn(fmoe_ctx* ctx, const void* x, const int32_t* kept_idx, int32_t n_kept,
                    const int32_t* n_kept_dev, const int32_t* expert_offsets,
                    const int32_t* perm_src, void* y, void* y_shared, void* ws, size_t ws_bytes,
                    void* stream);

/* Eq.4: out[p] = (residual[t]) + sum_i y_shared[i][p] + sum_s topk_gate[t,s] * y[inv_perm[p,s]]
 * with t = kept_idx[p]; fp32 accumulation in that order, one rounding to dtype.  y, y_shared,
 * n_kept as given to fmoe_expert_ffn.
 * residual [T,H] dtype or NULL; out [n_kept,H] dtype. */
int fmoe_combine(fmoe_ctx* ctx, const void* y, const void* y_shared, const int32_t* inv_perm,
                 const float* topk_gate, const int32_t* kept_idx, int32_t n_kept,
                 const int32_t* n_kept_dev, const void* residual, void* out, void* stream);

/* The whole layer: route -> prune (if params != NULL and prune_mode != 0 and retention < 1)
 * -> permute -> expert_ffn -> combine, enqueued back to back.  Equivalent to the five calls.
 * out [T capacity,H] dtype (first T' rows valid); kept_idx [T]; new_cu_seqlens [B+1];
 * is_visual_out [T capacity] or NULL: the modality mask of the kept tokens.
 * add_residual != 0 adds x[t] to the layer output (x <- x + MoE(x)).
 * Because an MoE layer acts on every token independently, dropping a token before the experts
 * gives the kept tokens the same outputs as dropping it after the layer; both prune modes
 * therefore run the experts on the kept tokens only.
 * Window merging (params->gamma > 0) is where the two modes differ.  prune_mode 1: the rows of x are
 * merged (fmoe_prune's x_merged), every kept token is routed again on the merged input, the experts
 * run on it and add_residual adds the merged rows.  prune_mode 2: the layer runs on all T tokens, the
 * windows are scored on this layer's probabilities and the OUTPUT rows are compacted, a merged window
 * replaced by the merged row of its tokens' outputs (Eq.16-18 on the layer output, residual included
 * when add_residual != 0).
 * bf16: x (T*H*2 bytes) and the hidden buffers (T*Kmax*S_m*2, T*N_s*S_s*2 bytes) must each stay
 * below 4 GiB, else FMOE_ERR_UNSUPPORTED (32-bit row offsets in the expert GEMMs).  T > 0 with
 * B == 0 is FMOE_ERR_INVALID_ARG. */
int fmoe_layer_forward(fmoe_ctx* ctx, const fmoe_prune_params* params, const void* x,
                       const uint8_t* is_visual, const int32_t* cu_seqlens, int32_t B, int32_t T,
                       const float* attn_importance, int add_residual, void* out,
                       int32_t* kept_idx, int32_t* new_cu_seqlens, uint8_t* is_visual_out,
                       void* ws, size_t ws_bytes, void* stream);

/* ---- the layer stack: per-layer expert activation (Sec. 3.1) and pruning stages (Sec. 3.2, App. D) ----
 *
 * fmoe_kept_counts [host arithmetic only] -- the token budget of Sec. 3.2.3 per sequence: a pruning
 * stage with retention r keeps eta_b = floor(r*N_v,b + 1/2) visual tokens of sequence b, clamped to
 * [min(1,N_v,b), N_v,b] (r is taken at fp32 precision and the product in fp64, exactly as the kernels
 * do), and every text token.  visual_lens [B] host in, kept_visual_lens [B] host out (may alias).
 * Because the rule keeps an exact count, a caller can size every later call without reading the device.
 * FMOE_ERR_INVALID_ARG for r outside (0,1], B < 0 or a negative length.
 *
 * fmoe_stage_retention [host arithmetic only] -- App. D: a cumulative retain ratio r reached in
 * `stages` pruning stages of equal per-stage ratio beta = r^(1/stages); *beta is the fp32 value the
 * stages are run with.  FMOE_ERR_INVALID_ARG for r outside (0,1] or stages < 1. */
int fmoe_kept_counts(const int32_t* visual_lens, int32_t B, float retention, int32_t* kept_visual_lens);
int fmoe_stage_retention(float retention, int32_t stages, float* beta);

/* What one layer of a stack does: its experts per token (Sec. 3.1: K for every token below layer
 * l_v, K_v for visual tokens from l_v on) and its pruning stage, if any (prune.prune_mode == 0 or
 * prune.retention == 1: none). */
typedef struct {
  int32_t k_text, k_visual;
  fmoe_prune_params prune;
} fmoe_layer_plan;

/* Fill plan[n_layers] [host]: k = (K, K) in layers below l_v and (K, K_v) from l_v on (l_v = n_layers:
 * never reduced); a pruning stage in each of the n_stages layers prune_layers[] (ascending, 0-based; the
 * stage acts inside that layer, after its routing, so the layers after it see the shorter sequence),
 * each with the fields of *stage except retention, which becomes the per-stage ratio
 * fmoe_stage_retention(stage->retention, n_stages).  stage may be NULL iff n_stages == 0. */
int fmoe_stack_plan(int32_t n_layers, int32_t K, int32_t K_v, int32_t l_v, const int32_t* prune_layers,
                    int32_t n_stages, const fmoe_prune_params* stage, fmoe_layer_plan* plan);

/* Workspace bytes of fmoe_stack_forward for a batch of up to max_tokens tokens in max_seqs sequences
 * (two activation buffers, masks, index lists, plus the largest per-layer workspace of the plan). [host] */
size_t fmoe_stack_workspace_bytes(fmoe_ctx* const* layers, const fmoe_layer_plan* plan, int32_t n_layers,
                                  int32_t max_tokens, int32_t max_seqs);

/* x <- x + MoE_l(x) for l = 0 .. n_layers-1, every layer one fmoe_layer_forward with add_residual on
 * the context layers[l] (all of one d_model, dtype and device; weights set), its top-k switched to
 * plan[l] with fmoe_set_topk and plan[l].prune as its pruning stage.  Kernel launches only: the token
 * count handed to the layers after a stage comes from fmoe_kept_counts on visual_lens / text_lens
 * [B] [host], the per-sequence token counts of the input batch (their sum must be T).
 * attn [n_layers] [host array of device pointers] or NULL: attn[l] = attention importance [T_l] for the
 * stage of layer l (Eq.7), NULL entries = none.
 * out [T capacity, d_model]: the first *n_out rows are the stack's output; kept_idx [T capacity]: for
 * each output row the index of its token in the input batch (identity without pruning);
 * new_cu_seqlens [B+1]; is_visual_out [T capacity] or NULL; n_out [host] or NULL: rows of out, known
 * on the host from the budget rule.  x is not modified.  The contexts' k_text / k_visual are left at
 * the last layer's plan. */
int fmoe_stack_forward(fmoe_ctx* const* layers, const fmoe_layer_plan* plan, int32_t n_layers,
                       const void* x, const uint8_t* is_visual, const int32_t* cu_seqlens,
                       const int32_t* visual_lens, const int32_t* text_lens, int32_t B, int32_t T,
                       const float* const* attn, void* out, int32_t* kept_idx, int32_t* new_cu_seqlens,
                       uint8_t* is_visual_out, int32_t* n_out, void* ws, size_t ws_bytes, void* stream);

/* Instrumentation (not part of the paper's path): per-kernel GPU time of the most recent hot
 * call.  fmoe_profile_enable(ctx,1) creates one HIP event pair per kernel slot and makes every
 * later launch on this context record them on its stream; (ctx,0) stops recording.
 * fmoe_profile_read waits for the recorded events and writes the milliseconds of each slot to
 * ms[fmoe_profile_slots()] [host] (-1 for slots the last call did not launch), then clears the
 * "launched" marks.  fmoe_profile_name gives a slot's kernel name. */
int fmoe_profile_enable(fmoe_ctx* ctx, int enable);
int fmoe_profile_slots(void);
const char* fmoe_profile_name(int slot);
int fmoe_profile_read(fmoe_ctx* ctx, float* ms);

/* ---- Diagnostics: the paper's analysis statistics on the layer's tensors.  They feed no decision
 * of the layer.  All pointers are device pointers unless marked [host]; nothing is allocated and
 * the host is not synchronised; results are reproducible run to run (fixed reduction orders).
 *
 * fmoe_adjacent_similarity -- routing similarity of adjacent tokens (Fig. 1; Eq.8 on a two-token
 * window): pair_sim[t] = cosine of the routing-probability rows probs[t] and probs[t+1] ([T,E] fp32,
 * E = the context's n_experts) when t and t+1 lie in the same sequence of cu_seqlens [B+1] and have
 * the same modality in is_visual [T]; -2 where t starts no such pair (pair_sim [T], out).
 * mean [2] / count [2] (out): average and number of the pairs, index 0 text, 1 vision (mean 0
 * without pairs).
 *
 * fmoe_magnitude_stability -- magnitude stability of expert outputs (App. C.1): row_norm[r] =
 * Euclidean norm of row r of y [M, d_model] (the routed experts' outputs before the gate-weighted
 * sum, as fmoe_expert_ffn writes them; context dtype), for the first M rows or *M_dev of them when
 * M_dev is not NULL (a device count such as expert_offsets + E).  The modality of row r is that of
 * the token is_visual[kept_idx[perm_src[r]]] (kept_idx NULL: is_visual[perm_src[r]]).  stats [2][4]
 * (out) = mean, population standard deviation, CV = sigma/mean and V = 1/(1+CV) of the norms of
 * text rows (index 0) and vision rows (index 1); a modality without rows reports 0, 0, 0, 1.
 * row_norm [M] is an output and the scratch of the call.
 *
 * fmoe_row_cosine -- out[r] = cosine between row r of a and of b ([n, d_model], context dtype; 0
 * where a row is all zero), e.g. the measured angle between the layer outputs with K and with m
 * active experts (App. C).  n_dev as above.
 *
 * fmoe_gate_cosine -- the angle App. C predicts for orthonormal expert outputs: out[t] =
 * sqrt(sum_{i<m} g_i^2 / sum_{i<K} g_i^2) from gates [T,K] fp32, each row a token's K gates in
 * descending order (fmoe_route's topk_gate for tokens routed with K experts; a common scale
 * cancels); 0 for rows with fewer than K positive gates.  FMOE_ERR_INVALID_ARG unless 0 <= m <= K. */
int fmoe_adjacent_similarity(fmoe_ctx* ctx, const float* probs, const uint8_t* is_visual,
                             const int32_t* cu_seqlens, int32_t B, int32_t T, float* pair_sim, float* mean,
                             int32_t* count, void* stream);
int fmoe_magnitude_stability(fmoe_ctx* ctx, const void* y, int32_t M, const int32_t* M_dev,
                             const int32_t* perm_src, const int32_t* kept_idx, const uint8_t* is_visual,
                             float* row_norm, float* stats, void* stream);
int fmoe_row_cosine(fmoe_ctx* ctx, const void* a, const void* b, int32_t n, const int32_t* n_dev, float* out,
                    void* stream);
int fmoe_gate_cosine(fmoe_ctx* ctx, const float* gates, int32_t T, int32_t K, int32_t m, float* out,
                     void* stream);

/* ---- theoretical FLOPs (App. E) [host arithmetic only: no device, no context, no stream] ----------
 * Per-layer cost on x tokens: attention 4*x^2*H + 8*x*H^2, plus the MoE FFN 2*x*H*E + 6*x*H*S_m*k
 * (k = K, or K_v where activation is reduced) or, in a dense layer, the MLP 6*x*H*S.
 * ratios[0] = R_prune (token pruning only), ratios[1] = R_act (reduced activation from layer l_v on,
 * no pruning), ratios[2] = R_comb (both): total FLOPs over all layers divided by the unmodified model's;
 * the saving the paper's tables print is 1 - R.  The tables' l_v counts MoE layers from one: their
 * (l_v, K_v) entries are reproduced with l_v = table value - 1 + n_dense here.
 * FMOE_ERR_NULL_PTR for a NULL argument, FMOE_ERR_INVALID_ARG for values outside the ranges above
 * (non-positive sizes, beta outside (0,1], prune layers not ascending or outside the model). */
int fmoe_flops_ratios(const fmoe_flops_model* model, double* ratios /* [3], host, out */);

#ifdef __cplusplus
}
#endif
#endif /* FMOE_H_ */
