"""Thin ctypes binding over libfmoe.so (declared in include/fmoe.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.  PyTorch
supplies device memory and the current stream.  There is no fallback: if the library has not
been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfmoe.so")

FMOE_F32, FMOE_BF16 = 0, 1
TOPK, RANDOMK, MINK = 0, 1, 2   # fmoe_set_selection strategies
EXPORTS = ["fmoe_version", "fmoe_last_error", "fmoe_create", "fmoe_destroy", "fmoe_set_topk",
           "fmoe_set_selection",
           "fmoe_set_weights", "fmoe_workspace_bytes", "fmoe_route", "fmoe_prune", "fmoe_permute",
           "fmoe_expert_ffn", "fmoe_combine", "fmoe_layer_forward", "fmoe_profile_enable",
           "fmoe_profile_slots", "fmoe_profile_name", "fmoe_profile_read", "fmoe_adjacent_similarity",
           "fmoe_magnitude_stability", "fmoe_row_cosine", "fmoe_gate_cosine", "fmoe_flops_ratios",
           "fmoe_kept_counts", "fmoe_stage_retention", "fmoe_stack_plan", "fmoe_stack_workspace_bytes",
           "fmoe_stack_forward", "fmoe_permute_noalloc", "fmoe_set_ffn_shape"]


class FmoeConfig(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_experts", C.c_int32), ("d_ffn", C.c_int32),
                ("n_shared", C.c_int32), ("d_ffn_shared", C.c_int32), ("k_text", C.c_int32),
                ("k_visual", C.c_int32), ("renormalize", C.c_int32), ("dtype", C.c_int32)]


class FmoeFlopsModel(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_dense", C.c_int32), ("H", C.c_double), ("S", C.c_double),
                ("S_m", C.c_double), ("E", C.c_double), ("K", C.c_double), ("K_v", C.c_double),
                ("l_v", C.c_int32), ("n_prune", C.c_int32), ("prune_layers", C.c_int32 * 8),
                ("beta", C.c_double), ("L_v", C.c_double)]


class FmoePruneParams(C.Structure):
    _fields_ = [("retention", C.c_float), ("window", C.c_int32), ("alpha", C.c_float),
                ("gamma", C.c_float), ("sim_mode", C.c_int32), ("prune_mode", C.c_int32),
                ("merge_mode", C.c_int32)]


class FmoeLayerPlan(C.Structure):
    _fields_ = [("k_text", C.c_int32), ("k_visual", C.c_int32), ("prune", FmoePruneParams)]


class FmoeError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"fmoe error {code}: {msg}")
        self.code = code


_lib = None


def load():
    """Load libfmoe.so and declare the prototypes.  Raises if the library is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not built: run `python -m paper_2511_17885_amd.build` "
                           "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    lib.fmoe_version.restype = C.c_char_p
    lib.fmoe_last_error.restype = C.c_char_p
    lib.fmoe_create.argtypes = [C.POINTER(vp), C.POINTER(FmoeConfig), C.c_int]
    lib.fmoe_destroy.argtypes = [vp]
    lib.fmoe_destroy.restype = None
    lib.fmoe_set_topk.argtypes = [vp, i32, i32]
    lib.fmoe_set_selection.argtypes = [vp, i32, i32, C.c_uint64]
    lib.fmoe_set_ffn_shape.argtypes = [vp, i32]
    lib.fmoe_set_weights.argtypes = [vp] + [vp] * 8 + [vp]
    lib.fmoe_workspace_bytes.argtypes = [vp, i32, i32]
    lib.fmoe_workspace_bytes.restype = sz
    lib.fmoe_route.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp]
    lib.fmoe_prune.argtypes = [vp, C.POINTER(FmoePruneParams), vp, vp, vp, i32, i32, vp, vp, vp, vp,
                               vp, vp, vp, vp, sz, vp]
    lib.fmoe_permute.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.fmoe_permute_noalloc.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp]
    lib.fmoe_expert_ffn.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.fmoe_combine.argtypes = [vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp]
    lib.fmoe_layer_forward.argtypes = [vp, C.POINTER(FmoePruneParams), vp, vp, vp, i32, i32, vp,
                                       C.c_int, vp, vp, vp, vp, vp, sz, vp]
    lib.fmoe_adjacent_similarity.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, vp, vp]
    lib.fmoe_magnitude_stability.argtypes = [vp, vp, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.fmoe_row_cosine.argtypes = [vp, vp, vp, i32, vp, vp, vp]
    lib.fmoe_gate_cosine.argtypes = [vp, vp, i32, i32, i32, vp, vp]
    lib.fmoe_flops_ratios.argtypes = [C.POINTER(FmoeFlopsModel), C.POINTER(C.c_double)]
    i32p = C.POINTER(C.c_int32)
    lib.fmoe_kept_counts.argtypes = [i32p, i32, C.c_float, i32p]
    lib.fmoe_stage_retention.argtypes = [C.c_float, i32, C.POINTER(C.c_float)]
    lib.fmoe_stack_plan.argtypes = [i32, i32, i32, i32, i32p, i32, C.POINTER(FmoePruneParams),
                                    C.POINTER(FmoeLayerPlan)]
    lib.fmoe_stack_workspace_bytes.argtypes = [C.POINTER(vp), C.POINTER(FmoeLayerPlan), i32, i32, i32]
    lib.fmoe_stack_workspace_bytes.restype = sz
    lib.fmoe_stack_forward.argtypes = [C.POINTER(vp), C.POINTER(FmoeLayerPlan), i32, vp, vp, vp, i32p, i32p,
                                       i32, i32, C.POINTER(vp), vp, vp, vp, vp, i32p, vp, sz, vp]
    lib.fmoe_profile_enable.argtypes = [vp, C.c_int]
    lib.fmoe_profile_slots.argtypes = []
    lib.fmoe_profile_name.argtypes = [C.c_int]
    lib.fmoe_profile_name.restype = C.c_char_p
    lib.fmoe_profile_read.argtypes = [vp, C.POINTER(C.c_float)]
    for name in EXPORTS:
        if name not in ("fmoe_version", "fmoe_last_error", "fmoe_destroy", "fmoe_workspace_bytes",
                        "fmoe_profile_name", "fmoe_stack_workspace_bytes"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise FmoeError(rc, load().fmoe_last_error().decode())


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_contiguous()
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def prune_params(retention=1.0, window=1, alpha=1.0, gamma=0.0, sim_mode=0, prune_mode=1, merge_mode=0):
    return FmoePruneParams(float(retention), int(window), float(alpha), float(gamma), int(sim_mode),
                           int(prune_mode), int(merge_mode))


class FMoE:
    """One MoE layer shape on one GPU.  Methods mirror the C entry points one to one."""

    def __init__(self, *, d_model, n_experts, d_ffn, k_text, k_visual, dtype, n_shared=0,
                 d_ffn_shared=0, renormalize=True, device=0):
        self.lib = load()
        self.torch_dtype = {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]
        self.cfg = FmoeConfig(d_model, n_experts, d_ffn, n_shared, d_ffn_shared, k_text, k_visual,
                              int(bool(renormalize)), FMOE_BF16 if dtype == "bf16" else FMOE_F32)
        self.device = torch.device("cuda", device)
        self._ctx = C.c_void_p()
        _check(self.lib.fmoe_create(C.byref(self._ctx), C.byref(self.cfg), device))
        self._weights = None
        self._ws = None

    def close(self):
        if getattr(self, "_ctx", None) and self._ctx.value:
            self.lib.fmoe_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- shape helpers
    @property
    def kmax(self):
        return max(self.cfg.k_text, self.cfg.k_visual)

    @property
    def E(self):
        return self.cfg.n_experts

    @property
    def d(self):
        return self.cfg.d_model

    def set_topk(self, k_text, k_visual):
        _check(self.lib.fmoe_set_topk(self._ctx, k_text, k_visual))
        self.cfg.k_text, self.cfg.k_visual = k_text, k_visual

    def set_selection(self, strategy, k_base, seed=0):
        """Selection-strategy ablation: TOPK / RANDOMK / MINK among the token's top-k_base experts."""
        _check(self.lib.fmoe_set_selection(self._ctx, int(strategy), int(k_base), int(seed)))

    def set_ffn_shape(self, shape):
        """0: expert GEMM shape chosen by size, 1: weight-stream shape, 2: dense shape (fmoe_set_ffn_shape)."""
        _check(self.lib.fmoe_set_ffn_shape(self._ctx, int(shape)))

    def set_weights(self, router_w, router_bias, w_gate, w_up, w_down, ws_gate=None, ws_up=None,
                    ws_down=None, release_packed=False):
        """release_packed: a bf16 context reads its expert weights from the library's packed copies only,
        so once the packing kernels have run the caller's expert tensors need not be kept alive; with
        this flag the binding waits for the stream and holds on to the router bias alone."""
        self._weights = (router_w, router_bias, w_gate, w_up, w_down, ws_gate, ws_up, ws_down)
        _check(self.lib.fmoe_set_weights(self._ctx, *[_ptr(t) for t in self._weights], _stream()))
        if release_packed and self.cfg.dtype == FMOE_BF16:
            torch.cuda.current_stream().synchronize()
            self._weights = (router_bias,)

    def workspace_bytes(self, max_tokens, max_seqs=1):
        return int(self.lib.fmoe_workspace_bytes(self._ctx, max_tokens, max_seqs))

    def workspace(self, max_tokens, max_seqs=1):
        need = self.workspace_bytes(max_tokens, max_seqs)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._ws

    def _i32(self, *shape):
        return torch.empty(shape, dtype=torch.int32, device=self.device)

    def _f32(self, *shape):
        return torch.empty(shape, dtype=torch.float32, device=self.device)

    # ---- instrumentation
    def profile_enable(self, on=True):
        _check(self.lib.fmoe_profile_enable(self._ctx, int(bool(on))))

    def profile_read(self):
        """{kernel name: milliseconds} for the kernels the last hot call launched."""
        n = self.lib.fmoe_profile_slots()
        ms = (C.c_float * n)()
        _check(self.lib.fmoe_profile_read(self._ctx, ms))
        return {self.lib.fmoe_profile_name(i).decode(): float(ms[i]) for i in range(n) if ms[i] >= 0}

    # ---- the entry points
    def route(self, x, is_visual, want_probs=True):
        T = x.shape[0]
        K = max(self.kmax, 1)
        probs = self._f32(T, self.E) if want_probs else None
        idx, gate = self._i32(T, K), self._f32(T, K)
        _check(self.lib.fmoe_route(self._ctx, _ptr(x), _ptr(is_visual), T, _ptr(probs), _ptr(idx),
                                   _ptr(gate), _stream()))
        return probs, idx[:, :self.kmax], gate[:, :self.kmax]

    def prune(self, params, probs, is_visual, cu_seqlens, attn=None, want_scores=False, x=None):
        """Returns (kept_idx, new_cu_seqlens, scores or None); with window merging (params.gamma > 0,
        x = the tensor whose rows are merged) also (is_merged, x_merged)."""
        T, B = probs.shape[0], cu_seqlens.shape[0] - 1
        kept, new_cu = self._i32(max(T, 1)), self._i32(B + 1)
        scores = self._f32(max(T, 1)) if want_scores else None
        merging = params.gamma > 0
        x_merged = torch.empty((max(T, 1), self.d), dtype=self.torch_dtype, device=self.device) if merging else None
        is_merged = torch.zeros(max(T, 1), dtype=torch.uint8, device=self.device) if merging else None
        ws = self.workspace(T, B)
        _check(self.lib.fmoe_prune(self._ctx, C.byref(params), _ptr(probs), _ptr(is_visual),
                                   _ptr(cu_seqlens), B, T, _ptr(attn), _ptr(x) if merging else None,
                                   _ptr(kept), _ptr(new_cu), _ptr(scores), _ptr(x_merged), _ptr(is_merged),
                                   _ptr(ws), ws.numel(), _stream()))
        if merging:
            return kept, new_cu, scores, is_merged, x_merged
        return kept, new_cu, scores

    def permute(self, topk_idx, kept_idx, n_kept, n_kept_dev=None):
        K = max(self.kmax, 1)
        offs, perm, inv = self._i32(self.E + 1), self._i32(max(n_kept * K, 1)), self._i32(max(n_kept, 1), K)
        ws = self.workspace(n_kept, 1)
        _check(self.lib.fmoe_permute(self._ctx, _ptr(topk_idx), _ptr(kept_idx), n_kept, _ptr(n_kept_dev),
                                     _ptr(offs), _ptr(perm), _ptr(inv), _ptr(ws), ws.numel(), _stream()))
        return offs, perm, inv

    def permute_noalloc(self, topk_idx, kept_idx, n_kept, n_kept_dev=None):
        """fmoe_permute_noalloc: the same permutation with the kernels' scratch in the library's static
        device array (no workspace, no allocation inside the call; outputs are the caller's)."""
        K = max(self.kmax, 1)
        offs, perm, inv = self._i32(self.E + 1), self._i32(max(n_kept * K, 1)), self._i32(max(n_kept, 1), K)
        _check(self.lib.fmoe_permute_noalloc(self._ctx, _ptr(topk_idx), _ptr(kept_idx), n_kept, _ptr(n_kept_dev),
                                             _ptr(offs), _ptr(perm), _ptr(inv), _stream()))
        return offs, perm, inv

    def expert_ffn(self, x, kept_idx, n_kept, expert_offsets, perm_src, n_kept_dev=None):
        K = max(self.kmax, 1)
        y = torch.empty((max(n_kept * K, 1), self.d), dtype=self.torch_dtype, device=self.device)
        ysh = None
        if self.cfg.n_shared > 0:
            ysh = torch.empty((self.cfg.n_shared, max(n_kept, 1), self.d), dtype=self.torch_dtype,
                              device=self.device)
        ws = self.workspace(n_kept, 1)
        _check(self.lib.fmoe_expert_ffn(self._ctx, _ptr(x), _ptr(kept_idx), n_kept, _ptr(n_kept_dev),
                                        _ptr(expert_offsets), _ptr(perm_src), _ptr(y), _ptr(ysh),
                                        _ptr(ws), ws.numel(), _stream()))
        return y, ysh

    def combine(self, y, y_shared, inv_perm, topk_gate, kept_idx, n_kept, residual=None,
                n_kept_dev=None):
        out = torch.empty((max(n_kept, 1), self.d), dtype=self.torch_dtype, device=self.device)
        _check(self.lib.fmoe_combine(self._ctx, _ptr(y), _ptr(y_shared), _ptr(inv_perm),
                                     _ptr(topk_gate), _ptr(kept_idx), n_kept, _ptr(n_kept_dev),
                                     _ptr(residual), _ptr(out), _stream()))
        return out

    def layer_forward(self, x, is_visual, cu_seqlens, params=None, attn=None, add_residual=False,
                      out=None, kept_idx=None, new_cu=None, is_visual_out=None, want_mask=False):
        """Enqueues the whole layer; returns (out [T cap, d], kept_idx [T cap], new_cu_seqlens
        [B+1], is_visual_out or None).  new_cu_seqlens[-1] is T' (on the device)."""
        T, B = x.shape[0], cu_seqlens.shape[0] - 1
        if out is None:
            out = torch.empty((max(T, 1), self.d), dtype=self.torch_dtype, device=self.device)
        if kept_idx is None:
            kept_idx = self._i32(max(T, 1))
        if new_cu is None:
            new_cu = self._i32(B + 1)
        if is_visual_out is None and want_mask:
            is_visual_out = torch.empty(max(T, 1), dtype=torch.uint8, device=self.device)
        ws = self.workspace(T, B)
        _check(self.lib.fmoe_layer_forward(self._ctx, C.byref(params) if params is not None else None,
                                           _ptr(x), _ptr(is_visual), _ptr(cu_seqlens), B, T, _ptr(attn),
                                           int(bool(add_residual)), _ptr(out), _ptr(kept_idx),
                                           _ptr(new_cu), _ptr(is_visual_out), _ptr(ws), ws.numel(),
                                           _stream()))
        return out, kept_idx, new_cu, is_visual_out


    # ---- diagnostics
    def adjacent_similarity(self, probs, is_visual, cu_seqlens):
        """Returns (pair_sim [T], mean [2], count [2]); index 0 text pairs, 1 vision pairs."""
        T, B = probs.shape[0], cu_seqlens.shape[0] - 1
        pair, mean, count = self._f32(max(T, 1)), self._f32(2), self._i32(2)
        _check(self.lib.fmoe_adjacent_similarity(self._ctx, _ptr(probs), _ptr(is_visual), _ptr(cu_seqlens), B, T,
                                                 _ptr(pair), _ptr(mean), _ptr(count), _stream()))
        return pair[:T], mean, count

    def magnitude_stability(self, y, M, perm_src, kept_idx, is_visual, M_dev=None):
        """Returns (row_norm [M], stats [2,4] = mean, sigma, CV, V for text / vision rows)."""
        norms, stats = self._f32(max(M, 1)), self._f32(2, 4)
        _check(self.lib.fmoe_magnitude_stability(self._ctx, _ptr(y), M, _ptr(M_dev), _ptr(perm_src),
                                                 _ptr(kept_idx), _ptr(is_visual), _ptr(norms), _ptr(stats),
                                                 _stream()))
        return norms[:M], stats

    def row_cosine(self, a, b, n=None, n_dev=None):
        n = a.shape[0] if n is None else n
        out = self._f32(max(n, 1))
        _check(self.lib.fmoe_row_cosine(self._ctx, _ptr(a), _ptr(b), n, _ptr(n_dev), _ptr(out), _stream()))
        return out[:n]

    def gate_cosine(self, gates, m):
        T, K = gates.shape
        out = self._f32(max(T, 1))
        _check(self.lib.fmoe_gate_cosine(self._ctx, _ptr(gates), T, K, int(m), _ptr(out), _stream()))
        return out[:T]


def flops_ratios(*, n_layers, H, S_m, E, K, L_v, K_v=None, l_v=None, prune_layers=(), beta=1.0, n_dense=0, S=0.0):
    """(R_prune, R_act, R_comb) of App. E from fmoe_flops_ratios: the FLOPs left with token pruning, with
    reduced expert activation from layer l_v on, and with both, as fractions of the unmodified model's."""
    prune_layers = [int(p) for p in prune_layers]
    if len(prune_layers) > 8:
        raise ValueError("at most 8 pruning stages")
    m = FmoeFlopsModel(n_layers=int(n_layers), n_dense=int(n_dense), H=float(H), S=float(S), S_m=float(S_m),
                       E=float(E), K=float(K), K_v=float(K if K_v is None else K_v),
                       l_v=int(n_layers if l_v is None else l_v), n_prune=len(prune_layers),
                       prune_layers=(C.c_int32 * 8)(*prune_layers), beta=float(beta), L_v=float(L_v))
    out = (C.c_double * 3)()
    _check(load().fmoe_flops_ratios(C.byref(m), out))
    return out[0], out[1], out[2]


def kept_visual_lens(visual_lens, retention):
    """Per-sequence visual token counts after one pruning stage (fmoe_kept_counts: the budget rule of
    Sec. 3.2.3 on the host), which lets a caller size the next layer's call without reading the device."""
    n = len(visual_lens)
    src = (C.c_int32 * max(n, 1))(*[int(v) for v in visual_lens])
    dst = (C.c_int32 * max(n, 1))()
    _check(load().fmoe_kept_counts(src, n, float(retention), dst))
    return [int(dst[b]) for b in range(n)]


def kept_count(visual_lens, text_lens, retention):
    """T' of a pruned batch, on the host: every sequence keeps its budget of visual tokens
    (kept_visual_lens) and all its text tokens."""
    return sum(kept_visual_lens(visual_lens, retention)) + sum(text_lens)


def stage_retention(retention, stages):
    """App. D (fmoe_stage_retention): the per-stage ratio beta of `stages` equal stages reaching `retention`."""
    beta = C.c_float()
    _check(load().fmoe_stage_retention(float(retention), int(stages), C.byref(beta)))
    return beta.value


def stage_schedule(retention, prune_layers, window=1, alpha=1.0, gamma=0.0, sim_mode=0, prune_mode=1,
                   merge_mode=0):
    """{layer: prune params} of a multi-stage schedule: every listed layer runs a stage with the
    per-stage ratio of App. D; the other fields are shared by the stages."""
    beta = stage_retention(retention, len(prune_layers)) if len(prune_layers) else 1.0
    return {int(l): prune_params(beta, window, alpha, gamma, sim_mode, prune_mode, merge_mode)
            for l in prune_layers}


class FMoEStack:
    """A stack of MoE layers with x <- x + MoE_l(x), per-layer (k_text, k_visual) (Sec. 3.1: reduced
    activation from layer l_v on) and pruning stages at chosen layers (Sec. 3.2; App. D).  One
    fmoe_stack_forward call: the sequencing, the budget bookkeeping and the index composition all
    happen inside the library."""

    def __init__(self, layers, k_schedule, prune_after_layer=None, params=None, prune_schedule=None):
        self.layers = list(layers)
        sched = dict(prune_schedule or {})
        if prune_after_layer is not None and params is not None:
            sched[int(prune_after_layer)] = params
        assert len(self.layers) == len(k_schedule)
        n = len(self.layers)
        self.plan = (FmoeLayerPlan * n)()
        for l, (kt, kv) in enumerate(k_schedule):
            self.plan[l].k_text, self.plan[l].k_visual = int(kt), int(kv)
            self.plan[l].prune = sched.get(l, prune_params(retention=1.0, window=1, prune_mode=0))
        self._ctxs = (C.c_void_p * n)(*[m._ctx.value for m in self.layers])
        self._ws = None

    def workspace_bytes(self, max_tokens, max_seqs):
        return int(load().fmoe_stack_workspace_bytes(self._ctxs, self.plan, len(self.layers), max_tokens, max_seqs))

    def forward(self, x, is_visual, cu_seqlens, visual_lens, text_lens, attn=None, out=None, kept_idx=None,
                new_cu=None, want_mask=False):
        """visual_lens / text_lens: per-sequence token counts on the host.  attn: {layer: importance
        [T at that layer]} for stages that use the attention term.  Returns (x_out [T', d], kept_idx
        [T'] indices into the input batch, new_cu_seqlens), with want_mask also the modality mask of the
        output rows."""
        m0 = self.layers[0]
        T, B, n = x.shape[0], cu_seqlens.shape[0] - 1, len(self.layers)
        need = self.workspace_bytes(T, B)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=m0.device)
        if out is None:
            out = torch.empty((max(T, 1), m0.d), dtype=m0.torch_dtype, device=m0.device)
        if kept_idx is None:
            kept_idx = torch.empty(max(T, 1), dtype=torch.int32, device=m0.device)
        if new_cu is None:
            new_cu = torch.empty(B + 1, dtype=torch.int32, device=m0.device)
        nv = (C.c_int32 * max(B, 1))(*[int(v) for v in visual_lens])
        nt = (C.c_int32 * max(B, 1))(*[int(v) for v in text_lens])
        attn_ptrs = None
        if attn:
            attn_ptrs = (C.c_void_p * n)(*[attn[l].data_ptr() if attn.get(l) is not None else None
                                           for l in range(n)])
        n_out = C.c_int32()
        vis_out = torch.empty(max(T, 1), dtype=torch.uint8, device=m0.device) if want_mask else None
        _check(load().fmoe_stack_forward(self._ctxs, self.plan, n, _ptr(x), _ptr(is_visual), _ptr(cu_seqlens),
                                         nv, nt, B, T, attn_ptrs, _ptr(out), _ptr(kept_idx), _ptr(new_cu),
                                         _ptr(vis_out), C.byref(n_out), _ptr(self._ws), self._ws.numel(), _stream()))
        for l, m in enumerate(self.layers):   # the contexts' top-k now is the last layer's plan
            m.cfg.k_text, m.cfg.k_visual = self.plan[l].k_text, self.plan[l].k_visual
        if want_mask:
            return out[:n_out.value], kept_idx[:n_out.value], new_cu, vis_out[:n_out.value]
        return out[:n_out.value], kept_idx[:n_out.value], new_cu
