"""ctypes front-end of the CPU oracle (oracle/fmoe_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by bench.py's
cpu_baseline leg.  The product package never imports this module.  Only argument marshalling
lives here; the arithmetic is in the C++ file (the two host formulas of the appendices, the merge-rate
bound of App. D and the FLOPs ratios of App. E, are written out below).
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None

_f32p = C.POINTER(C.c_float)
_f64p = C.POINTER(C.c_double)
_i32p = C.POINTER(C.c_int32)
_u8p = C.POINTER(C.c_uint8)


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _b
            _b.build()
        _lib = C.CDLL(_LIB_PATH)
        _lib.orc_exp_canon.restype = C.c_float
        _lib.orc_exp_canon.argtypes = [C.c_float]
        _lib.orc_sum_canon.restype = C.c_float
        _lib.orc_sum_canon.argtypes = [_f32p, C.c_int]
        _lib.orc_dot_canon.restype = C.c_float
        _lib.orc_dot_canon.argtypes = [_f32p, _f32p, C.c_int]
        _lib.orc_dot_seq.restype = C.c_float
        _lib.orc_dot_seq.argtypes = [_f32p, _f32p, C.c_int]
        _lib.orc_round_store.restype = C.c_float
        _lib.orc_round_store.argtypes = [C.c_double, C.c_int]
    return _lib


def _p(a: Optional[np.ndarray], ty):
    if a is None:
        return None
    return a.ctypes.data_as(ty)


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _u8(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.uint8)


def num_threads() -> int:
    return int(lib().orc_num_threads())


def exp_canon(x: float) -> np.float32:
    return np.float32(lib().orc_exp_canon(C.c_float(float(x))))


def sum_canon(v) -> np.float32:
    v = _f32(v)
    return np.float32(lib().orc_sum_canon(_p(v, _f32p), int(v.size)))


def dot_canon(a, b) -> np.float32:
    a, b = _f32(a), _f32(b)
    assert a.size == b.size
    return np.float32(lib().orc_dot_canon(_p(a, _f32p), _p(b, _f32p), int(a.size)))


def dot_seq(a, b) -> np.float32:
    a, b = _f32(a), _f32(b)
    assert a.size == b.size
    return np.float32(lib().orc_dot_seq(_p(a, _f32p), _p(b, _f32p), int(a.size)))


def round_store(v: float, is_bf16: bool) -> np.float32:
    return np.float32(lib().orc_round_store(C.c_double(float(v)), int(is_bf16)))


def route(x, is_visual, router_w, router_bias, k_text, k_visual, renormalize=True, shadow=False):
    """Eq.1-3, Eq.5.  Returns probs [T,E] f32, topk_idx [T,Kmax] i32, topk_gate [T,Kmax] f32
    (and the fp64 shadow probabilities when shadow=True)."""
    x, router_w, router_bias, is_visual = _f32(x), _f32(router_w), _f32(router_bias), _u8(is_visual)
    T, d = x.shape
    E = router_w.shape[0]
    assert router_w.shape[1] == d and is_visual.shape[0] == T
    Kmax = max(k_text, k_visual)
    probs = np.empty((T, E), np.float32)
    idx = np.empty((T, Kmax), np.int32)
    gate = np.empty((T, Kmax), np.float32)
    p64 = np.empty((T, E), np.float64) if shadow else None
    rc = lib().orc_route(_p(x, _f32p), _p(is_visual, _u8p), T, d, E, _p(router_w, _f32p),
                         _p(router_bias, _f32p), int(k_text), int(k_visual), int(bool(renormalize)),
                         _p(probs, _f32p), _p(idx, _i32p), _p(gate, _f32p), _p(p64, _f64p))
    if rc != 0:
        raise ValueError("orc_route: bad arguments")
    return (probs, idx, gate, p64) if shadow else (probs, idx, gate)


TOPK, RANDOMK, MINK = 0, 1, 2


def splitmix64_nth(seed: int, n: int) -> int:
    lib().orc_splitmix64_nth.restype = C.c_uint64
    lib().orc_splitmix64_nth.argtypes = [C.c_uint64, C.c_uint64]
    return int(lib().orc_splitmix64_nth(seed, n))


def route_select(x, is_visual, router_w, router_bias, k_text, k_visual, strategy, k_base, seed=0,
                 renormalize=True):
    """Routing with the selection-strategy ablation of Sec. 4 (TopK / RandomK / MinK among the token's
    top-k_base experts, for tokens whose k is below k_base).  Returns probs, topk_idx, topk_gate."""
    x, router_w, router_bias, is_visual = _f32(x), _f32(router_w), _f32(router_bias), _u8(is_visual)
    T, d = x.shape
    E = router_w.shape[0]
    Kmax = max(k_text, k_visual)
    probs = np.empty((T, E), np.float32)
    idx = np.empty((T, Kmax), np.int32)
    gate = np.empty((T, Kmax), np.float32)
    fn = lib().orc_route_select
    fn.argtypes = [_f32p, _u8p, C.c_int, C.c_int, C.c_int, _f32p, _f32p, C.c_int, C.c_int, C.c_int, C.c_int,
                   C.c_int, C.c_uint64, _f32p, _i32p, _f32p]
    rc = fn(_p(x, _f32p), _p(is_visual, _u8p), T, d, E, _p(router_w, _f32p), _p(router_bias, _f32p),
            int(k_text), int(k_visual), int(bool(renormalize)), int(strategy), int(k_base), int(seed),
            _p(probs, _f32p), _p(idx, _i32p), _p(gate, _f32p))
    if rc != 0:
        raise ValueError("orc_route_select: bad arguments")
    return probs, idx, gate


def gamma_hat(retain_ratio, window, stages=3):
    """App. D: the merge rate at which merging alone reaches the token budget,
    (1/beta - 1)/(W - 1) with the per-stage retain ratio beta = r^(1/stages)."""
    beta = float(retain_ratio) ** (1.0 / stages)
    return (1.0 / beta - 1.0) / (window - 1)


def flops_layer(x, H, E, S_m, K):
    """App. E, baseline FLOPs with B = 1: C(x), one MoE transformer layer on a subsequence of x
    tokens = attention 4x^2 H + 8xH^2 plus MoE FFN 2xHE + 6xH S_m K."""
    x, H, E, S_m, K = float(x), float(H), float(E), float(S_m), float(K)
    return 4.0 * x * x * H + 8.0 * x * H * H + 2.0 * x * H * E + 6.0 * x * H * S_m * K


def flops_ratios(stage_layers, *, H, E, S_m, K, K_v, l_v, beta, L_v, n_dense=0, S=0.0):
    """App. E's closed forms, stage by stage.  `stage_layers` = the number of MoE layers N_s that run at
    vision length L_v, beta L_v, beta^2 L_v, ... (InternVL3.5: 6, 3, 4, 35; DeepSeek-VL2: 2, 3, 3, 21
    after its one dense layer).  C'(x) is C(x) with K_v in place of K; Delta_s = C'_s - C_s; m_s = the
    MoE layers of stage s whose index is l_v or more.
        R_prune = (D + sum_s N_s C_s) / (D + N C_0)
        R_act   = (D + (N - M) C_0 + M C'_0) / (D + N C_0),  M = sum_s m_s
        R_comb  = (D + sum_s [N_s C_s + m_s Delta_s]) / (D + N C_0)
    with N = sum_s N_s and D = the n_dense leading dense layers at full length, each its attention plus
    the MLP 6 L_v H S (the appendix prints the MLP term alone; the savings it tabulates for DeepSeek-VL2
    need the dense layer's attention in D as well).  Returns (R_prune, R_act, R_comb)."""
    N = sum(stage_layers)
    c0 = flops_layer(L_v, H, E, S_m, K)
    D = n_dense * (4.0 * L_v * L_v * H + 8.0 * L_v * H * H + 6.0 * L_v * H * S)
    den = D + N * c0
    num_prune = num_comb = D
    first = n_dense   # index of the stage's first layer
    M = 0
    for s, n_s in enumerate(stage_layers):
        x = L_v * beta ** s
        c_s, cp_s = flops_layer(x, H, E, S_m, K), flops_layer(x, H, E, S_m, K_v)
        m_s = sum(1 for i in range(first, first + n_s) if i >= l_v)
        num_prune += n_s * c_s
        num_comb += n_s * c_s + m_s * (cp_s - c_s)
        M += m_s
        first += n_s
    num_act = D + (N - M) * c0 + M * flops_layer(L_v, H, E, S_m, K_v)
    return num_prune / den, num_act / den, num_comb / den


def prune(probs, is_visual, cu_seqlens, retention, window, alpha=1.0, gamma=0.0, sim_mode=0,
          attn=None, x=None, is_bf16=False, merge_mean=False):
    """Sec. 3.2 (scores, budget, merge, drop).  Returns kept_idx [T'] i32 ascending, new_cu_seqlens
    [B+1], window scores C (sequences concatenated); with x [T,d] also is_merged [T'] u8 and the
    layer input after merging x_merged [T',d] (needed when gamma > 0)."""
    probs, is_visual, cu, attn = _f32(probs), _u8(is_visual), _i32(cu_seqlens), _f32(attn)
    x = _f32(x)
    T, E = probs.shape
    B = cu.shape[0] - 1
    offs = np.empty(B + 1, np.int32)
    nwin = lib().orc_window_counts(_p(is_visual, _u8p), _p(cu, _i32p), B, int(window), _p(offs, _i32p))
    kept = np.empty(max(T, 1), np.int32)
    new_cu = np.empty(B + 1, np.int32)
    scores = np.empty(max(nwin, 1), np.float32)
    d = 0 if x is None else x.shape[1]
    is_merged = None if x is None else np.zeros(max(T, 1), np.uint8)
    x_merged = None if x is None else np.empty((max(T, 1), d), np.float32)
    n = lib().orc_prune(_p(probs, _f32p), _p(is_visual, _u8p), _p(cu, _i32p), B, T, E,
                        C.c_float(retention), int(window), C.c_float(alpha), C.c_float(gamma),
                        int(sim_mode), _p(attn, _f32p), _p(kept, _i32p), _p(new_cu, _i32p),
                        _p(scores, _f32p), _p(x, _f32p), int(d), int(bool(is_bf16)),
                        _p(is_merged, _u8p), _p(x_merged, _f32p), int(bool(merge_mean)))
    if n < 0:
        raise ValueError("orc_prune: bad arguments")
    if x is None:
        return kept[:n].copy(), new_cu, scores[:nwin].copy()
    return kept[:n].copy(), new_cu, scores[:nwin].copy(), is_merged[:n].copy(), x_merged[:n].copy()


def permute(topk_idx, kept_idx, E):
    """Dispatch order: rows sorted by (expert, kept position).  Returns expert_offsets [E+1],
    perm_src [M], inv_perm [n_kept, Kmax]."""
    topk_idx = _i32(topk_idx)
    T, Kmax = topk_idx.shape
    kept_idx = _i32(kept_idx)
    n_kept = T if kept_idx is None else int(kept_idx.shape[0])
    offs = np.empty(E + 1, np.int32)
    perm = np.empty(max(n_kept * Kmax, 1), np.int32)
    inv = np.empty((n_kept, Kmax), np.int32)
    M = lib().orc_permute(_p(topk_idx, _i32p), Kmax, _p(kept_idx, _i32p), n_kept, E,
                          _p(offs, _i32p), _p(perm, _i32p), _p(inv, _i32p))
    return offs, perm[:M].copy(), inv


def expert_ffn(x, kept_idx, expert_offsets, perm_src, w_gate, w_up, w_down, is_bf16, rows_sel=None):
    """Routed SwiGLU experts on the permuted rows; y [M,d] fp64 (rows not in rows_sel stay 0)."""
    x, w_gate, w_up, w_down = _f32(x), _f32(w_gate), _f32(w_up), _f32(w_down)
    kept_idx, offs, perm, rows_sel = _i32(kept_idx), _i32(expert_offsets), _i32(perm_src), _i32(rows_sel)
    E, F, d = w_gate.shape
    assert w_down.shape == (E, d, F) and x.shape[1] == d
    M = int(offs[E])
    y = np.zeros((M, d), np.float64)
    lib().orc_expert_ffn(_p(x, _f32p), _p(kept_idx, _i32p), _p(offs, _i32p), _p(perm, _i32p), E, d, F,
                         int(is_bf16), _p(w_gate, _f32p), _p(w_up, _f32p), _p(w_down, _f32p),
                         _p(rows_sel, _i32p), 0 if rows_sel is None else int(rows_sel.size),
                         _p(y, _f64p))
    return y


def shared_ffn(x, kept_idx, n_kept, ws_gate, ws_up, ws_down, is_bf16, pos_sel=None):
    """Sum of the always-on shared experts per kept token; [n_kept,d] fp64."""
    x, ws_gate, ws_up, ws_down = _f32(x), _f32(ws_gate), _f32(ws_up), _f32(ws_down)
    kept_idx, pos_sel = _i32(kept_idx), _i32(pos_sel)
    Ns, Fs, d = ws_gate.shape
    y = np.zeros((n_kept, d), np.float64)
    lib().orc_shared_ffn(_p(x, _f32p), _p(kept_idx, _i32p), int(n_kept), d, Ns, Fs, int(is_bf16),
                         _p(ws_gate, _f32p), _p(ws_up, _f32p), _p(ws_down, _f32p),
                         _p(pos_sel, _i32p), 0 if pos_sel is None else int(pos_sel.size), _p(y, _f64p))
    return y


def combine(y, y_shared, inv_perm, topk_gate, kept_idx, d, residual, is_bf16, pos_sel=None):
    """Eq.4 on the permuted rows.  Returns (out f32 container [n_kept,d], out fp64 unrounded)."""
    y = np.ascontiguousarray(y, np.float64)
    y_shared = None if y_shared is None else np.ascontiguousarray(y_shared, np.float64)
    inv_perm, topk_gate, kept_idx = _i32(inv_perm), _f32(topk_gate), _i32(kept_idx)
    residual, pos_sel = _f32(residual), _i32(pos_sel)
    n_kept, Kmax = inv_perm.shape
    out = np.zeros((n_kept, d), np.float32)
    out64 = np.zeros((n_kept, d), np.float64)
    lib().orc_combine(_p(y, _f64p), _p(y_shared, _f64p), _p(inv_perm, _i32p), _p(topk_gate, _f32p),
                      _p(kept_idx, _i32p), n_kept, Kmax, int(d), _p(residual, _f32p), int(is_bf16),
                      _p(pos_sel, _i32p), 0 if pos_sel is None else int(pos_sel.size),
                      _p(out, _f32p), _p(out64, _f64p))
    return out, out64


def token_outputs(x, tokens, topk_idx, topk_gate, w, is_bf16, add_residual=False):
    """Eq.4 directly for the listed token indices (no permutation).  `w` has the fields of
    workloads.LayerWeights.  Returns (out f32 container, out fp64)."""
    x, tokens, topk_idx, topk_gate = _f32(x), _i32(tokens), _i32(topk_idx), _f32(topk_gate)
    w_gate, w_up, w_down = _f32(w.w_gate), _f32(w.w_up), _f32(w.w_down)
    ws_gate, ws_up, ws_down = _f32(w.ws_gate), _f32(w.ws_up), _f32(w.ws_down)
    E, F, d = w_gate.shape
    Ns, Fs = (0, 0) if ws_gate is None else ws_gate.shape[:2]
    Kmax = topk_idx.shape[1]
    n = int(tokens.size)
    out = np.zeros((n, d), np.float32)
    out64 = np.zeros((n, d), np.float64)
    lib().orc_token_outputs(_p(x, _f32p), _p(tokens, _i32p), n, d, E, F, Ns, Fs, int(is_bf16), Kmax,
                            _p(topk_idx, _i32p), _p(topk_gate, _f32p), _p(w_gate, _f32p),
                            _p(w_up, _f32p), _p(w_down, _f32p), _p(ws_gate, _f32p), _p(ws_up, _f32p),
                            _p(ws_down, _f32p), int(bool(add_residual)), _p(out, _f32p), _p(out64, _f64p))
    return out, out64


def layer_forward(x, is_visual, cu_seqlens, w, *, k_text, k_visual, is_bf16, retention=1.0,
                  window=1, alpha=1.0, gamma=0.0, sim_mode=0, attn=None, add_residual=False,
                  renormalize=True, do_prune=True, ffn=True, merge_mean=False, strategy=TOPK, k_base=0,
                  seed=0, after_layer=False):
    """The whole path: route -> prune -> permute -> experts -> combine (the steps chained, nothing
    else).  Returns a dict with every intermediate.  strategy / k_base / seed: the selection-strategy
    ablation (route_select); merge_mean: plain mean instead of MLERP for merged tokens.
    after_layer: pruning acts on the layer's output instead of its input.  Without merging that is the
    same thing (a token's output does not depend on the other tokens); with gamma > 0 the layer runs on
    every token and Sec. 3.2.3 (Eq.14-18) is applied to the output rows: "out" then holds the compacted
    rows with merged windows replaced by their merged output row, "out_full" / "out_full_f64" the
    layer's output before compaction."""
    T = x.shape[0]
    E = w.router_w.shape[0]
    d = x.shape[1]

    def _route(xx, vv):
        if strategy == TOPK:
            return route(xx, vv, w.router_w, w.router_bias, k_text, k_visual, renormalize)
        return route_select(xx, vv, w.router_w, w.router_bias, k_text, k_visual, strategy, k_base, seed,
                            renormalize)

    probs, idx, gate = _route(x, is_visual)
    if do_prune and retention < 1.0 and gamma > 0.0 and after_layer:
        every = np.arange(T, dtype=np.int32)
        offs, perm, inv = permute(idx, every, E)
        y = expert_ffn(x, every, offs, perm, w.w_gate, w.w_up, w.w_down, is_bf16)
        ysh = None
        if w.ws_gate is not None:
            ysh = shared_ffn(x, every, T, w.ws_gate, w.ws_up, w.ws_down, is_bf16)
        full, full64 = combine(y, ysh, inv, gate, every, d, x if add_residual else None, is_bf16)
        kept, new_cu, scores, is_merged, out_m = prune(probs, is_visual, cu_seqlens, retention, window,
                                                       alpha, gamma, sim_mode, attn, x=full, is_bf16=is_bf16,
                                                       merge_mean=merge_mean)
        return dict(probs=probs, topk_idx=idx, topk_gate=gate, kept_idx=kept, new_cu_seqlens=new_cu,
                    scores=scores, is_merged=is_merged, out=out_m, out_full=full, out_full_f64=full64)
    if do_prune and retention < 1.0 and gamma > 0.0:
        # window merging changes the layer input: the kept rows are gathered (merged windows replaced by
        # their merged token), every kept token is routed again on that tensor (only the merged ones can
        # come out differently) and the rest of the layer runs on it
        kept, new_cu, scores, is_merged, x_m = prune(probs, is_visual, cu_seqlens, retention, window,
                                                     alpha, gamma, sim_mode, attn, x=x, is_bf16=is_bf16,
                                                     merge_mean=merge_mean)
        vis_m = _u8(is_visual)[kept]
        probs_m, idx_m, gate_m = _route(x_m, vis_m)
        ident = np.arange(kept.shape[0], dtype=np.int32)
        offs, perm, inv = permute(idx_m, ident, E)
        res = dict(probs=probs, topk_idx=idx_m, topk_gate=gate_m, kept_idx=kept, new_cu_seqlens=new_cu,
                   scores=scores, expert_offsets=offs, perm_src=perm, inv_perm=inv, is_merged=is_merged,
                   x_merged=x_m)
        if ffn:
            y = expert_ffn(x_m, ident, offs, perm, w.w_gate, w.w_up, w.w_down, is_bf16)
            ysh = None
            if w.ws_gate is not None:
                ysh = shared_ffn(x_m, ident, ident.shape[0], w.ws_gate, w.ws_up, w.ws_down, is_bf16)
            out, out64 = combine(y, ysh, inv, gate_m, ident, d, x_m if add_residual else None, is_bf16)
            res.update(y=y, y_shared=ysh, out=out, out_f64=out64)
        return res
    if do_prune and retention < 1.0:
        kept, new_cu, scores = prune(probs, is_visual, cu_seqlens, retention, window,
                                     alpha, gamma, sim_mode, attn)
    else:
        kept, new_cu, scores = np.arange(T, dtype=np.int32), _i32(cu_seqlens).copy(), None
    offs, perm, inv = permute(idx, kept, E)
    res = dict(probs=probs, topk_idx=idx, topk_gate=gate, kept_idx=kept, new_cu_seqlens=new_cu,
               scores=scores, expert_offsets=offs, perm_src=perm, inv_perm=inv)
    if ffn:
        y = expert_ffn(x, kept, offs, perm, w.w_gate, w.w_up, w.w_down, is_bf16)
        ysh = None
        if w.ws_gate is not None:
            ysh = shared_ffn(x, kept, kept.shape[0], w.ws_gate, w.ws_up, w.ws_down, is_bf16)
        out, out64 = combine(y, ysh, inv, gate, kept, d, x if add_residual else None, is_bf16)
        res.update(y=y, y_shared=ysh, out=out, out_f64=out64)
    return res


def adjacent_similarity(probs, is_visual, cu_seqlens):
    """Fig. 1 statistic.  Returns pair_sim [T] f32 (-2 where no pair starts), mean [2] f64 (text,
    vision), count [2] i32."""
    probs, is_visual, cu = _f32(probs), _u8(is_visual), _i32(cu_seqlens)
    T, E = probs.shape
    pair = np.empty(max(T, 1), np.float32)
    mean = np.zeros(2, np.float64)
    count = np.zeros(2, np.int32)
    lib().orc_adjacent_similarity(_p(probs, _f32p), _p(is_visual, _u8p), _p(cu, _i32p), cu.shape[0] - 1, T, E,
                                  _p(pair, _f32p), _p(mean, _f64p), _p(count, _i32p))
    return pair[:T], mean, count


def magnitude_stability(y, row_is_visual):
    """App. C.1.  Returns row_norm [M] f32 and stats [2,4] f64 = (mu, sigma, CV, V) for text, vision."""
    y, vis = _f32(y), _u8(row_is_visual)
    M, d = y.shape
    norms = np.empty(max(M, 1), np.float32)
    stats = np.zeros((2, 4), np.float64)
    lib().orc_magnitude_stability(_p(y, _f32p), M, d, _p(vis, _u8p), _p(norms, _f32p), _p(stats, _f64p))
    return norms[:M], stats


def row_cosine(a, b):
    a, b = _f32(a), _f32(b)
    assert a.shape == b.shape
    out = np.empty(max(a.shape[0], 1), np.float32)
    lib().orc_row_cosine(_p(a, _f32p), _p(b, _f32p), a.shape[0], a.shape[1], _p(out, _f32p))
    return out[:a.shape[0]]


def gate_cosine(gates, m):
    """App. C closed form from each token's K gates in descending order."""
    gates = _f32(gates)
    T, K = gates.shape
    out = np.empty(max(T, 1), np.float32)
    if lib().orc_gate_cosine(_p(gates, _f32p), T, K, int(m), _p(out, _f32p)) != 0:
        raise ValueError("orc_gate_cosine: bad arguments")
    return out[:T]
