"""GPU parity: every entry point of libfmoe.so, called through the C ABI, against the CPU oracle
on the same seeded inputs.  Expert ids, probabilities, window scores, kept set and permutation
must match bit for bit; FFN / combine outputs within the max-norm relative tolerance of the
storage dtype (1e-5 fp32, 2e-2 bf16)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_17885_amd import binding
from paper_2511_17885_amd import workloads as W
from harness import (HALF_ULP, TOL, assert_outputs_close, assert_residual_outputs_close, dev, host, inputs,
                     make_layer, max_rel_err, torch_dtype)

pytestmark = pytest.mark.gpu


def _case(seed, **kw):
    base = dict(T_v=[40], T_t=[9], d=64, E=8, F=32, k_text=2, k_visual=1, retention=0.5, window=3,
                dtype=W.F32, n_shared=0, F_shared=None, bias_std=0.0, n_components=0, interleave=False)
    base.update(kw)
    return pytest.param(seed, base, id=f"s{seed}-" + "-".join(f"{k}{v}" for k, v in kw.items()
                                                             if k not in ("T_v", "T_t")))


SMALL = [
    _case(100),
    _case(101, T_v=[37, 5, 0, 14], T_t=[4, 0, 6, 3], E=12, k_text=4, k_visual=2, interleave=True),
    _case(102, T_v=[129], T_t=[31], d=200, E=65, F=72, k_text=6, k_visual=3, bias_std=1.0, window=5),
    _case(103, T_v=[61, 70], T_t=[3, 2], d=128, E=128, F=64, k_text=8, k_visual=4, dtype=W.BF16,
          bias_std=1.5, n_components=6, window=5),
    _case(104, T_v=[90], T_t=[10], d=96, E=256, F=40, k_text=16, k_visual=7, dtype=W.BF16, window=4),
    _case(105, T_v=[50], T_t=[14], d=64, E=6, F=48, k_text=3, k_visual=0, n_shared=2, F_shared=24,
          dtype=W.BF16, retention=0.25),
    _case(106, T_v=[0, 0], T_t=[9, 4], E=5, k_text=5, k_visual=2),                      # all text
    _case(107, T_v=[33, 2], T_t=[0, 0], E=7, k_text=1, k_visual=1, retention=0.75, window=4),  # all visual, N_v < W
    _case(108, T_v=[300, 77, 1], T_t=[20, 1, 1], d=256, E=64, F=96, k_text=6, k_visual=3, dtype=W.BF16,
          n_shared=2, F_shared=64, bias_std=1.0, n_components=12, retention=0.5, window=3),
    _case(109, T_v=[45], T_t=[5], E=9, k_text=3, k_visual=3, retention=0.9, window=1),
]


def _wl(seed, kw):
    return W.small_random(seed, **kw)


def _x_rows(wl, o):
    """The rows a residual run adds to the expert term: the kept input rows, or the merged layer input."""
    return o["x_merged"] if "x_merged" in o else wl.x[o["kept_idx"]]


def _oracle(wl, **over):
    kw = dict(k_text=wl.k_text, k_visual=wl.k_visual, is_bf16=wl.dtype == W.BF16,
              retention=wl.retention, window=wl.window)
    kw.update(over)
    return oracle.layer_forward(wl.x, wl.is_visual, wl.cu_seqlens, wl.weights, **kw)


# ---------------------------------------------------------------- route
@pytest.mark.parametrize("seed,kw", SMALL)
def test_route(seed, kw):
    wl = _wl(seed, kw)
    if wl.T == 0:
        pytest.skip("empty")
    m = make_layer(wl)
    x, vis, cu = inputs(wl)
    probs, idx, gate = m.route(x, vis)
    torch.cuda.synchronize()
    o_probs, o_idx, o_gate = oracle.route(wl.x, wl.is_visual, wl.weights.router_w,
                                          wl.weights.router_bias, wl.k_text, wl.k_visual)
    assert np.array_equal(host(idx), o_idx)
    assert np.array_equal(host(probs), o_probs)            # same fixed-order fp32 arithmetic
    assert np.abs(host(gate) - o_gate).max() <= 1e-6


@pytest.mark.parametrize("dtype,d,E,T_v,T_t", [
    (W.F32, 512, 24, [4100], [37]),        # fp32, four chunks of 128: the shallow operand pipeline from 4096 tokens on
    (W.BF16, 1280, 64, [3000, 1200], [50, 13]),   # bf16, ten chunks (five in flight below 4096 tokens)
    (W.BF16, 640, 40, [4095], [0]),        # five chunks: an odd count, one token below the switch
    (W.BF16, 640, 40, [4096], [3]),        # ... and above it (the chunk count is rounded up to an even one)
    (W.F32, 384, 16, [16500], [20]),       # three chunks, two token tiles per block
])
def test_route_large_batches(dtype, d, E, T_v, T_t):
    """The router's launch shapes for large batches (operand pipeline two chunks deep from 4096 tokens on,
    two token tiles per block from 16384): probabilities and expert lists bit for bit, gates to 1e-6."""
    wl = W.small_random(620 + d, T_v=T_v, T_t=T_t, d=d, E=E, F=16, k_text=4, k_visual=2, retention=0.5, window=3,
                        dtype=dtype, bias_std=1.0, n_components=12)
    m = make_layer(wl)
    x, vis, cu = inputs(wl)
    probs, idx, gate = m.route(x, vis)
    torch.cuda.synchronize()
    o_probs, o_idx, o_gate = oracle.route(wl.x, wl.is_visual, wl.weights.router_w, wl.weights.router_bias, 4, 2)
    assert np.array_equal(host(idx), o_idx)
    assert np.array_equal(host(probs), o_probs)
    assert np.abs(host(gate) - o_gate).max() <= 1e-6


def test_route_ties_duplicated_router_rows():
    wl = W.small_random(110, T_v=[20], T_t=[12], d=64, E=10, F=32, k_text=10, k_visual=4,
                        retention=0.5, window=3)
    wl.weights.router_w[7] = wl.weights.router_w[2]
    wl.weights.router_w[9] = wl.weights.router_w[0]
    m = make_layer(wl)
    x, vis, cu = inputs(wl)
    _, idx, gate = m.route(x, vis)
    o_probs, o_idx, o_gate = oracle.route(wl.x, wl.is_visual, wl.weights.router_w, None, 10, 4)
    assert np.array_equal(host(idx), o_idx)
    # all-equal logits: the lowest indices win, in order
    wl.weights.router_w[:] = 0
    m = make_layer(wl)
    _, idx, gate = m.route(x, vis)
    idx = host(idx)
    for t in range(wl.T):
        k = 4 if wl.is_visual[t] else 10
        assert list(idx[t, :k]) == list(range(k)) and np.all(idx[t, k:] == -1)


def test_route_renormalize_off_and_set_topk():
    wl = W.small_random(111, T_v=[30], T_t=[10], d=64, E=16, F=32, k_text=4, k_visual=2,
                        retention=0.5, window=3, bias_std=1.0)
    m = make_layer(wl, renormalize=False)
    x, vis, cu = inputs(wl)
    _, idx, gate = m.route(x, vis)
    o = oracle.route(wl.x, wl.is_visual, wl.weights.router_w, wl.weights.router_bias, 4, 2, renormalize=False)
    assert np.array_equal(host(idx), o[1]) and np.array_equal(host(gate), o[2])
    m2 = make_layer(wl)
    m2.set_topk(6, 6)                                       # the per-layer switch of Sec. 3.1
    _, idx, gate = m2.route(x, vis)
    o = oracle.route(wl.x, wl.is_visual, wl.weights.router_w, wl.weights.router_bias, 6, 6)
    assert np.array_equal(host(idx), o[1]) and np.abs(host(gate) - o[2]).max() <= 1e-6


# ---------------------------------------------------------------- prune
@pytest.mark.parametrize("seed,kw", SMALL)
@pytest.mark.parametrize("sim_mode", [0, 1])
def test_prune(seed, kw, sim_mode):
    wl = _wl(seed, kw)
    o_probs, _, _ = oracle.route(wl.x, wl.is_visual, wl.weights.router_w, wl.weights.router_bias,
                                 wl.k_text, wl.k_visual)
    o_kept, o_cu, o_scores = oracle.prune(o_probs, wl.is_visual, wl.cu_seqlens, wl.retention, wl.window,
                                          sim_mode=sim_mode)
    m = make_layer(wl)
    pp = binding.prune_params(retention=wl.retention, window=wl.window, sim_mode=sim_mode)
    kept, new_cu, scores = m.prune(pp, dev(o_probs), dev(wl.is_visual), dev(wl.cu_seqlens), want_scores=True)
    torch.cuda.synchronize()
    new_cu = host(new_cu)
    assert np.array_equal(new_cu, o_cu)
    assert np.array_equal(host(kept)[:new_cu[-1]], o_kept)
    # scores live at slot cu[b] + i
    scores = host(scores)
    got = []
    for b in range(wl.B):
        s, e = wl.cu_seqlens[b], wl.cu_seqlens[b + 1]
        nv = int(wl.is_visual[s:e].sum())
        got.append(scores[s:s + (nv + wl.window - 1) // wl.window])
    got = np.concatenate(got) if got else np.zeros(0, np.float32)
    assert np.array_equal(got, o_scores)


@pytest.mark.parametrize("E,window", [(256, 9), (64, 40), (100, 21), (256, 8)])
@pytest.mark.parametrize("sim_mode", [0, 1])
def test_prune_windows_around_the_size_of_the_staging_tile(E, window, sim_mode):
    """The scoring kernel stages a window's probability rows in a tile of 2048 floats per wavefront and
    re-reads global memory for wider windows (W*E > 2048): both sides of that limit, ragged sequences, a
    ragged last window, with the attention term; scores, kept set and bounds bit for bit."""
    wl = W.small_random(140 + window, T_v=[3 * window + 2, 1, 7 * window, window - 1], T_t=[3, 2, 0, 5], d=32, E=E,
                        F=16, k_text=4, k_visual=2, retention=0.6, window=window, n_components=7, bias_std=1.0,
                        interleave=True)
    rng = np.random.default_rng(77)
    attn = rng.random(wl.T).astype(np.float32) ** 2
    o_probs, _, _ = oracle.route(wl.x, wl.is_visual, wl.weights.router_w, wl.weights.router_bias, 4, 2)
    o_kept, o_cu, o_scores = oracle.prune(o_probs, wl.is_visual, wl.cu_seqlens, wl.retention, window, alpha=0.7,
                                          attn=attn, sim_mode=sim_mode)
    m = make_layer(wl)
    pp = binding.prune_params(retention=wl.retention, window=window, alpha=0.7, sim_mode=sim_mode)
    kept, new_cu, scores = m.prune(pp, dev(o_probs), dev(wl.is_visual), dev(wl.cu_seqlens), attn=dev(attn),
                                   want_scores=True)
    torch.cuda.synchronize()
    new_cu = host(new_cu)
    assert np.array_equal(new_cu, o_cu)
    assert np.array_equal(host(kept)[:new_cu[-1]], o_kept)
    scores = host(scores)
    got = []
    for b in range(wl.B):
        s, e = wl.cu_seqlens[b], wl.cu_seqlens[b + 1]
        nv = int(wl.is_visual[s:e].sum())
        got.append(scores[s:s + (nv + window - 1) // window])
    assert np.array_equal(np.concatenate(got), o_scores)


@pytest.mark.parametrize("T_v,T_t", [([1023], [0]), ([1000], [24]), ([1024], [1]), ([700, 0, 2500, 1, 1900], [30, 5, 0, 0, 9])])
@pytest.mark.parametrize("gamma", [0.0, 0.2])
def test_prune_over_several_compaction_blocks(T_v, T_t, gamma):
    """The compaction runs over blocks of 1024 positions (position T carries the total): batches that end
    just below, at and above a block boundary and one of several ragged sequences over five blocks, with
    and without window merging; kept set, merged flags and sequence bounds bit for bit."""
    wl = W.small_random(171, T_v=T_v, T_t=T_t, d=32, E=16, F=16, k_text=3, k_visual=2, retention=0.45, window=3,
                        n_components=9, bias_std=1.0, interleave=True)
    o_probs, _, _ = oracle.route(wl.x, wl.is_visual, wl.weights.router_w, wl.weights.router_bias, 3, 2)
    o_kept, o_cu, _, o_mrg, _ = oracle.prune(o_probs, wl.is_visual, wl.cu_seqlens, wl.retention, 3, gamma=gamma,
                                             x=wl.x)
    m = make_layer(wl)
    pp = binding.prune_params(retention=wl.retention, window=3, gamma=gamma)
    if gamma > 0:
        kept, new_cu, _, mrg, _ = m.prune(pp, dev(o_probs), dev(wl.is_visual), dev(wl.cu_seqlens), x=dev(wl.x))
    else:
        kept, new_cu, _ = m.prune(pp, dev(o_probs), dev(wl.is_visual), dev(wl.cu_seqlens))
    torch.cuda.synchronize()
    new_cu = host(new_cu)
    assert np.array_equal(new_cu, o_cu)
    assert np.array_equal(host(kept)[:new_cu[-1]], o_kept)
    if gamma > 0:
        assert np.array_equal(host(mrg)[:new_cu[-1]], o_mrg)


@pytest.mark.parametrize("window,gamma", [(3, 0.0), (5, 0.0), (2, 0.25)])
def test_prune_many_short_sequences(window, gamma):
    """Several hundred sequences of zero to a dozen tokens, some without a visual token, some empty: every
    sequence owns its own window slots and window units, sequence bounds are found by binary search, and the
    compaction blocks cut through many sequences; kept set, scores and bounds bit for bit."""
    rng = np.random.default_rng(404)
    n_seq = 700
    T_v = [int(v) for v in rng.choice([0, 0, 1, 2, 3, 4, 5, 7, 11], size=n_seq)]
    T_t = [int(v) for v in rng.choice([0, 0, 1, 2], size=n_seq)]
    wl = W.small_random(405, T_v=T_v, T_t=T_t, d=32, E=12, F=16, k_text=3, k_visual=2, retention=0.5, window=window,
                        n_components=5, bias_std=1.0, interleave=True)
    assert wl.B == n_seq and wl.T > 2048
    o_probs, _, _ = oracle.route(wl.x, wl.is_visual, wl.weights.router_w, wl.weights.router_bias, 3, 2)
    res = oracle.prune(o_probs, wl.is_visual, wl.cu_seqlens, wl.retention, window, gamma=gamma,
                       x=wl.x if gamma > 0 else None)
    m = make_layer(wl)
    pp = binding.prune_params(retention=wl.retention, window=window, gamma=gamma)
    if gamma > 0:
        kept, new_cu, scores, mrg, _ = m.prune(pp, dev(o_probs), dev(wl.is_visual), dev(wl.cu_seqlens), x=dev(wl.x),
                                               want_scores=True)
    else:
        kept, new_cu, scores = m.prune(pp, dev(o_probs), dev(wl.is_visual), dev(wl.cu_seqlens), want_scores=True)
    torch.cuda.synchronize()
    new_cu = host(new_cu)
    assert np.array_equal(new_cu, res[1])
    assert np.array_equal(host(kept)[:new_cu[-1]], res[0])
    if gamma > 0:
        assert np.array_equal(host(mrg)[:new_cu[-1]], res[3])
    scores = host(scores)
    got = []
    for b in range(wl.B):
        s0, e0 = wl.cu_seqlens[b], wl.cu_seqlens[b + 1]
        nv = int(wl.is_visual[s0:e0].sum())
        got.append(scores[s0:s0 + (nv + window - 1) // window])
    assert np.array_equal(np.concatenate(got), res[2])


@pytest.mark.parametrize("alpha", [0.3, 0.6, 1.0])
def test_prune_with_attention_importance(alpha):
    wl = W.small_random(112, T_v=[75, 31], T_t=[6, 5], d=64, E=24, F=32, k_text=4, k_visual=2,
                        retention=0.5, window=5, n_components=5, interleave=True)
    rng = np.random.default_rng(5)
    attn = rng.random(wl.T).astype(np.float32) ** 2
    o_probs, _, _ = oracle.route(wl.x, wl.is_visual, wl.weights.router_w, None, 4, 2)
    o_kept, o_cu, _ = oracle.prune(o_probs, wl.is_visual, wl.cu_seqlens, 0.5, 5, alpha=alpha, attn=attn)
    m = make_layer(wl)
    pp = binding.prune_params(retention=0.5, window=5, alpha=alpha)
    kept, new_cu, _ = m.prune(pp, dev(o_probs), dev(wl.is_visual), dev(wl.cu_seqlens), attn=dev(attn))
    new_cu = host(new_cu)
    assert np.array_equal(new_cu, o_cu) and np.array_equal(host(kept)[:new_cu[-1]], o_kept)


def test_prune_tied_scores_identical_windows():
    # windows made of identical rows all score exactly alike: the index decides
    E, Wn, n = 16, 3, 20
    row = np.random.default_rng(6).random(E).astype(np.float32)
    row /= row.sum()
    probs = np.tile(row, (Wn * n, 1))
    vis = np.ones(Wn * n, np.uint8)
    cu = np.array([0, Wn * n], np.int32)
    o_kept, o_cu, o_sc = oracle.prune(probs, vis, cu, 0.5, Wn)
    assert len(set(o_sc.tolist())) == 1
    wl = W.small_random(113, T_v=[Wn * n], T_t=[0], d=64, E=E, F=32, k_text=2, k_visual=1,
                        retention=0.5, window=Wn)
    m = make_layer(wl)
    kept, new_cu, _ = m.prune(binding.prune_params(retention=0.5, window=Wn), dev(probs), dev(vis), dev(cu))
    new_cu = host(new_cu)
    assert np.array_equal(new_cu, o_cu) and np.array_equal(host(kept)[:new_cu[-1]], o_kept)
    assert list(o_kept) == list(range(Wn * n // 2, Wn * n))     # the first half of the windows goes


# ---------------------------------------------------------------- prune with window merging
def _merge_gammas(wl):
    g = [0.05, 0.3]
    if wl.window > 1 and wl.retention < 1.0:
        g.append(min(oracle.gamma_hat(wl.retention, wl.window, stages=1), 0.95))   # App. D: merging alone
    return g


def _check_merged_rows(x_m, o_xm, o_is_merged, dtype):
    """Ordinary rows are copies (bit-exact); merged rows are one rounding of an fp64 result on both
    sides, so they may differ by one unit in the last place where the fp64 sums disagree."""
    plain = o_is_merged == 0
    assert np.array_equal(x_m[plain], o_xm[plain])
    if (~plain).any():
        assert max_rel_err(x_m[~plain], o_xm[~plain]) <= TOL[dtype]
        assert (x_m[~plain] != o_xm[~plain]).mean() <= 1e-3


@pytest.mark.parametrize("seed,kw", SMALL)
def test_prune_merge(seed, kw):
    wl = _wl(seed, kw)
    bf = wl.dtype == W.BF16
    o_probs, _, _ = oracle.route(wl.x, wl.is_visual, wl.weights.router_w, wl.weights.router_bias,
                                 wl.k_text, wl.k_visual)
    m = make_layer(wl)
    x, vis, cu = inputs(wl)
    for gamma in _merge_gammas(wl):
        o_kept, o_cu, _, o_mrg, o_xm = oracle.prune(o_probs, wl.is_visual, wl.cu_seqlens, wl.retention,
                                                    wl.window, gamma=gamma, x=wl.x, is_bf16=bf)
        pp = binding.prune_params(retention=wl.retention, window=wl.window, gamma=gamma)
        kept, new_cu, _, mrg, x_m = m.prune(pp, dev(o_probs), vis, cu, x=x)
        torch.cuda.synchronize()
        new_cu = host(new_cu)
        n = int(new_cu[-1])
        assert np.array_equal(new_cu, o_cu), gamma
        assert np.array_equal(host(kept)[:n], o_kept), gamma
        assert np.array_equal(host(mrg)[:n], o_mrg), gamma
        _check_merged_rows(host(x_m)[:n], o_xm, o_mrg, wl.dtype)


@pytest.mark.parametrize("gamma", [0.02, 0.2, 0.7])
def test_prune_merge_with_attention_and_short_last_window(gamma):
    # N_v = 77 and 32 with W = 5: both sequences end in a 2-token window; the attention term moves the
    # last window around in the merge order
    wl = W.small_random(116, T_v=[77, 32], T_t=[6, 5], d=96, E=24, F=32, k_text=4, k_visual=2,
                        retention=0.4, window=5, n_components=5, interleave=True)
    rng = np.random.default_rng(7)
    attn = rng.random(wl.T).astype(np.float32) ** 2
    o_probs, _, _ = oracle.route(wl.x, wl.is_visual, wl.weights.router_w, None, 4, 2)
    m = make_layer(wl)
    x, vis, cu = inputs(wl)
    for alpha in (1.0, 0.5):
        a = None if alpha == 1.0 else attn
        o_kept, o_cu, _, o_mrg, o_xm = oracle.prune(o_probs, wl.is_visual, wl.cu_seqlens, 0.4, 5, alpha=alpha,
                                                    gamma=gamma, attn=a, x=wl.x)
        pp = binding.prune_params(retention=0.4, window=5, alpha=alpha, gamma=gamma)
        kept, new_cu, _, mrg, x_m = m.prune(pp, dev(o_probs), vis, cu, attn=dev(a), x=x)
        new_cu = host(new_cu)
        n = int(new_cu[-1])
        assert np.array_equal(new_cu, o_cu) and np.array_equal(host(kept)[:n], o_kept)
        assert np.array_equal(host(mrg)[:n], o_mrg)
        _check_merged_rows(host(x_m)[:n], o_xm, o_mrg, wl.dtype)


def test_prune_merge_many_windows_several_blocks():
    # more windows than one counting tile and one compaction pass hold
    wl = W.small_random(117, T_v=[2600, 1301], T_t=[40, 9], d=64, E=16, F=32, k_text=2, k_visual=1,
                        retention=0.5, window=3, n_components=20)
    o_probs, _, _ = oracle.route(wl.x, wl.is_visual, wl.weights.router_w, None, 2, 1)
    m = make_layer(wl)
    x, vis, cu = inputs(wl)
    for gamma in (0.05, oracle.gamma_hat(0.5, 3, stages=1) * 0.9):
        o_kept, o_cu, _, o_mrg, o_xm = oracle.prune(o_probs, wl.is_visual, wl.cu_seqlens, 0.5, 3, gamma=gamma,
                                                    x=wl.x)
        kept, new_cu, _, mrg, x_m = m.prune(binding.prune_params(retention=0.5, window=3, gamma=gamma),
                                            dev(o_probs), vis, cu, x=x)
        new_cu = host(new_cu)
        n = int(new_cu[-1])
        assert np.array_equal(new_cu, o_cu) and np.array_equal(host(kept)[:n], o_kept)
        assert np.array_equal(host(mrg)[:n], o_mrg) and o_mrg.sum() > 50
        _check_merged_rows(host(x_m)[:n], o_xm, o_mrg, wl.dtype)


# ---------------------------------------------------------------- permute
@pytest.mark.parametrize("seed,kw", SMALL)
def test_permute(seed, kw):
    wl = _wl(seed, kw)
    o = _oracle(wl, ffn=False)
    m = make_layer(wl)
    for kept in (o["kept_idx"], None):
        n = wl.T if kept is None else len(kept)
        if n == 0:
            continue
        o_offs, o_perm, o_inv = oracle.permute(o["topk_idx"], kept, wl.E)
        offs, perm, inv = m.permute(dev(o["topk_idx"]), dev(kept), n)
        torch.cuda.synchronize()
        assert np.array_equal(host(offs), o_offs)
        assert np.array_equal(host(perm)[:o_offs[-1]], o_perm)
        assert np.array_equal(host(inv)[:n], o_inv)


def test_permute_many_blocks_and_device_count():
    wl = W.small_random(114, T_v=[1500], T_t=[100], d=64, E=33, F=32, k_text=5, k_visual=2,
                        retention=0.5, window=3, bias_std=2.0)
    o = _oracle(wl, ffn=False)
    m = make_layer(wl)
    kept = o["kept_idx"]
    n = len(kept)
    kept_cap = np.concatenate([kept, np.zeros(wl.T - n, np.int32)])
    n_dev = dev(np.array([n], np.int32))
    offs, perm, inv = m.permute(dev(o["topk_idx"]), dev(kept_cap), wl.T, n_kept_dev=n_dev)
    assert np.array_equal(host(offs), o["expert_offsets"])
    assert np.array_equal(host(perm)[:o["expert_offsets"][-1]], o["perm_src"])
    assert np.array_equal(host(inv)[:n], o["inv_perm"])


# ---------------------------------------------------------------- experts + combine
SHAPES = [pytest.param(1, id="stream"), pytest.param(2, id="dense")]   # fmoe_set_ffn_shape (bf16 expert GEMMs)


def _skip_fp32_duplicate(wl, shape):
    if wl.dtype == W.F32 and shape == 2:
        pytest.skip("the GEMM shape only exists for bf16")


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("seed,kw", SMALL)
def test_expert_ffn_and_combine(seed, kw, shape):
    wl = _wl(seed, kw)
    _skip_fp32_duplicate(wl, shape)
    o = _oracle(wl, add_residual=True)
    n = len(o["kept_idx"])
    if n == 0:
        pytest.skip("empty")
    m = make_layer(wl, ffn_shape=shape)
    x, vis, cu = inputs(wl)
    kept = dev(o["kept_idx"])
    y, ysh = m.expert_ffn(x, kept, n, dev(o["expert_offsets"]), dev(o["perm_src"]))
    torch.cuda.synchronize()
    M = int(o["expert_offsets"][-1])
    tol = TOL[wl.dtype]
    if M > 0:
        assert max_rel_err(host(y)[:M], o["y"]) <= tol
    if wl.n_shared:   # per-expert outputs; the oracle holds their sum
        assert max_rel_err(host(ysh).astype(np.float64).sum(0)[:n], o["y_shared"]) <= tol
    out = m.combine(y, ysh, dev(o["inv_perm"]), dev(o["topk_gate"]), kept, n, residual=x)
    assert_residual_outputs_close(host(out)[:n], o["out_f64"], _x_rows(wl, o), wl.dtype, "combine + residual")
    o_plain = _oracle(wl)                                   # and the expert term on its own
    out = m.combine(y, ysh, dev(o["inv_perm"]), dev(o["topk_gate"]), kept, n)
    assert_outputs_close(host(out)[:n], o_plain["out_f64"], wl.dtype, "combine")


# ---------------------------------------------------------------- whole layer
@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("seed,kw", SMALL)
def test_layer_forward(seed, kw, shape):
    wl = _wl(seed, kw)
    _skip_fp32_duplicate(wl, shape)
    o = _oracle(wl, add_residual=True)
    m = make_layer(wl, ffn_shape=shape)
    x, vis, cu = inputs(wl)
    pp = binding.prune_params(retention=wl.retention, window=wl.window)
    out, kept, new_cu, vis_out = m.layer_forward(x, vis, cu, pp, add_residual=True, want_mask=True)
    torch.cuda.synchronize()
    new_cu = host(new_cu)
    n = int(new_cu[-1])
    assert np.array_equal(new_cu, o["new_cu_seqlens"])
    assert np.array_equal(host(kept)[:n], o["kept_idx"])
    assert np.array_equal(host(vis_out)[:n], wl.is_visual[o["kept_idx"]])
    if n:
        assert_residual_outputs_close(host(out)[:n], o["out_f64"], _x_rows(wl, o), wl.dtype, "layer + residual")
    # determinism: a second run gives identical bits
    out2, kept2, _, _ = m.layer_forward(x, vis, cu, pp, add_residual=True)
    assert torch.equal(out[:n], out2[:n]) and torch.equal(kept[:n], kept2[:n])
    # the expert term on its own (Eq.4 without the residual), at the tolerance proper
    out3, _, _, _ = m.layer_forward(x, vis, cu, pp)
    if n:
        assert_outputs_close(host(out3)[:n], _oracle(wl)["out_f64"], wl.dtype, "layer")


def test_layer_forward_equals_chained_calls_and_no_prune_path():
    wl = W.small_random(115, T_v=[200, 90], T_t=[17, 8], d=128, E=32, F=64, k_text=4, k_visual=2,
                        retention=0.5, window=3, dtype=W.BF16, n_shared=1, F_shared=32, bias_std=1.0,
                        n_components=8)
    m = make_layer(wl)
    x, vis, cu = inputs(wl)
    pp = binding.prune_params(retention=0.5, window=3)
    out, kept, new_cu, _ = m.layer_forward(x, vis, cu, pp)
    n = int(host(new_cu)[-1])
    probs, idx, gate = m.route(x, vis)
    kept2, new_cu2, _ = m.prune(pp, probs, vis, cu)
    assert torch.equal(new_cu, new_cu2) and torch.equal(kept[:n], kept2[:n])
    offs, perm, inv = m.permute(idx.contiguous(), kept2, n)
    y, ysh = m.expert_ffn(x, kept2, n, offs, perm)
    out2 = m.combine(y, ysh, inv, gate.contiguous(), kept2, n)
    assert torch.equal(out[:n], out2[:n])
    # params = None and retention = 1 both mean: keep everything
    for p in (None, binding.prune_params(retention=1.0, window=3)):
        out3, kept3, new_cu3, _ = m.layer_forward(x, vis, cu, p)
        assert np.array_equal(host(new_cu3), wl.cu_seqlens)
        assert np.array_equal(host(kept3), np.arange(wl.T))
        o = _oracle(wl, retention=1.0)
        assert max_rel_err(host(out3), o["out_f64"]) <= TOL[wl.dtype]


@pytest.mark.parametrize("seed,kw", SMALL)
def test_layer_forward_merge(seed, kw):
    # Sec. 3.2.3 inside the layer: merged layer input, kept tokens routed again, experts on that tensor
    wl = _wl(seed, kw)
    m = make_layer(wl)
    x, vis, cu = inputs(wl)
    for gamma in _merge_gammas(wl)[-2:]:
        o = _oracle(wl, add_residual=True, gamma=gamma)
        pp = binding.prune_params(retention=wl.retention, window=wl.window, gamma=gamma)
        out, kept, new_cu, vis_out = m.layer_forward(x, vis, cu, pp, add_residual=True, want_mask=True)
        torch.cuda.synchronize()
        new_cu = host(new_cu)
        n = int(new_cu[-1])
        assert np.array_equal(new_cu, o["new_cu_seqlens"])
        assert np.array_equal(host(kept)[:n], o["kept_idx"])
        assert np.array_equal(host(vis_out)[:n], wl.is_visual[o["kept_idx"]])
        if n:
            assert_residual_outputs_close(host(out)[:n], o["out_f64"], _x_rows(wl, o), wl.dtype, f"gamma {gamma}")
            out2, _, _, _ = m.layer_forward(x, vis, cu, pp)
            assert_outputs_close(host(out2)[:n], _oracle(wl, gamma=gamma)["out_f64"], wl.dtype, f"gamma {gamma}")


def _check_after_layer_rows(got, o, x_all, dtype, what):
    """Output rows of a layer that merges after the layer (oracle record `o` of after_layer=True; x_all:
    the layer input when the residual was added, else None).  Ordinary kept rows: the un-pruned layer's
    rows at the dtype's tolerance.  Merged rows: each side merges its own stored output rows (which
    differ by the GEMM's rounding) with one rounding of an fp64 result at the end, and the rescaling to
    the largest row norm can stretch a difference by the ratio of that norm to the mean's."""
    k = o["kept_idx"]
    plain = o["is_merged"] == 0
    ref64 = o["out_full_f64"]
    if x_all is not None:
        assert_residual_outputs_close(got[plain], ref64[k[plain]], x_all[k[plain]], dtype, what)
        scale = np.abs(ref64 - x_all).max()
    else:
        assert_outputs_close(got[plain], ref64[k[plain]], dtype, what)
        scale = np.abs(ref64).max()
    if (~plain).any():
        g = got[~plain].astype(np.float64)
        r = o["out"][~plain].astype(np.float64)
        bound = 4 * TOL[dtype] * scale + 4 * HALF_ULP[dtype] * np.maximum(np.abs(g), np.abs(r))
        assert (np.abs(g - r) <= bound).all(), (what, float(np.abs(g - r).max()), float(scale))


@pytest.mark.parametrize("seed,kw", SMALL)
def test_layer_forward_merge_after_the_layer(seed, kw):
    """Sec. 3.2.3 applied to the layer's output (prune_mode 2 with gamma > 0): the experts run on every
    token, the windows are scored on this layer's probabilities, and the output rows are compacted with
    merged windows replaced by the merged row of their tokens' outputs (Eq.16-18)."""
    wl = _wl(seed, kw)
    m = make_layer(wl)
    x, vis, cu = inputs(wl)
    for residual in (True, False):
        full_gpu = host(m.layer_forward(x, vis, cu, None, add_residual=residual)[0]).copy()
        for gamma in _merge_gammas(wl)[-2:]:
            o = _oracle(wl, add_residual=residual, gamma=gamma, after_layer=True)
            pp = binding.prune_params(retention=wl.retention, window=wl.window, gamma=gamma, prune_mode=2)
            out, kept, new_cu, vis_out = m.layer_forward(x, vis, cu, pp, add_residual=residual, want_mask=True)
            torch.cuda.synchronize()
            new_cu = host(new_cu)
            n = int(new_cu[-1])
            what = f"gamma {gamma} residual {residual}"
            assert np.array_equal(new_cu, o["new_cu_seqlens"]), what
            assert np.array_equal(host(kept)[:n], o["kept_idx"]), what
            assert np.array_equal(host(vis_out)[:n], wl.is_visual[o["kept_idx"]]), what
            if not n:
                continue
            got = host(out)[:n]
            k = o["kept_idx"]
            # an ordinary kept row is the un-pruned layer's row, bit for bit on the GPU
            assert np.array_equal(got[o["is_merged"] == 0], full_gpu[k[o["is_merged"] == 0]]), what
            _check_after_layer_rows(got, o, wl.x if residual else None, wl.dtype, what)


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
@pytest.mark.parametrize("B", [0, 3])
def test_empty_batch(dtype, B):
    """No tokens at all (no sequences, or sequences that are all empty): every entry point returns without
    work, the fused layer reports zero kept tokens per sequence, and a normal batch run right after on the
    same context is unaffected."""
    wl = _wl(108 if dtype == W.BF16 else 101, SMALL[8 if dtype == W.BF16 else 1].values[1])
    m = make_layer(wl)
    td = torch_dtype(wl)
    x0 = torch.empty((0, wl.d), dtype=td, device="cuda")
    vis0 = torch.empty(0, dtype=torch.uint8, device="cuda")
    cu0 = torch.zeros(B + 1, dtype=torch.int32, device="cuda")
    for pp in (None, binding.prune_params(retention=0.5, window=3),
               binding.prune_params(retention=0.5, window=3, gamma=0.1),
               binding.prune_params(retention=0.5, window=3, gamma=0.1, prune_mode=2)):
        new_cu = torch.full((B + 1,), 7, dtype=torch.int32, device="cuda")
        m.layer_forward(x0, vis0, cu0, pp, new_cu=new_cu)
        torch.cuda.synchronize()
        assert not host(new_cu).any()
    probs, idx, gate = m.route(x0, vis0)
    assert probs.shape[0] == 0 and idx.shape[0] == 0
    kept, new_cu, _ = m.prune(binding.prune_params(retention=0.5, window=3), probs, vis0, cu0)
    offs, perm, inv = m.permute(idx.contiguous(), None, 0)
    torch.cuda.synchronize()
    assert not host(new_cu).any() and not host(offs).any()
    y, ysh = m.expert_ffn(x0, None, 0, offs, perm)
    m.combine(y, ysh, inv, gate.contiguous(), None, 0)
    torch.cuda.synchronize()
    # the context still works
    x, vis, cu = inputs(wl)
    out, kept, new_cu, _ = m.layer_forward(x, vis, cu, binding.prune_params(retention=wl.retention, window=wl.window))
    torch.cuda.synchronize()
    o = _oracle(wl)
    n = int(host(new_cu)[-1])
    assert np.array_equal(host(kept)[:n], o["kept_idx"])
    assert max_rel_err(host(out)[:n], o["out_f64"]) <= TOL[wl.dtype]


@pytest.mark.parametrize("gamma", [0.0, 0.3])
def test_layer_forward_replays_from_a_captured_graph(gamma):
    """The fused layer is kernel launches only (no allocation, no host synchronisation, no memset), so a
    caller can capture it into a graph.  Every replay, with eager work and synchronisations of the
    program in between, must give the eager call's result bit for bit."""
    wl = _wl(108, SMALL[8].values[1])
    m = make_layer(wl)
    x, vis, cu = inputs(wl)
    pp = binding.prune_params(retention=wl.retention, window=wl.window, gamma=gamma)
    out_e, kept_e, cu_e, _ = m.layer_forward(x, vis, cu, pp, add_residual=True)   # also sizes the workspace
    torch.cuda.synchronize()
    n = int(host(cu_e)[-1])
    ref_out, ref_kept, ref_cu = host(out_e)[:n].copy(), host(kept_e)[:n].copy(), host(cu_e).copy()
    out_g, kept_g, cu_g = torch.empty_like(out_e), torch.empty_like(kept_e), torch.empty_like(cu_e)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        m.layer_forward(x, vis, cu, pp, add_residual=True, out=out_g, kept_idx=kept_g, new_cu=cu_g)
    for rep in range(4):
        out_g.fill_(float("nan"))
        kept_g.fill_(-1)
        cu_g.fill_(-1)
        junk = (x.float() * (rep + 1)).sum()   # eager work of the program between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.isfinite(float(junk))
        assert np.array_equal(host(cu_g), ref_cu), rep
        assert np.array_equal(host(kept_g)[:n], ref_kept), rep
        assert np.array_equal(host(out_g)[:n], ref_out), rep


# ---------------------------------------------------------------- the benchmark configurations
def _check_layer(m, wl, x_np, vis_np, cu_np, lw, k_text, k_visual, do_prune, add_residual=False, what=""):
    """One fused layer on the GPU against the oracle's layer on the same input bytes: expert ids,
    probabilities, kept set, sequence bounds and permutation bit for bit; outputs on EVERY kept row
    within the dtype's tolerance.  Returns the oracle's result (its output feeds the next layer of a
    teacher-forced stack: the oracle never sees a value from the GPU)."""
    is_bf16 = wl.dtype == W.BF16
    td = torch_dtype(wl)
    x, vis, cu = dev(x_np, td), dev(vis_np), dev(cu_np)
    m.set_topk(k_text, k_visual)
    pp = binding.prune_params(retention=wl.retention, window=wl.window) if do_prune else None
    out, kept, new_cu, vis_out = m.layer_forward(x, vis, cu, pp, add_residual=add_residual, want_mask=True)
    torch.cuda.synchronize()
    o = oracle.layer_forward(x_np, vis_np, cu_np, lw, k_text=k_text, k_visual=k_visual, is_bf16=is_bf16,
                             retention=wl.retention, window=wl.window, do_prune=do_prune,
                             add_residual=add_residual)
    new_cu = host(new_cu)
    n = int(new_cu[-1])
    assert np.array_equal(new_cu, o["new_cu_seqlens"]), what
    assert np.array_equal(host(kept)[:n], o["kept_idx"]), what
    assert np.array_equal(host(vis_out)[:n], vis_np[o["kept_idx"]]), what
    probs, idx, gate = m.route(x, vis)
    assert np.array_equal(host(idx), o["topk_idx"]), what
    assert np.array_equal(host(probs), o["probs"]), what
    assert np.abs(host(gate) - o["topk_gate"]).max() <= 1e-6, what
    offs, perm, inv = m.permute(idx.contiguous(), kept, n)
    assert np.array_equal(host(offs), o["expert_offsets"]), what
    assert np.array_equal(host(perm)[:o["expert_offsets"][-1]], o["perm_src"]), what
    assert np.array_equal(host(inv)[:n], o["inv_perm"]), what
    got = host(out)[:n]
    assert np.isfinite(got).all(), what
    if add_residual:
        assert_residual_outputs_close(got, o["out_f64"], x_np[o["kept_idx"]], wl.dtype, what)
        # and the expert term alone (Eq.4 without the residual) at the tolerance proper
        out2, _, _, _ = m.layer_forward(x, vis, cu, pp)
        torch.cuda.synchronize()
        moe_ref = o["out_f64"] - x_np[o["kept_idx"]].astype(np.float64)
        assert_outputs_close(host(out2)[:n], moe_ref, wl.dtype, what + ", expert term")
    else:
        assert_outputs_close(got, o["out_f64"], wl.dtype, what)
    return o


def _check_config(wl):
    m = make_layer(wl)
    o = _check_layer(m, wl, wl.x, wl.is_visual, wl.cu_seqlens, wl.weights, wl.k_text, wl.k_visual,
                     do_prune=wl.retention < 1.0, what=wl.name)
    return len(o["kept_idx"])


@pytest.mark.parametrize("cfg", ["c2", "s108", "kloop"])
def test_expert_gemm_shapes_agree_bit_for_bit(cfg):
    """Both shapes of the bf16 expert GEMM add the products of a dot product in ascending k: whatever the
    size, they must give the same bits (fmoe_set_ffn_shape)."""
    wl = {"c2": W.config2, "s108": lambda: _wl(108, SMALL[8].values[1]),
          "kloop": lambda: W.small_random(8123, T_v=[150, 40], T_t=[30, 7], d=712, E=12, F=456, k_text=4, k_visual=2,
                                          retention=0.5, window=3, dtype=W.BF16, n_shared=1, F_shared=392,
                                          bias_std=1.5)}[cfg]()
    x, vis, cu = inputs(wl)
    pp = binding.prune_params(retention=wl.retention, window=wl.window)
    outs = []
    for shape in (1, 2):
        m = make_layer(wl, ffn_shape=shape)
        out, kept, new_cu, _ = m.layer_forward(x, vis, cu, pp)
        n = int(host(new_cu)[-1])
        outs.append(out[:n].clone())
    assert torch.equal(outs[0], outs[1])
    with pytest.raises(RuntimeError):
        m.set_ffn_shape(3)


def test_config2_dsvl2_tiny_dense_shape():
    wl = W.config2()
    m = make_layer(wl, ffn_shape=2)
    o = _check_layer(m, wl, wl.x, wl.is_visual, wl.cu_seqlens, wl.weights, wl.k_text, wl.k_visual, do_prune=True,
                     what="c2, dense shape")
    assert len(o["kept_idx"]) == 768 + 64


def test_config1_tiny_fp32():
    assert _check_config(W.config1()) == 52


def test_config2_dsvl2_tiny():
    assert _check_config(W.config2()) == 768 + 64


@pytest.mark.parametrize("retention,kept_visual", [(0.25, 960), (0.5, 1920), (0.75, 2880)])
def test_config3_dsvl2_small_retention_sweep(retention, kept_visual):
    # every kept row of the full-size layer is compared (the oracle's layer takes about ten seconds)
    assert _check_config(W.config3(retention)) == kept_visual + 256


def test_config3_full_activation_no_pruning():
    # the standard MoE layer (k 6/6, r = 1): the reference point of the retention sweep, 384 rows per expert
    wl = W.config3(1.0, k_visual=6)
    assert _check_config(wl) == wl.T


def test_config4_internvl35():
    assert _check_config(W.config4()) == 3968 + 256


# ---------------------------------------------------------------- the ragged multi-layer stack
def _lens(wl):
    lens = np.diff(wl.cu_seqlens)
    nv = [int(wl.is_visual[s:e].sum()) for s, e in zip(wl.cu_seqlens[:-1], wl.cu_seqlens[1:])]
    return nv, [int(n - v) for n, v in zip(lens, nv)]


def _oracle_stack(wl, schedule=None, layers=None):
    """x <- x + MoE_l(x) layer by layer on the CPU; `schedule` = {layer: dict(retention, window, alpha,
    gamma)} (default: one stage after `prune_after_layer`).  Returns the final (x, kept_total, cu) and
    the per-layer records (input x / mask / cu, the oracle's result)."""
    is_bf16 = wl.dtype == W.BF16
    if schedule is None:
        schedule = {wl.prune_after_layer: dict(retention=wl.retention, window=wl.window)}
    x, vis, cu = wl.x, wl.is_visual, wl.cu_seqlens
    kept_total = None
    records = []
    for l in range(len(wl.layers)):
        lw = wl.layers[l] if layers is None else layers[l]
        kt, kv = wl.k_schedule[l]
        st = schedule.get(l)
        o = oracle.layer_forward(x, vis, cu, lw, k_text=kt, k_visual=kv, is_bf16=is_bf16,
                                 add_residual=True, do_prune=st is not None,
                                 **(st if st is not None else dict(retention=1.0, window=wl.window)))
        records.append(dict(x=x, vis=vis, cu=cu, o=o, stage=st))
        if st is not None:
            kept = o["kept_idx"]
            kept_total = kept if kept_total is None else kept_total[kept]
            vis, cu = vis[kept], o["new_cu_seqlens"]
        x = o["out"]
    return x, kept_total, cu, records


def _gpu_layers(wl):
    return [make_layer(wl, layer=l) for l in range(len(wl.layers))]


def _gpu_stack(wl, layers, schedule=None):
    """The stack through fmoe_stack_forward.  schedule: {layer: prune params}."""
    if schedule is None:
        schedule = {wl.prune_after_layer: binding.prune_params(retention=wl.retention, window=wl.window, prune_mode=2)}
    stack = binding.FMoEStack(layers, wl.k_schedule, prune_schedule=schedule)
    x, vis, cu = inputs(wl)
    nv, nt = _lens(wl)
    out, kept, new_cu = stack.forward(x, vis, cu, nv, nt)
    torch.cuda.synchronize()
    return out, kept, new_cu


def _gpu_chain(wl, layers, schedule):
    """The same stack as single fmoe_layer_forward calls chained by the test (what fmoe_stack_forward
    must reproduce bit for bit: same kernels, same order)."""
    x, vis, cu = inputs(wl)
    kept_total = None
    for l, m in enumerate(layers):
        m.set_topk(*wl.k_schedule[l])
        pp = schedule.get(l)
        out, kept, new_cu, vis_out = m.layer_forward(x, vis, cu, pp, add_residual=True, want_mask=pp is not None)
        if pp is not None:
            n = int(host(new_cu)[-1])
            kept_total = kept[:n].clone() if kept_total is None else kept_total[kept[:n].long()]
            x, vis, cu = out[:n].clone(), vis_out[:n].clone(), new_cu.clone()
        else:
            x = out[:x.shape[0]].clone()
    return x, kept_total, cu


def _teacher_forced(wl, layers, records, only=None):
    """Every GPU layer gets the ORACLE's input of that layer: decisions bit for bit and outputs on every
    kept row at the dtype's tolerance, at every layer, unconditionally."""
    for l, r in enumerate(records):
        if only is not None and l not in only:
            continue
        st = r["stage"]
        m = layers[l]
        kt, kv = wl.k_schedule[l]
        is_bf16 = wl.dtype == W.BF16
        td = torch_dtype(wl)
        x, vis, cu = dev(r["x"], td), dev(r["vis"]), dev(r["cu"])
        m.set_topk(kt, kv)
        pp = None
        if st is not None:
            after = st.get("after_layer", False) or not st.get("gamma", 0.0) > 0
            pp = binding.prune_params(retention=st["retention"], window=st["window"], alpha=st.get("alpha", 1.0),
                                      gamma=st.get("gamma", 0.0), prune_mode=2 if after else 1)
        out, kept, new_cu, _ = m.layer_forward(x, vis, cu, pp, add_residual=True)
        torch.cuda.synchronize()
        o = r["o"]
        new_cu = host(new_cu)
        n = int(new_cu[-1])
        assert np.array_equal(new_cu, o["new_cu_seqlens"]), l
        assert np.array_equal(host(kept)[:n], o["kept_idx"]), l
        _, idx, gate = m.route(x, vis, want_probs=False)
        if "x_merged" not in o:                       # (with merging the list is that of the merged input)
            assert np.array_equal(host(idx), o["topk_idx"]), l
        if "out_full_f64" in o:                       # merging after the layer
            _check_after_layer_rows(host(out)[:n], o, r["x"], wl.dtype, f"layer {l}")
        else:
            assert_residual_outputs_close(host(out)[:n], o["out_f64"], _x_rows_of(r), wl.dtype, f"layer {l}")


def _x_rows_of(r):
    o = r["o"]
    return o["x_merged"] if "x_merged" in o else r["x"][o["kept_idx"]]


@pytest.mark.parametrize("gamma,prune_mode", [(0.0, 1), (0.05, 1), (0.05, 2)])
def test_stack_three_stage_schedule_fp32(gamma, prune_mode):
    # App. D: r = 0.5 reached in three stages of beta = r^(1/3) after layers 2, 5, 8 (the DeepSeek-VL2
    # setting of App. A: W = 3, gamma = 0.05), reduced top-k from layer 2 on; merging on the layer input
    # (mode 1) or on the layer output (mode 2)
    wl = W.config5(n_layers=10, d=128, E=64, F=64, len_div=32, text_len=128, dtype=W.F32)
    sched = binding.stage_schedule(0.5, [2, 5, 8], window=3, gamma=gamma, prune_mode=prune_mode)
    assert abs(sched[2].retention ** 3 - 0.5) < 1e-6
    o_sched = {l: dict(retention=p.retention, window=p.window, alpha=p.alpha, gamma=p.gamma,
                       after_layer=prune_mode == 2)
               for l, p in sched.items()}
    layers = _gpu_layers(wl)
    ref, ref_kept, ref_cu, records = _oracle_stack(wl, o_sched)
    _teacher_forced(wl, layers, records)                      # per layer: 1e-5, decisions bit for bit
    out, kept, new_cu = _gpu_stack(wl, layers, sched)         # the library's stack driver ...
    c_out, c_kept, c_cu = _gpu_chain(wl, layers, sched)       # ... equals the chained single-layer calls
    assert torch.equal(out, c_out) and torch.equal(kept, c_kept) and torch.equal(new_cu, c_cu)
    # (free-running, the two sides' activations differ by fp32 rounding after the first layer, which may
    # flip a near-tied later decision: decisions are compared layer by layer on identical inputs above;
    # the per-sequence counts are exact whatever near-ties do)
    assert np.array_equal(host(new_cu), ref_cu)
    assert kept.shape[0] == ref_kept.shape[0]
    nv, nt = _lens(wl)
    lens = nv
    for _ in range(3):
        lens = binding.kept_visual_lens(lens, sched[2].retention)
    assert out.shape[0] == sum(lens) + sum(nt) == ref.shape[0]
    assert abs(sum(lens) / sum(nv) - 0.5) < 0.02           # the cumulative ratio of App. D


def test_stack_ragged_12_layers_fp32():
    # config 5 in structure (8 ragged sequences, 12 layers, k 6/6 then 6/3, pruning after layer 2)
    # at sizes the oracle finishes in seconds
    wl = W.config5(n_layers=12, d=128, E=64, F=64, len_div=32, text_len=128, dtype=W.F32)
    layers = _gpu_layers(wl)
    ref, ref_kept, ref_cu, records = _oracle_stack(wl)
    _teacher_forced(wl, layers, records)
    sched = {wl.prune_after_layer: binding.prune_params(retention=wl.retention, window=wl.window, prune_mode=2)}
    out, kept, new_cu = _gpu_stack(wl, layers)
    c_out, c_kept, c_cu = _gpu_chain(wl, layers, sched)
    assert torch.equal(out, c_out) and torch.equal(kept, c_kept) and torch.equal(new_cu, c_cu)
    assert np.array_equal(host(new_cu), ref_cu)
    nv, nt = _lens(wl)
    assert out.shape[0] == binding.kept_count(nv, nt, wl.retention) == ref.shape[0] == kept.shape[0]


def test_stack_stages_take_their_attention_importance():
    """fmoe_stack_forward hands attn[l] (Eq.7, one vector per stage, sized for the tokens that reach the
    stage) to the stage of layer l: with alpha < 1 the stack must equal the chained single-layer calls
    bit for bit, differ from the stack run without attention, and the first stage must keep the
    oracle's set."""
    wl = W.config5(n_layers=6, d=128, E=64, F=64, len_div=32, text_len=96, dtype=W.F32)
    layers = _gpu_layers(wl)
    sched = binding.stage_schedule(0.5, [1, 3], window=3, alpha=0.5)
    nv, nt = _lens(wl)
    T1 = wl.T
    T2 = binding.kept_count(nv, nt, sched[1].retention)
    rng = np.random.default_rng(31)
    attn = {1: dev(rng.random(T1).astype(np.float32) ** 2), 3: dev(rng.random(T2).astype(np.float32) ** 2)}
    stack = binding.FMoEStack(layers, wl.k_schedule, prune_schedule=sched)
    x, vis, cu = inputs(wl)
    out, kept, new_cu = stack.forward(x, vis, cu, nv, nt, attn=attn)
    out0, kept0, _ = stack.forward(x, vis, cu, nv, nt)
    torch.cuda.synchronize()
    # the same stack as chained calls with the same attention vectors
    xc, visc, cuc = x, vis, cu
    kept_total = None
    for l, m in enumerate(layers):
        m.set_topk(*wl.k_schedule[l])
        pp = sched.get(l)
        o, k, ncu, vout = m.layer_forward(xc, visc, cuc, pp, attn=attn.get(l), add_residual=True, want_mask=pp is not None)
        if pp is not None:
            n = int(host(ncu)[-1])
            assert n == (T2 if l == 1 else out.shape[0])
            kept_total = k[:n].clone() if kept_total is None else kept_total[k[:n].long()]
            xc, visc, cuc = o[:n].clone(), vout[:n].clone(), ncu.clone()
        else:
            xc = o[:xc.shape[0]].clone()
    assert torch.equal(out, xc) and torch.equal(kept, kept_total) and torch.equal(new_cu, cuc)
    assert not torch.equal(kept, kept0)                       # the attention term changed the kept set
    # the stack's modality mask of its output rows (with and without stages)
    _, kept_m, _, mask = stack.forward(x, vis, cu, nv, nt, attn=attn, want_mask=True)
    assert torch.equal(kept_m, kept) and np.array_equal(host(mask), wl.is_visual[host(kept)])
    plain = binding.FMoEStack(layers[:2], wl.k_schedule[:2], prune_schedule={})
    _, kept_p, _, mask_p = plain.forward(x, vis, cu, nv, nt, want_mask=True)
    assert np.array_equal(host(kept_p), np.arange(wl.T)) and np.array_equal(host(mask_p), wl.is_visual)
    # first stage against the oracle (layer 0 without pruning, then layer 1 with the attention term)
    lw0, lw1 = wl.layers[0], wl.layers[1]
    o0 = oracle.layer_forward(wl.x, wl.is_visual, wl.cu_seqlens, lw0, k_text=wl.k_schedule[0][0],
                              k_visual=wl.k_schedule[0][1], is_bf16=False, add_residual=True, do_prune=False,
                              retention=1.0, window=3)
    m1 = layers[1]
    m1.set_topk(*wl.k_schedule[1])
    _, k1, ncu1, _ = m1.layer_forward(dev(o0["out"]), vis, cu, sched[1], attn=attn[1], add_residual=True)
    o1 = oracle.layer_forward(o0["out"], wl.is_visual, wl.cu_seqlens, lw1, k_text=wl.k_schedule[1][0],
                              k_visual=wl.k_schedule[1][1], is_bf16=False, add_residual=True, do_prune=True,
                              retention=sched[1].retention, window=3, alpha=0.5, attn=host(attn[1]))
    n1 = int(host(ncu1)[-1])
    assert np.array_equal(host(ncu1), o1["new_cu_seqlens"]) and np.array_equal(host(k1)[:n1], o1["kept_idx"])


def test_stack_without_stages_returns_the_identity_index_list():
    wl = W.config5(n_layers=2, d=64, E=16, F=32, len_div=64, text_len=64, dtype=W.F32)
    layers = _gpu_layers(wl)
    out, kept, new_cu = _gpu_stack(wl, layers, schedule={})
    c_out, _, _ = _gpu_chain(wl, layers, {})
    assert torch.equal(out, c_out)
    assert np.array_equal(host(kept), np.arange(wl.T)) and np.array_equal(host(new_cu), wl.cu_seqlens)


def test_stack_ragged_bf16_teacher_forced():
    # bf16 storage, config 5's schedule over six layers.  Rounding differences between the sides can flip
    # later near-tied decisions of a free-running stack, so every GPU layer is fed the oracle's input for
    # that layer: ids, kept set and permutation must then agree bit for bit and the outputs within 2e-2
    # at every layer
    wl = W.config5(n_layers=6, d=256, E=64, F=128, len_div=16, text_len=64)
    layers = _gpu_layers(wl)
    ref, ref_kept, ref_cu, records = _oracle_stack(wl)
    _teacher_forced(wl, layers, records)
    sched = {wl.prune_after_layer: binding.prune_params(retention=wl.retention, window=wl.window, prune_mode=2)}
    out, kept, new_cu = _gpu_stack(wl, layers)
    c_out, c_kept, c_cu = _gpu_chain(wl, layers, sched)
    assert torch.equal(out, c_out) and torch.equal(kept, c_kept) and torch.equal(new_cu, c_cu)
    nv, nt = _lens(wl)
    assert out.shape[0] == binding.kept_count(nv, nt, wl.retention) == ref.shape[0]
    assert np.array_equal(host(new_cu), ref_cu)               # counts are exact whatever the near-ties do


# ---------------------------------------------------------------- config 5 at its real size
# 8 packed sequences (22016 tokens), d = 2048, 64 experts of 1408 + 2 shared, 12 layers of distinct
# weights, k 6/6 in layers 0-1 and 6/3 from layer 2, pruning to 50 % once in layer 2.
_C5 = {}


def _c5():
    if "wl" not in _C5:
        _C5["wl"] = W.config5()
        _C5["input"] = (_C5["wl"].x, _C5["wl"].is_visual, _C5["wl"].cu_seqlens)
    return _C5["wl"]


@pytest.mark.parametrize("layer", [0, 1, 2, 3])
def test_config5_full_size_layers_teacher_forced(layer):
    """Layers 0-3 of the full-size stack (two full-activation layers with about 2000 rows per expert, the
    pruning layer, the first layer on the pruned batch), each on the oracle's own output of the layer
    before it: every decision bit for bit, outputs on all kept rows."""
    wl = _c5()
    if layer > 0 and _C5.get("done") != layer - 1:
        pytest.skip("needs the oracle's output of the layer before (run the layers in order)")
    x_np, vis_np, cu_np = _C5["input"]
    lw = wl.layers[layer]
    kt, kv = wl.k_schedule[layer]
    td = torch_dtype(wl)
    m = binding.FMoE(d_model=wl.d, n_experts=wl.E, d_ffn=wl.F, n_shared=wl.n_shared, d_ffn_shared=wl.F_shared,
                     k_text=kt, k_visual=kv, dtype=wl.dtype)
    m.set_weights(dev(lw.router_w, td), dev(lw.router_bias), dev(lw.w_gate, td), dev(lw.w_up, td),
                  dev(lw.w_down, td), dev(lw.ws_gate, td), dev(lw.ws_up, td), dev(lw.ws_down, td))
    do_prune = layer == wl.prune_after_layer
    o = _check_layer(m, wl, x_np, vis_np, cu_np, lw, kt, kv, do_prune, add_residual=True, what=f"c5 layer {layer}")
    if layer < 2:
        assert len(o["kept_idx"]) == wl.T and int(o["expert_offsets"][-1]) == 6 * wl.T
    if do_prune:
        nv, nt = _lens(wl)
        assert len(o["kept_idx"]) == binding.kept_count(nv, nt, wl.retention)
        vis_np, cu_np = vis_np[o["kept_idx"]], o["new_cu_seqlens"]
    _C5["input"] = (o["out"], vis_np, cu_np)
    _C5["done"] = layer
    m.close()
    del m
    torch.cuda.empty_cache()


def test_config5_full_size_stack_runs_all_twelve_layers():
    """The whole config-5 stack at its real size through fmoe_stack_forward: row count, sequence bounds
    and index list against the host bookkeeping, outputs finite; the first three layers re-run as
    chained single-layer calls reproduce the stack's pruning decisions."""
    import concurrent.futures as cf
    wl = _c5()
    td = torch_dtype(wl)

    def make(l):
        lw = wl.layers[l]
        return lw

    layers = []
    with cf.ThreadPoolExecutor(max_workers=3) as ex:
        for l, lw in enumerate(ex.map(make, range(len(wl.layers)))):
            kt, kv = wl.k_schedule[l]
            m = binding.FMoE(d_model=wl.d, n_experts=wl.E, d_ffn=wl.F, n_shared=wl.n_shared,
                             d_ffn_shared=wl.F_shared, k_text=kt, k_visual=kv, dtype=wl.dtype)
            m.set_weights(dev(lw.router_w, td), dev(lw.router_bias), dev(lw.w_gate, td), dev(lw.w_up, td),
                          dev(lw.w_down, td), dev(lw.ws_gate, td), dev(lw.ws_up, td), dev(lw.ws_down, td),
                          release_packed=True)
            layers.append(m)
    sched = {wl.prune_after_layer: binding.prune_params(retention=wl.retention, window=wl.window, prune_mode=2)}
    out, kept, new_cu = _gpu_stack(wl, layers, sched)
    nv, nt = _lens(wl)
    n = binding.kept_count(nv, nt, wl.retention)
    assert out.shape[0] == n == kept.shape[0]
    kept_v = binding.kept_visual_lens(nv, wl.retention)
    assert list(np.diff(host(new_cu))) == [v + t for v, t in zip(kept_v, nt)]
    k = host(kept)
    assert (np.diff(k) > 0).all() and k[0] >= 0 and k[-1] < wl.T
    assert wl.is_visual[k].sum() == sum(kept_v) and (wl.is_visual[k] == 0).sum() == sum(nt)
    assert torch.isfinite(out.float()).all()
    # layers 0-2 as chained calls: same bits up to the stage, same kept set
    x, vis, cu = inputs(wl)
    for l in range(3):
        layers[l].set_topk(*wl.k_schedule[l])
        o, kp, nc, _ = layers[l].layer_forward(x, vis, cu, sched.get(l), add_residual=True)
        x = o
    assert torch.equal(kp[:n], kept) and torch.equal(nc, new_cu)
    for m in layers:
        m.close()
    torch.cuda.empty_cache()


# ---------------------------------------------------------------- diagnostics (the paper's analysis statistics)
DIAG_TOL = 2e-5   # fp32 arithmetic inside a row against the fp64 oracle; the statistics are O(1)


@pytest.mark.parametrize("seed,kw", [SMALL[1], SMALL[3], SMALL[8]])
def test_adjacent_similarity(seed, kw):
    wl = _wl(seed, kw)
    o_probs, _, _ = oracle.route(wl.x, wl.is_visual, wl.weights.router_w, wl.weights.router_bias,
                                 wl.k_text, wl.k_visual)
    o_pair, o_mean, o_count = oracle.adjacent_similarity(o_probs, wl.is_visual, wl.cu_seqlens)
    m = make_layer(wl)
    pair, mean, count = m.adjacent_similarity(dev(o_probs), dev(wl.is_visual), dev(wl.cu_seqlens))
    pair, mean, count = host(pair), host(mean), host(count)
    assert np.array_equal(count, o_count)
    assert np.array_equal(pair < -1.5, o_pair < -1.5)            # the same pairs exist
    assert np.abs(pair - o_pair).max() <= DIAG_TOL
    assert np.abs(mean - o_mean).max() <= DIAG_TOL


@pytest.mark.parametrize("seed,kw", [SMALL[1], SMALL[3], SMALL[5], SMALL[8]])
def test_magnitude_stability_and_output_angle(seed, kw):
    wl = _wl(seed, kw)
    o = _oracle(wl)
    n, M = len(o["kept_idx"]), int(o["expert_offsets"][-1])
    m = make_layer(wl)
    x, vis, cu = inputs(wl)
    # App. C.1 on the routed experts' outputs of the layer (the oracle's rows, rounded to the dtype)
    y_rows = dev(np.asarray(o["y"], np.float32), torch_dtype(wl))
    row_vis = wl.is_visual[o["kept_idx"][o["perm_src"]]]
    o_norm, o_stats = oracle.magnitude_stability(host(y_rows), row_vis)
    m_dev = dev(np.array([M], np.int32))
    norms, stats = m.magnitude_stability(y_rows, M, dev(o["perm_src"]), dev(o["kept_idx"]), vis, M_dev=m_dev)
    assert np.abs(host(norms) - o_norm).max() <= DIAG_TOL * max(1.0, o_norm.max())
    assert np.abs(host(stats) - o_stats).max() <= DIAG_TOL * max(1.0, np.abs(o_stats).max())
    # App. C: angle between the layer output with all K experts and with the reduced k_visual
    full = _oracle(wl, k_visual=wl.k_text)
    assert np.array_equal(full["kept_idx"], o["kept_idx"])       # pruning does not look at k
    a, b = dev(full["out"], torch_dtype(wl)), dev(o["out"], torch_dtype(wl))
    cos = host(m.row_cosine(a, b))
    assert np.abs(cos - oracle.row_cosine(host(a), host(b))).max() <= DIAG_TOL
    # and the closed form from the K gates
    K = wl.k_text
    o_probs, _, o_gate = oracle.route(wl.x, wl.is_visual, wl.weights.router_w, wl.weights.router_bias, K, K)
    pred = host(m.gate_cosine(dev(o_gate), wl.k_visual))
    assert np.abs(pred - oracle.gate_cosine(o_gate, wl.k_visual)).max() <= DIAG_TOL
    if wl.k_visual > 0:
        assert (pred >= np.sqrt(wl.k_visual / K) - 1e-5).all()


# ---------------------------------------------------------------- ablation switches (Sec. 4)
@pytest.mark.parametrize("strategy", [binding.TOPK, binding.RANDOMK, binding.MINK])
@pytest.mark.parametrize("seed,kw", [SMALL[1], SMALL[3], SMALL[4], SMALL[5], SMALL[8]])
def test_route_selection_strategies(seed, kw, strategy):
    wl = _wl(seed, kw)
    k_base = wl.k_text
    m = make_layer(wl)
    m.set_selection(strategy, k_base, seed=1234 + seed)
    x, vis, cu = inputs(wl)
    probs, idx, gate = m.route(x, vis)
    o_probs, o_idx, o_gate = oracle.route_select(wl.x, wl.is_visual, wl.weights.router_w, wl.weights.router_bias,
                                                 wl.k_text, wl.k_visual, strategy, k_base, seed=1234 + seed)
    assert np.array_equal(host(probs), o_probs)
    assert np.array_equal(host(idx), o_idx)
    assert np.abs(host(gate) - o_gate).max() <= 1e-6
    if strategy != binding.TOPK and wl.k_visual > 0:
        _, idx_top, _ = oracle.route(wl.x, wl.is_visual, wl.weights.router_w, wl.weights.router_bias,
                                     wl.k_text, wl.k_visual)
        assert not np.array_equal(o_idx, idx_top)              # the switch does something


def test_selection_k_base_above_kmax_and_text_reduction():
    # reduce BOTH modalities (the "All" row of the modality ablation) from a candidate list longer
    # than either k: k_base = 8 > Kmax = 4
    wl = W.small_random(118, T_v=[70], T_t=[30], d=64, E=32, F=32, k_text=4, k_visual=2, retention=0.5,
                        window=3, bias_std=1.0)
    m = make_layer(wl)
    x, vis, cu = inputs(wl)
    for strategy in (binding.RANDOMK, binding.MINK):
        m.set_selection(strategy, 8, seed=9)
        _, idx, gate = m.route(x, vis)
        _, o_idx, o_gate = oracle.route_select(wl.x, wl.is_visual, wl.weights.router_w, wl.weights.router_bias,
                                               4, 2, strategy, 8, seed=9)
        assert np.array_equal(host(idx), o_idx) and np.abs(host(gate) - o_gate).max() <= 1e-6
    with pytest.raises(RuntimeError):
        m.set_selection(3, 8)
    with pytest.raises(RuntimeError):
        m.set_selection(1, 33)


@pytest.mark.parametrize("seed,kw", [SMALL[3], SMALL[8]])
def test_layer_forward_ablation_switches(seed, kw):
    # MinK selection + plain-mean merging through the whole layer
    wl = _wl(seed, kw)
    m = make_layer(wl)
    m.set_selection(binding.MINK, wl.k_text)
    x, vis, cu = inputs(wl)
    o = _oracle(wl, add_residual=True, gamma=0.3, merge_mean=True, strategy=oracle.MINK, k_base=wl.k_text)
    pp = binding.prune_params(retention=wl.retention, window=wl.window, gamma=0.3, merge_mode=1)
    out, kept, new_cu, _ = m.layer_forward(x, vis, cu, pp, add_residual=True)
    new_cu = host(new_cu)
    n = int(new_cu[-1])
    assert np.array_equal(new_cu, o["new_cu_seqlens"]) and np.array_equal(host(kept)[:n], o["kept_idx"])
    assert_residual_outputs_close(host(out)[:n], o["out_f64"], _x_rows(wl, o), wl.dtype, "MinK + mean merge")
    out2, _, _, _ = m.layer_forward(x, vis, cu, pp)
    o2 = _oracle(wl, gamma=0.3, merge_mean=True, strategy=oracle.MINK, k_base=wl.k_text)
    assert_outputs_close(host(out2)[:n], o2["out_f64"], wl.dtype, "MinK + mean merge, expert term")
    # mean mode alone, through fmoe_prune
    o_probs, _, _ = oracle.route(wl.x, wl.is_visual, wl.weights.router_w, wl.weights.router_bias,
                                 wl.k_text, wl.k_visual)
    o_kept, o_cu, _, o_mrg, o_xm = oracle.prune(o_probs, wl.is_visual, wl.cu_seqlens, wl.retention, wl.window,
                                                gamma=0.3, x=wl.x, is_bf16=wl.dtype == W.BF16, merge_mean=True)
    kept, new_cu, _, mrg, x_m = m.prune(pp, dev(o_probs), vis, cu, x=x)
    n = int(host(new_cu)[-1])
    assert np.array_equal(host(kept)[:n], o_kept) and np.array_equal(host(mrg)[:n], o_mrg)
    _check_merged_rows(host(x_m)[:n], o_xm, o_mrg, wl.dtype)


# ---------------------------------------------------------------- randomized sweep
def _random_case(seed):
    rng = np.random.default_rng(7000 + seed)
    E = int(rng.choice([3, 5, 8, 16, 33, 64, 100, 128, 256]))
    k_text = int(rng.integers(1, min(E, 16) + 1))
    k_visual = int(rng.integers(0, k_text + 1))
    n_seq = int(rng.integers(1, 6))
    T_v = [int(v) for v in rng.choice([0, 1, 2, 7, 30, 64, 101, 257], size=n_seq)]
    T_t = [int(v) for v in rng.choice([0, 1, 3, 9, 20], size=n_seq)]
    if sum(T_v) + sum(T_t) == 0:
        T_t[0] = 4
    n_shared = int(rng.choice([0, 0, 1, 2]))
    kw = dict(T_v=T_v, T_t=T_t, d=int(rng.choice([16, 40, 64, 136, 256, 320])), E=E,
              F=int(rng.choice([8, 24, 64, 104])), k_text=k_text, k_visual=k_visual,
              retention=float(rng.choice([0.1, 0.3, 0.5, 0.77, 0.95, 1.0])), window=int(rng.integers(1, 9)),
              dtype=str(rng.choice([W.F32, W.BF16])), n_shared=n_shared,
              F_shared=int(rng.choice([8, 40])) if n_shared else None, bias_std=float(rng.choice([0.0, 1.0, 2.5])),
              n_components=int(rng.choice([0, 4, 16])), interleave=bool(rng.integers(0, 2)))
    if k_visual == 0 and n_shared == 0:
        kw["k_visual"] = 1                                  # K_v = 0 needs shared experts (Sec. 3.1)
    extra = dict(gamma=float(rng.choice([0.0, 0.0, 0.1, 0.6])), alpha=float(rng.choice([1.0, 0.6, 0.0])),
                 use_attn=bool(rng.integers(0, 2)), sim_mode=int(rng.integers(0, 2)))
    return kw, extra


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("seed", range(32))
def test_randomized_layer_sweep(seed, shape):
    kw, extra = _random_case(seed)
    wl = W.small_random(7000 + seed, **kw)
    _skip_fp32_duplicate(wl, shape)
    rng = np.random.default_rng(9000 + seed)
    attn = (rng.random(wl.T).astype(np.float32) ** 2) if extra["use_attn"] else None
    alpha = extra["alpha"] if attn is not None else 1.0
    over = dict(add_residual=True, gamma=extra["gamma"], alpha=alpha, attn=attn, sim_mode=extra["sim_mode"])
    o = _oracle(wl, **over)
    m = make_layer(wl, ffn_shape=shape)
    x, vis, cu = inputs(wl)
    pp = binding.prune_params(retention=wl.retention, window=wl.window, alpha=alpha, gamma=extra["gamma"],
                              sim_mode=extra["sim_mode"])
    out, kept, new_cu, vis_out = m.layer_forward(x, vis, cu, pp, attn=dev(attn), add_residual=True, want_mask=True)
    torch.cuda.synchronize()
    new_cu = host(new_cu)
    n = int(new_cu[-1])
    assert np.array_equal(new_cu, o["new_cu_seqlens"]), (kw, extra)
    assert np.array_equal(host(kept)[:n], o["kept_idx"]), (kw, extra)
    assert np.array_equal(host(vis_out)[:n], wl.is_visual[o["kept_idx"]])
    if n:
        assert_residual_outputs_close(host(out)[:n], o["out_f64"], _x_rows(wl, o), wl.dtype, str((kw, extra)))
        out2, _, _, _ = m.layer_forward(x, vis, cu, pp, attn=dev(attn))
        over["add_residual"] = False
        assert_outputs_close(host(out2)[:n], _oracle(wl, **over)["out_f64"], wl.dtype, str((kw, extra)))


@pytest.mark.parametrize("T_v,T_t,window", [
    ([4096], [0], 4),        # 4096 tokens, 1024 windows: the largest batch of the single-workgroup dispatch kernel
    ([4095], [1], 4),        # 1024 windows, the last one short
    ([4092], [4], 3),        # 1364 windows in one sequence: the general kernels, although T = 4096
    ([4096], [1], 4),        # one token more than the single-workgroup kernel takes
    ([1024, 1024, 1024, 1020], [1, 1, 1, 1], 1),   # W = 1: every visual token is a window of its own
])
def test_layer_forward_at_the_small_batch_limits(T_v, T_t, window):
    """Both sides of the size limits that decide between the single-workgroup prune/dispatch kernel and the
    general kernel chain give the oracle's kept set, permutation and outputs."""
    wl = W.small_random(4242, T_v=T_v, T_t=T_t, d=64, E=16, F=32, k_text=3, k_visual=2, retention=0.6,
                        window=window, dtype=W.F32, bias_std=1.0, n_components=24)
    o = _oracle(wl)
    m = make_layer(wl)
    x, vis, cu = inputs(wl)
    out, kept, new_cu, _ = m.layer_forward(x, vis, cu, binding.prune_params(retention=wl.retention, window=window))
    torch.cuda.synchronize()
    new_cu = host(new_cu)
    n = int(new_cu[-1])
    assert np.array_equal(new_cu, o["new_cu_seqlens"])
    assert np.array_equal(host(kept)[:n], o["kept_idx"])
    assert max_rel_err(host(out)[:n], o["out_f64"]) <= TOL[wl.dtype]


def test_layer_forward_general_chain_over_many_sequences():
    """More than 4096 tokens in 1500 sequences of a few tokens each (empty ones among them): the fused layer
    takes the general kernel chain, the router's launch carries one ordinal block per sequence, and every
    window-indexed array is cut into 1500 pieces; kept set, bounds, mask and outputs against the oracle."""
    rng = np.random.default_rng(77)
    n_seq = 1500
    T_v = [int(v) for v in rng.choice([0, 1, 2, 3, 4, 6, 9], size=n_seq)]
    T_t = [int(v) for v in rng.choice([0, 0, 1, 2], size=n_seq)]
    wl = W.small_random(515, T_v=T_v, T_t=T_t, d=64, E=16, F=32, k_text=3, k_visual=2, retention=0.55, window=3,
                        dtype=W.F32, n_components=6, bias_std=1.0, interleave=True)
    assert wl.T > 4096 and wl.B == n_seq
    o = _oracle(wl, add_residual=True)
    m = make_layer(wl)
    x, vis, cu = inputs(wl)
    out, kept, new_cu, vis_out = m.layer_forward(x, vis, cu, binding.prune_params(retention=wl.retention, window=3),
                                                 add_residual=True, want_mask=True)
    torch.cuda.synchronize()
    new_cu = host(new_cu)
    n = int(new_cu[-1])
    assert np.array_equal(new_cu, o["new_cu_seqlens"])
    assert np.array_equal(host(kept)[:n], o["kept_idx"])
    assert np.array_equal(host(vis_out)[:n], wl.is_visual[o["kept_idx"]])
    assert_residual_outputs_close(host(out)[:n], o["out_f64"], _x_rows(wl, o), wl.dtype, "1500 sequences")


@pytest.mark.parametrize("with_attention", [False, True])
def test_layer_forward_merge_after_the_layer_over_several_compaction_blocks(with_attention):
    """Merging on the layer output at a size where the experts run in several row tiles per expert, the
    compaction in several blocks and the merge order (redundancy) differs from the drop order (attention
    first): decisions bit for bit, ordinary and merged rows against the oracle."""
    wl = W.small_random(616, T_v=[2200, 3, 1500, 900], T_t=[30, 2, 0, 50], d=128, E=32, F=64, k_text=4, k_visual=2,
                        retention=0.5, window=3, dtype=W.BF16, n_shared=1, F_shared=32, bias_std=1.0,
                        n_components=24)
    assert wl.T > 4096
    attn = None
    if with_attention:
        attn = np.random.default_rng(6).random(wl.T).astype(np.float32)
    gamma = 0.1
    o = _oracle(wl, add_residual=True, gamma=gamma, alpha=0.6 if with_attention else 1.0, attn=attn,
                after_layer=True)
    assert o["is_merged"].sum() > 50
    m = make_layer(wl)
    x, vis, cu = inputs(wl)
    pp = binding.prune_params(retention=wl.retention, window=wl.window, gamma=gamma, prune_mode=2,
                              alpha=0.6 if with_attention else 1.0)
    out, kept, new_cu, vis_out = m.layer_forward(x, vis, cu, pp, add_residual=True, want_mask=True,
                                                 attn=None if attn is None else dev(attn))
    torch.cuda.synchronize()
    new_cu = host(new_cu)
    n = int(new_cu[-1])
    assert np.array_equal(new_cu, o["new_cu_seqlens"])
    assert np.array_equal(host(kept)[:n], o["kept_idx"])
    assert np.array_equal(host(vis_out)[:n], wl.is_visual[o["kept_idx"]])
    _check_after_layer_rows(host(out)[:n], o, wl.x, wl.dtype, f"attention {with_attention}")


@pytest.mark.parametrize("shape", SHAPES)
def test_layer_forward_general_chain_at_the_widest_routing(shape):
    """The largest expert count and top-k the library takes (256 experts, 16 per text token), shared experts,
    bf16, several ragged sequences and more tokens than the single-workgroup kernel handles."""
    wl = W.small_random(5151, T_v=[2500, 1, 1800, 700], T_t=[40, 3, 0, 77], d=96, E=256, F=40, k_text=16, k_visual=7,
                        retention=0.4, window=5, dtype=W.BF16, n_shared=2, F_shared=24, bias_std=1.0, n_components=40)
    assert wl.T > 4096
    o = _oracle(wl, add_residual=True)
    m = make_layer(wl, ffn_shape=shape)
    x, vis, cu = inputs(wl)
    out, kept, new_cu, _ = m.layer_forward(x, vis, cu, binding.prune_params(retention=wl.retention, window=wl.window),
                                           add_residual=True)
    torch.cuda.synchronize()
    new_cu = host(new_cu)
    n = int(new_cu[-1])
    assert np.array_equal(new_cu, o["new_cu_seqlens"])
    assert np.array_equal(host(kept)[:n], o["kept_idx"])
    assert_residual_outputs_close(host(out)[:n], o["out_f64"], _x_rows(wl, o), wl.dtype, "widest routing")
    out2, _, _, _ = m.layer_forward(x, vis, cu, binding.prune_params(retention=wl.retention, window=wl.window))
    assert_outputs_close(host(out2)[:n], _oracle(wl)["out_f64"], wl.dtype, "widest routing, expert term")


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("d,F", [(448, 576), (576, 640), (640, 704), (832, 960), (960, 448), (72, 1032), (1032, 72)])
def test_expert_ffn_k_loop_lengths(d, F, shape):
    # bf16 expert GEMMs at reduction lengths of 2..17 k-tiles of 64: every combination of steady-loop
    # iterations and left-over steps of both kernel shapes' k loops (the weight-stream shape: rounds of 4
    # tiles + 3..6 left over; the dense shape: rounds of 8 half-tiles + 0, 2, 4 or 6 left over), reduction
    # lengths that are not a multiple of 64, ragged row counts
    wl = W.small_random(8000 + d, T_v=[150, 40], T_t=[30, 7], d=d, E=12, F=F, k_text=4, k_visual=2,
                        retention=0.5, window=3, dtype=W.BF16, n_shared=1, F_shared=F - 64, bias_std=1.5)
    o = _oracle(wl, add_residual=True)
    n = len(o["kept_idx"])
    m = make_layer(wl, ffn_shape=shape)
    x, vis, cu = inputs(wl)
    out, kept, new_cu, _ = m.layer_forward(x, vis, cu, binding.prune_params(retention=0.5, window=3),
                                           add_residual=True)
    assert np.array_equal(host(kept)[:n], o["kept_idx"])
    assert_residual_outputs_close(host(out)[:n], o["out_f64"], _x_rows(wl, o), wl.dtype, "k loop")
    out2, _, _, _ = m.layer_forward(x, vis, cu, binding.prune_params(retention=0.5, window=3))
    assert_outputs_close(host(out2)[:n], _oracle(wl)["out_f64"], wl.dtype, "k loop, expert term")
    y, ysh = m.expert_ffn(x, dev(o["kept_idx"]), n, dev(o["expert_offsets"]), dev(o["perm_src"]))
    M = int(o["expert_offsets"][-1])
    assert max_rel_err(host(y)[:M], o["y"]) <= TOL[W.BF16]
    assert max_rel_err(host(ysh).astype(np.float64).sum(0)[:n], o["y_shared"]) <= TOL[W.BF16]
