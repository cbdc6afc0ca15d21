"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares, and
its host-side validation returns error codes without touching a GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2511_17885_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2511_17885_amd import build
        build.build()
    return binding.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "fmoe.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(fmoe_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert b"gfx950" in lib.fmoe_version()


def _cfg(**kw):
    base = dict(d_model=64, n_experts=8, d_ffn=32, n_shared=0, d_ffn_shared=0, k_text=2, k_visual=1,
                renormalize=1, dtype=0)
    base.update(kw)
    return binding.FmoeConfig(*[base[f[0]] for f in binding.FmoeConfig._fields_])


def _create(lib, cfg):
    ctx = C.c_void_p()
    rc = lib.fmoe_create(C.byref(ctx), C.byref(cfg), 0)
    return rc, ctx


def test_create_validates_config(lib):
    rc, ctx = _create(lib, _cfg())
    assert rc == 0 and ctx.value
    assert lib.fmoe_workspace_bytes(ctx, 64, 1) > 0
    assert lib.fmoe_workspace_bytes(ctx, 4096, 8) > lib.fmoe_workspace_bytes(ctx, 64, 1)
    lib.fmoe_destroy(ctx)
    for bad, code in [(dict(k_visual=9), -1), (dict(k_text=-1), -1), (dict(d_model=0), -1),
                      (dict(dtype=7), -1), (dict(n_experts=300), -5), (dict(d_model=100), -5),
                      (dict(n_shared=1, d_ffn_shared=0), -1), (dict(n_experts=32, k_text=17), -5)]:
        rc, ctx = _create(lib, _cfg(**bad))
        assert rc == code, (bad, rc, lib.fmoe_last_error())
        assert not ctx.value
        assert lib.fmoe_last_error() != b""
    assert lib.fmoe_create(None, C.byref(_cfg()), 0) == -2


def test_set_topk_and_null_argument_paths(lib):
    rc, ctx = _create(lib, _cfg())
    assert rc == 0
    assert lib.fmoe_set_topk(ctx, 4, 2) == 0
    assert lib.fmoe_set_topk(ctx, 9, 2) == -1
    # weights not set -> route refuses before any GPU work
    assert lib.fmoe_route(ctx, None, None, 4, None, None, None, None) == -1
    assert b"fmoe_set_weights" in lib.fmoe_last_error()
    # set_weights: NULL required pointer, stray shared weights
    assert lib.fmoe_set_weights(ctx, None, None, None, None, None, None, None, None, None) == -2
    # prune argument validation (host side only)
    pp = binding.prune_params(retention=0.5, window=3)
    assert lib.fmoe_prune(ctx, None, None, None, None, 1, 4, None, None, None, None, None, None, None, None, 0, None) == -2
    bad = binding.prune_params(retention=1.5, window=3)
    assert lib.fmoe_prune(ctx, C.byref(bad), None, None, None, 1, 4, None, None, None, None, None, None, None, None, 0, None) == -1
    bad = binding.prune_params(retention=0.5, window=0)
    assert lib.fmoe_prune(ctx, C.byref(bad), None, None, None, 1, 4, None, None, None, None, None, None, None, None, 0, None) == -1
    bad = binding.prune_params(retention=0.5, window=3, gamma=1.0)        # merge rate outside [0,1)
    assert lib.fmoe_prune(ctx, C.byref(bad), None, None, None, 1, 4, None, None, None, None, None, None, None, None, 0, None) == -1
    assert lib.fmoe_prune(ctx, C.byref(pp), None, None, None, 1, 4, None, None, None, None, None, None, None, None, 0, None) == -2
    # permute: missing workspace
    dummy = C.c_void_p(0x1000)
    assert lib.fmoe_permute(ctx, dummy, None, 8, None, dummy, dummy, dummy, None, 0, None) == -4
    assert lib.fmoe_permute(ctx, dummy, None, -1, None, dummy, dummy, dummy, None, 0, None) == -1
    assert lib.fmoe_permute(ctx, dummy, None, 8, None, dummy, dummy, dummy, C.c_void_p(0x10000), 16, None) == -4
    lib.fmoe_destroy(ctx)
    assert lib.fmoe_route(None, None, None, 4, None, None, None, None) == -2


def test_binding_fails_loudly_without_library(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libfmoe.so")
    with pytest.raises(RuntimeError):
        binding.load()


def test_stage_bookkeeping_matches_the_oracles_counts():
    """Host logic of the stack driver: the per-stage token counts (Sec. 3.2.3 budget, App. D equal
    per-stage ratio) must be the counts the pruning itself produces, stage after stage, with or
    without window merging."""
    import numpy as np
    import oracle
    rng = np.random.default_rng(11)
    sched = binding.stage_schedule(0.25, [5, 8, 12], window=5, gamma=0.1)
    assert sorted(sched) == [5, 8, 12] and sched[5].window == 5
    beta = sched[5].retention
    assert abs(beta ** 3 - 0.25) < 1e-6
    nv, nt = [57, 5, 0, 301], [3, 0, 4, 10]
    vis = np.concatenate([np.r_[np.ones(v, np.uint8), np.zeros(t, np.uint8)] for v, t in zip(nv, nt)])
    cu = np.concatenate([[0], np.cumsum([v + t for v, t in zip(nv, nt)])]).astype(np.int32)
    lens = list(nv)
    for _ in range(3):
        T = int(cu[-1])
        probs = rng.random((T, 12)).astype(np.float32)
        probs /= probs.sum(1, keepdims=True)
        x = rng.standard_normal((T, 8)).astype(np.float32)
        kept, new_cu, _, _, _ = oracle.prune(probs, vis, cu, beta, 5, gamma=0.1, x=x)
        lens = binding.kept_visual_lens(lens, beta)
        assert list(np.diff(new_cu)) == [v + t for v, t in zip(lens, nt)]
        assert int(new_cu[-1]) == binding.kept_count(lens, nt, 1.0)
        vis, cu = vis[kept], new_cu
    assert lens[2] == 0 and lens[1] >= 1                      # empty stays empty; N_v > 0 keeps >= 1


def test_switches_and_diagnostics_validate_their_arguments(lib):
    """Host-side checks of the ablation switches and the diagnostics entry points: bad values are
    refused with an error code before anything is enqueued (no GPU needed)."""
    cfg = binding.FmoeConfig(64, 8, 32, 0, 0, 2, 1, 1, binding.FMOE_F32)
    ctx = C.c_void_p()
    assert lib.fmoe_create(C.byref(ctx), C.byref(cfg), 0) == 0
    # selection strategy: 0..2, k_base within [0, min(E, 16)]
    assert lib.fmoe_set_selection(ctx, binding.MINK, 4, 7) == 0
    assert lib.fmoe_set_selection(ctx, 3, 4, 0) == -1
    assert lib.fmoe_set_selection(ctx, binding.RANDOMK, 9, 0) == -1          # E = 8
    assert lib.fmoe_set_selection(ctx, binding.RANDOMK, -1, 0) == -1
    assert lib.fmoe_set_selection(None, 0, 0, 0) == -2
    assert lib.fmoe_set_selection(ctx, binding.TOPK, 0, 0) == 0
    # expert GEMM shape: 0 by size, 1 weight-stream, 2 dense
    assert lib.fmoe_set_ffn_shape(ctx, 2) == 0 and lib.fmoe_set_ffn_shape(ctx, 0) == 0
    assert lib.fmoe_set_ffn_shape(ctx, 3) == -1 and lib.fmoe_set_ffn_shape(ctx, -1) == -1
    assert lib.fmoe_set_ffn_shape(None, 1) == -2
    # merge method: 0 (MLERP) or 1 (mean)
    bad = binding.prune_params(retention=0.5, window=3, gamma=0.1, merge_mode=2)
    assert lib.fmoe_prune(ctx, C.byref(bad), None, None, None, 1, 4, None, None, None, None, None, None, None,
                          None, 0, None) == -1
    assert b"merge_mode" in lib.fmoe_last_error()
    # diagnostics
    dummy = C.c_void_p(0x1000)
    assert lib.fmoe_gate_cosine(ctx, dummy, 4, 8, 9, dummy, None) == -1       # m > K
    assert lib.fmoe_gate_cosine(ctx, dummy, 4, 0, 0, dummy, None) == -1       # K < 1
    assert lib.fmoe_gate_cosine(ctx, None, 4, 8, 2, dummy, None) == -2
    assert lib.fmoe_gate_cosine(ctx, None, 0, 8, 2, None, None) == 0          # nothing to do
    assert lib.fmoe_adjacent_similarity(ctx, dummy, dummy, dummy, -1, 4, dummy, dummy, dummy, None) == -1
    assert lib.fmoe_adjacent_similarity(ctx, dummy, dummy, dummy, 0, 4, dummy, dummy, dummy, None) == -1
    assert lib.fmoe_adjacent_similarity(ctx, dummy, dummy, None, 1, 4, dummy, dummy, dummy, None) == -2
    assert lib.fmoe_magnitude_stability(ctx, dummy, -1, None, dummy, None, dummy, dummy, dummy, None) == -1
    assert lib.fmoe_magnitude_stability(ctx, dummy, 4, None, None, None, dummy, dummy, dummy, None) == -2
    assert lib.fmoe_row_cosine(ctx, dummy, None, 4, None, dummy, None) == -2
    assert lib.fmoe_row_cosine(ctx, None, None, 0, None, None, None) == 0
    lib.fmoe_destroy(ctx)


def test_flops_ratios_layer_loop_matches_the_closed_forms_and_the_printed_savings(lib):
    """fmoe_flops_ratios prices the model layer by layer; the oracle evaluates App. E's stage formulas."""
    import numpy as np
    import oracle
    from test_oracle_pins import FLOPS_MODELS, flops_table_rows
    for model, keep, beta, lv, kv, saving in flops_table_rows():
        m = dict(FLOPS_MODELS[model])
        shared, stages = m.pop("shared"), m.pop("stage_layers")
        n_layers = m["n_dense"] + sum(stages)
        prune_layers = (np.cumsum(stages[:-1]) + m["n_dense"] - 1).tolist()
        assert prune_layers == ([5, 8, 12] if model == "internvl35" else [2, 5, 8])
        l_v = n_layers if lv is None else lv - 1 + m["n_dense"]
        K_v = m["K"] if kv is None else kv + shared
        got = binding.flops_ratios(n_layers=n_layers, prune_layers=prune_layers, beta=beta, l_v=l_v, K_v=K_v, **m)
        assert round(100.0 * (1.0 - got[2]), 2) == saving
    rng = np.random.default_rng(11)
    for _ in range(50):
        n_dense = int(rng.integers(0, 3))
        stages = tuple(int(v) for v in rng.integers(1, 9, size=int(rng.integers(1, 6))))
        n_layers = n_dense + sum(stages)
        kw = dict(H=float(rng.integers(64, 8192)), E=float(rng.integers(4, 256)), S_m=float(rng.integers(64, 4096)),
                  K=float(rng.integers(2, 12)), L_v=float(rng.integers(16, 20000)), n_dense=n_dense,
                  S=float(rng.integers(256, 20000)))
        K_v = float(rng.integers(0, int(kw["K"]) + 1))
        l_v = int(rng.integers(0, n_layers + 1))
        beta = float(rng.uniform(0.3, 1.0))
        prune_layers = (np.cumsum(stages[:-1]) + n_dense - 1).tolist()
        got = binding.flops_ratios(n_layers=n_layers, prune_layers=prune_layers, beta=beta, l_v=l_v, K_v=K_v, **kw)
        want = oracle.flops_ratios(stages, K_v=K_v, l_v=l_v, beta=beta, **kw)
        assert np.allclose(got, want, rtol=1e-12, atol=0.0), (stages, n_dense, l_v, got, want)


def test_flops_ratios_validate_their_arguments(lib):
    ok = dict(n_layers=12, H=512, S_m=256, E=16, K=4, L_v=100, prune_layers=(2, 5), beta=0.8, l_v=3, K_v=2)
    assert all(0.0 < v <= 1.0 for v in binding.flops_ratios(**ok))
    for bad in (dict(n_layers=0), dict(H=0), dict(beta=0.0), dict(beta=1.5), dict(l_v=13), dict(prune_layers=(5, 2)),
                dict(prune_layers=(12,)), dict(n_dense=1, S=0.0), dict(K_v=-1), dict(L_v=0)):
        with pytest.raises(binding.FmoeError) as e:
            binding.flops_ratios(**{**ok, **bad})
        assert e.value.code == -1, bad   # FMOE_ERR_INVALID_ARG
    m = binding.FmoeFlopsModel()
    assert lib.fmoe_flops_ratios(None, (C.c_double * 3)()) == lib.fmoe_flops_ratios(C.byref(m), None) != 0


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU's throughput; asked for more it says so and exits before touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_budget_rule_and_stage_ratio_entry_points(lib):
    """fmoe_kept_counts (Sec. 3.2.3) against the rule written out here and against the counts the
    oracle's pruning produces; fmoe_stage_retention (App. D) against beta^stages = r."""
    import numpy as np
    import oracle
    rng = np.random.default_rng(3)
    for r in (0.25, 0.5, 0.63, 0.75, 0.9, 1.0, 1e-3):
        lens = [int(v) for v in rng.integers(0, 7000, size=9)] + [0, 1, 2, 3]
        got = binding.kept_visual_lens(lens, r)
        r32 = float(np.float32(r))
        want = [min(max(int(np.floor(r32 * n + 0.5)), min(1, n)), n) for n in lens]
        assert got == want, r
    # the count the pruning itself keeps (oracle), on a small ragged batch
    nv, nt = [41, 0, 7, 130], [2, 5, 0, 9]
    vis = np.concatenate([np.r_[np.ones(v, np.uint8), np.zeros(t, np.uint8)] for v, t in zip(nv, nt)])
    cu = np.concatenate([[0], np.cumsum([v + t for v, t in zip(nv, nt)])]).astype(np.int32)
    probs = rng.random((int(cu[-1]), 10)).astype(np.float32)
    _, new_cu, _ = oracle.prune(probs, vis, cu, 0.37, 4)
    assert list(np.diff(new_cu)) == [v + t for v, t in zip(binding.kept_visual_lens(nv, 0.37), nt)]
    for r, stages in ((0.5, 3), (0.25, 3), (0.75, 1), (1.0, 4), (0.1, 7)):
        beta = binding.stage_retention(r, stages)
        assert abs(beta ** stages - r) < 1e-6 and 0 < beta <= 1
    buf = (C.c_int32 * 2)(5, 6)
    assert lib.fmoe_kept_counts(buf, 2, 1.5, buf) == -1
    assert lib.fmoe_kept_counts(buf, 2, 0.0, buf) == -1
    assert lib.fmoe_kept_counts(buf, -1, 0.5, buf) == -1
    assert lib.fmoe_kept_counts(None, 2, 0.5, buf) == -2
    assert lib.fmoe_kept_counts(None, 0, 0.5, None) == 0
    neg = (C.c_int32 * 1)(-3)
    assert lib.fmoe_kept_counts(neg, 1, 0.5, neg) == -1
    beta = C.c_float()
    assert lib.fmoe_stage_retention(0.5, 0, C.byref(beta)) == -1
    assert lib.fmoe_stage_retention(0.0, 2, C.byref(beta)) == -1
    assert lib.fmoe_stage_retention(0.5, 2, None) == -2


def test_stack_plan_and_stack_argument_checks(lib):
    """fmoe_stack_plan: K everywhere below l_v, (K, K_v) from l_v on (Sec. 3.1); stages at the listed
    layers with the per-stage ratio of App. D.  fmoe_stack_forward / _workspace_bytes refuse
    inconsistent arguments before anything is enqueued."""
    n = 12
    plan = (binding.FmoeLayerPlan * n)()
    stage = binding.prune_params(retention=0.5, window=3, gamma=0.05)
    layers = (C.c_int32 * 3)(2, 5, 8)
    assert lib.fmoe_stack_plan(n, 6, 3, 2, layers, 3, C.byref(stage), plan) == 0
    beta = binding.stage_retention(0.5, 3)
    for l in range(n):
        assert (plan[l].k_text, plan[l].k_visual) == ((6, 6) if l < 2 else (6, 3))
        if l in (2, 5, 8):
            assert plan[l].prune.retention == beta and plan[l].prune.window == 3
            assert abs(plan[l].prune.gamma - 0.05) < 1e-7 and plan[l].prune.prune_mode == 1
        else:
            assert plan[l].prune.prune_mode == 0 and plan[l].prune.retention == 1.0
    assert lib.fmoe_stack_plan(n, 6, 3, n, None, 0, None, plan) == 0          # never reduced, never pruned
    assert all(plan[l].k_visual == 6 and plan[l].prune.prune_mode == 0 for l in range(n))
    assert lib.fmoe_stack_plan(n, 6, 3, 13, None, 0, None, plan) == -1
    assert lib.fmoe_stack_plan(n, 6, 3, 2, (C.c_int32 * 2)(5, 2), 2, C.byref(stage), plan) == -1
    assert lib.fmoe_stack_plan(n, 6, 3, 2, (C.c_int32 * 1)(12), 1, C.byref(stage), plan) == -1
    assert lib.fmoe_stack_plan(n, 6, 3, 2, layers, 3, None, plan) == -2
    assert lib.fmoe_stack_plan(0, 6, 3, 0, None, 0, None, plan) == -1
    assert lib.fmoe_stack_plan(n, 6, 3, 2, None, 0, None, None) == -2

    cfg = binding.FmoeConfig(64, 8, 32, 0, 0, 2, 1, 1, binding.FMOE_F32)
    ctxs = (C.c_void_p * 2)()
    for i in range(2):
        c = C.c_void_p()
        assert lib.fmoe_create(C.byref(c), C.byref(cfg), 0) == 0
        ctxs[i] = c.value
    plan2 = (binding.FmoeLayerPlan * 2)()
    assert lib.fmoe_stack_plan(2, 2, 1, 1, (C.c_int32 * 1)(1), 1, C.byref(stage), plan2) == 0
    small, big = lib.fmoe_stack_workspace_bytes(ctxs, plan2, 2, 64, 2), lib.fmoe_stack_workspace_bytes(ctxs, plan2, 2, 4096, 2)
    assert 0 < small < big
    assert big > lib.fmoe_workspace_bytes(ctxs[0], 4096, 2) + 2 * 4096 * 64 * 4       # two activation buffers on top
    dummy = C.c_void_p(0x1000)
    nv, nt = (C.c_int32 * 2)(30, 20), (C.c_int32 * 2)(4, 6)
    args = lambda T, ws, wsb: (ctxs, plan2, 2, dummy, dummy, dummy, nv, nt, 2, T, None, dummy, dummy, dummy, None,
                               None, ws, wsb, None)
    assert lib.fmoe_stack_forward(*args(61, dummy, 1 << 30)) == -3            # lengths add up to 60
    assert lib.fmoe_stack_forward(*args(60, None, 0)) == -4
    assert lib.fmoe_stack_forward(*args(60, C.c_void_p(0x10000), 256)) == -4
    assert lib.fmoe_stack_forward(ctxs, None, 2, *args(60, dummy, 0)[3:]) == -2
    plan2[1].k_text = 9                                                        # above E = 8
    assert lib.fmoe_stack_forward(*args(60, C.c_void_p(0x10000), 1 << 30)) == -1
    plan2[1].k_text = 2
    other = binding.FmoeConfig(128, 8, 32, 0, 0, 2, 1, 1, binding.FMOE_F32)     # another d_model
    c = C.c_void_p()
    assert lib.fmoe_create(C.byref(c), C.byref(other), 0) == 0
    mixed = (C.c_void_p * 2)(ctxs[0], c.value)
    assert lib.fmoe_stack_workspace_bytes(mixed, plan2, 2, 64, 2) == 0
    assert lib.fmoe_stack_forward(mixed, *args(60, C.c_void_p(0x10000), 1 << 30)[1:]) == -3
    for p in (ctxs[0], ctxs[1], c.value):
        lib.fmoe_destroy(C.c_void_p(p))


def test_four_gib_extents_and_empty_sequence_lists_are_refused(lib):
    """bf16 expert GEMMs address activation rows with 32-bit byte offsets; every such offset is clamped
    below 4 GiB inside the kernel and the host refuses buffers that could not be addressed -- before the
    weights are even looked at, so the refusal needs no GPU.  A batch with tokens but no sequence is an
    argument error (the pruning stage could not place its tokens)."""
    dummy = C.c_void_p(0x1000)
    cfg = binding.FmoeConfig(2048, 64, 1408, 2, 1408, 6, 3, 1, binding.FMOE_BF16)
    ctx = C.c_void_p()
    assert lib.fmoe_create(C.byref(ctx), C.byref(cfg), 0) == 0
    T_big = (1 << 32) // (2 * 2048) + 1                                       # x alone passes 4 GiB
    assert T_big < (1 << 24)
    lf = lambda T, B: lib.fmoe_layer_forward(ctx, None, dummy, dummy, dummy, B, T, None, 0, dummy, dummy, dummy,
                                              None, dummy, 0, None)
    assert lf(T_big, 1) == -5 and b"4 GiB" in lib.fmoe_last_error()
    T_hid = (1 << 32) // (2 * 6 * 1408) + 1                                   # x fits, the hidden buffer does not
    assert T_hid * 2048 * 2 < (1 << 32)
    assert lf(T_hid, 1) == -5 and b"hidden buffer" in lib.fmoe_last_error()
    assert lib.fmoe_expert_ffn(ctx, dummy, None, T_hid, None, dummy, dummy, dummy, dummy, dummy, 0, None) == -5
    assert lf(T_hid - 1, 1) == -1 and b"fmoe_set_weights" in lib.fmoe_last_error()   # in range: next check
    lib.fmoe_destroy(ctx)
    f32 = binding.FmoeConfig(2048, 64, 1408, 2, 1408, 6, 3, 1, binding.FMOE_F32)   # fp32 contexts use 64-bit pointers
    assert lib.fmoe_create(C.byref(ctx), C.byref(f32), 0) == 0
    assert lf(T_big, 1) == -1 and b"fmoe_set_weights" in lib.fmoe_last_error()
    # tokens but no sequence
    pp = binding.prune_params(retention=0.5, window=3)
    assert lib.fmoe_prune(ctx, C.byref(pp), dummy, dummy, dummy, 0, 4, None, None, dummy, dummy, None, None, None,
                          dummy, 0, None) == -1
    assert b"no sequence" in lib.fmoe_last_error()
    lib.fmoe_destroy(ctx)


def test_permute_noalloc_refuses_sizes_beyond_its_static_scratch(lib):
    cfg = binding.FmoeConfig(64, 8, 32, 0, 0, 8, 1, 1, binding.FMOE_F32)
    ctx = C.c_void_p()
    assert lib.fmoe_create(C.byref(ctx), C.byref(cfg), 0) == 0
    dummy = C.c_void_p(0x1000)
    call = lambda n: lib.fmoe_permute_noalloc(ctx, dummy, None, n, None, dummy, dummy, dummy, None)
    assert call(65537) == -5 and b"static scratch" in lib.fmoe_last_error()
    assert call(-1) == -1
    assert lib.fmoe_set_topk(ctx, 8, 8) == 0
    assert lib.fmoe_permute_noalloc(ctx, dummy, None, 16, None, None, dummy, dummy, None) == -2
    lib.fmoe_destroy(ctx)
    big = binding.FmoeConfig(64, 32, 32, 0, 0, 16, 16, 1, binding.FMOE_F32)   # 65536 x 16 = 2^20 slots: the limit
    assert lib.fmoe_create(C.byref(ctx), C.byref(big), 0) == 0
    assert lib.fmoe_permute_noalloc(ctx, dummy, None, 65536, None, None, dummy, dummy, None) == -2   # passes the size check
    lib.fmoe_destroy(ctx)
    assert lib.fmoe_permute_noalloc(None, dummy, None, 4, None, dummy, dummy, dummy, None) == -2


def test_build_check_catches_compiler_use_of_hand_placed_accumulation_registers(tmp_path):
    """The dense-shape GEMM kernels name their accumulation registers themselves; the build reads the
    compiler's assembly and must refuse any a<N> operand the compiler placed inside those kernels."""
    from paper_2511_17885_amd import build
    ok = ("_ZN1x16ffn_dense_kernelILb1ELi2EEEv:\n\ts_cbranch_scc1 .LBB0_2\n\ts_endpgm\n.LBB0_2:\n"   # an early exit
          "\tv_add_u32 v1, v2, v3\n\t;;#ASMSTART\n"
          "\tv_mfma_f32_16x16x32_bf16 a[0:3], v[4:7], v[8:11], a[0:3]\n\t;;#ASMEND\n\ts_endpgm\n.Lfunc_end0:\n"
          "_ZN1x17ffn_stream_kernelILb1EEEv:\n\tv_accvgpr_write_b32 a7, v0\n\ts_endpgm\n.Lfunc_end1:\n")
    p = tmp_path / "ok.s"
    p.write_text(ok)
    assert build.check_accumulation_registers(str(p)) == 1
    # planted after the kernel's first s_endpgm: the whole kernel is read, not only the code before its first exit
    for planted in ("\tv_accvgpr_write_b32 a5, v102\n", "\tbuffer_load_dwordx4 a[8:11], v1, s[0:3], 0 offen\n",
                    "\tv_accvgpr_read_b32 v101, a0\n"):
        bad = tmp_path / "bad.s"
        bad.write_text(ok.replace("\tv_add_u32 v1, v2, v3\n", planted))
        with pytest.raises(RuntimeError):
            build.check_accumulation_registers(str(bad))
    none = tmp_path / "none.s"
    none.write_text("_ZN1x17ffn_stream_kernelILb1EEEv:\n\ts_endpgm\n.Lfunc_end0:\n")
    with pytest.raises(RuntimeError):
        build.check_accumulation_registers(str(none))
    # and the assembly of the library as built passes
    real = os.path.join(os.path.dirname(binding.LIB_PATH), "_build", "ffn-hip-amdgcn-amd-amdhsa-gfx950.s")
    if os.path.exists(real):
        assert build.check_accumulation_registers(real) == 2
