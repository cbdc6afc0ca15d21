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
