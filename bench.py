#!/usr/bin/env python3
"""Benchmark of the MoE-layer prefill path on one MI355X.

Headline workload (default, `--workload c5_stack`): the ragged batched prefill -- 8 packed sequences
(22016 tokens), a 12-layer stack of DeepSeek-VL2-Small-shaped MoE layers with distinct weights,
x <- x + MoE_l(x), top-6 for every token in layers 0-1, top-6 / top-3 (text / visual) from layer 2,
routing-aware pruning of the visual tokens to 50 % once, in layer 2 -- the largest configuration that
fits one GPU.  A "step" is one fmoe_stack_forward call over the batch, already resident in HBM:
every layer runs router softmax, modality-dependent top-k, (pruning,) permutation by expert, the SwiGLU
grouped GEMMs and the gate-weighted combine.  Metric: MoE-layer prefill tokens/s = input tokens x
layers / stack time (every input token counts once per layer, whether or not pruning has removed it
by then), so that the figure compares with the single-layer workloads, where it is input tokens /
layer time.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5_stack|c2|c3|c4|...]

Prints ONE JSON line.  Besides the contract fields it carries
  roofline      the dominant kernel (gate/up grouped GEMM with the SwiGLU epilogue): algorithmic work per
                launch over its average launch duration (HIP events on the launch stream), against the
                roofline that binds it (dense bf16 MFMA peak on the stack, HBM peak on c2-c4); the other
                fraction is given beside it,
  kernels       the same for every kernel of the step (instrumentation pass after the timed one),
  cpu_baseline  the CPU oracle timed on the host cores on a bounded sample of the same workload,
  context       (headline run only) the single-layer workloads c2, c3, c4 measured the same way.
"""
import argparse
import concurrent.futures as cf
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
MFMA_F32_PEAK_TFLOPS = 157.3
VALU_F32_PEAK_TFLOPS = 157.3
GEMM1, GEMM2 = "gate_up_gemm", "down_gemm"   # work-table keys; the kernel that ran is named by the profile slots
# Bytes between the L2 caches and memory per launch of the dominant kernel, from two rocprofv3 --pmc runs per
# workload (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, KiB per dispatch; the factors are what a 256 MiB device
# copy reads on the same counters), averaged over the launches of one step --
# profiles/expert_gemm_hbm_traffic_c5_stack_c2_c3_c4.md.  The figures belong to the kernels as they
# were when that file was written; a workload without an entry has not been measured (traffic: null).
MEASURED_TRAFFIC_BYTES = {   # workload -> (the kernel the figure belongs to, bytes per launch)
    "c5_stack": ("ffn_dense_kernel<true>", int((1492851.1 * 2.0 + 219765.4) * 1024)),
    "c2": ("ffn_stream_kernel<true>", int((84300.2 * 2.0 + 7616.0) * 1024)),
    "c3": ("ffn_dense_kernel<true>", int((483120.4 * 2.0 + 32032.0) * 1024)),
    "c4": ("ffn_dense_kernel<true>", int((420595.5 * 2.0 + 26880.0) * 1024)),
}


def _dev(a, t=None):
    import numpy as np
    import torch
    if a is None:
        return None
    r = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return r.to(t).contiguous() if t is not None else r


def _make_ctx(binding, wl, lw, td, k_text=None, k_visual=None, release=True, ffn_shape=0):
    c = binding.FMoE(d_model=wl.d, n_experts=wl.E, d_ffn=wl.F, n_shared=wl.n_shared,
                     d_ffn_shared=wl.F_shared if wl.n_shared else 0,
                     k_text=wl.k_text if k_text is None else k_text,
                     k_visual=wl.k_visual if k_visual is None else k_visual, dtype=wl.dtype)
    c.set_weights(_dev(lw.router_w, td), _dev(lw.router_bias), _dev(lw.w_gate, td), _dev(lw.w_up, td),
                  _dev(lw.w_down, td), _dev(lw.ws_gate, td), _dev(lw.ws_up, td), _dev(lw.ws_down, td),
                  release_packed=release)
    c.set_ffn_shape(ffn_shape)
    return c


def _time_steps(torch, step, steps, warmup):
    """(mean ms per step over exactly `steps` steps between two synchronisations, median ms of
    per-step event pairs from a second loop of the same length)."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    mean_ms = ev0.elapsed_time(ev1) / steps
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, b in pairs:
        a.record()
        step()
        b.record()
    torch.cuda.synchronize()
    return mean_ms, statistics.median(a.elapsed_time(b) for a, b in pairs)


def _layer_work(d, F, E, Ns, Fs, es, Kmax, T_in, n_vis_in, n_kept, M, touched, prune, window, residual, bf16):
    """Algorithmic bytes and flops of one launch of every kernel of a layer."""
    gemm_peak = MFMA_BF16_PEAK_TFLOPS if bf16 else MFMA_F32_PEAK_TFLOPS
    sh = 1 if Ns else 0
    return {
        "route_kernel": dict(bytes=T_in * d * es + (n_vis_in * E * 4 if prune else 0) + T_in * Kmax * 8 + E * d * 4,
                             flops=2.0 * T_in * d * E, peak=MFMA_F32_PEAK_TFLOPS),
        GEMM1: dict(bytes=(touched * 2 * F * d + M * d + M * F + Ns * 2 * Fs * d + n_kept * d * sh + n_kept * Ns * Fs) * es,
                    flops=4.0 * M * d * F + 4.0 * n_kept * d * Fs * Ns, peak=gemm_peak),
        GEMM2: dict(bytes=(touched * d * F + M * F + M * d + Ns * d * Fs + n_kept * Ns * Fs + n_kept * d * Ns) * es,
                    flops=2.0 * M * d * F + 2.0 * n_kept * d * Fs * Ns, peak=gemm_peak),
        "combine_kernel": dict(bytes=(M * d + Ns * n_kept * d + n_kept * d + (n_kept * d if residual else 0)) * es
                               + n_kept * Kmax * 8, flops=2.0 * M * d, peak=VALU_F32_PEAK_TFLOPS),
        "window_score_kernel": dict(bytes=(n_vis_in * E * 4 + (n_vis_in // max(window, 1)) * 4) if prune else 0,
                                    flops=6.0 * n_vis_in * E if prune else 0.0, peak=VALU_F32_PEAK_TFLOPS),
        "permute_count_kernel": dict(bytes=n_kept * Kmax * 8, flops=0.0, peak=VALU_F32_PEAK_TFLOPS),
        "permute_scatter_kernel": dict(bytes=n_kept * Kmax * 12 + M * 4, flops=0.0, peak=VALU_F32_PEAK_TFLOPS),
    }


def _kernel_table(kms, launches, work):
    """kms: {kernel: total ms per step}, launches: {kernel: launches per step}, work: {kernel: summed
    bytes / flops per step}."""
    out = {}
    for name, ms in kms.items():
        n = max(launches.get(name, 1), 1)
        ent = {"us": round(ms * 1e3 / n, 2), "launches_per_step": n}
        w = work.get(name)
        if w and ms > 0 and (w["bytes"] > 0 or w["flops"] > 0):
            gbs = w["bytes"] / (ms * 1e-3) / 1e9
            tfl = w["flops"] / (ms * 1e-3) / 1e12
            ent.update(algo_bytes=int(w["bytes"] / n), GBps=round(gbs, 1), hbm_frac=round(gbs / HBM_PEAK_GBS, 4),
                       TFLOPs=round(tfl, 2), compute_frac=round(tfl / w["peak"], 4))
        out[name] = ent
    return out


def _gemm_names(names):
    """{work-table key: kernel name} for the expert GEMM kernels among `names` (either shape of the kernel)."""
    out = {}
    for n in names:
        if n.startswith("ffn_") and n.endswith("<true>"):
            out[GEMM1] = n
        if n.startswith("ffn_") and n.endswith("<false>"):
            out[GEMM2] = n
    return out


def _named_work(work, names):
    """The work table with the GEMM entries under the names of the kernels that ran."""
    g = _gemm_names(names)
    return {g.get(k, k): v for k, v in work.items()}


def _roofline(kernels, work, launches, workload, bound):
    cands = [n for n in kernels if n.startswith("ffn_") and n.endswith("<true>") and "GBps" in kernels[n]]
    if not cands:
        return None
    name = max(cands, key=lambda n: kernels[n]["us"] * kernels[n]["launches_per_step"])   # the dominant kernel
    k = kernels[name]
    n = max(launches.get(name, 1), 1)
    measured = MEASURED_TRAFFIC_BYTES.get(workload)
    r = {"kernel": name, "bound": bound, "us_per_launch": k["us"], "launches_per_step": n,
         "traffic": measured[1] if measured and measured[0] == name else None,
         "algo_bytes_per_launch": int(work[name]["bytes"] / n), "algo_flops_per_launch": work[name]["flops"] / n}
    if bound == "mfma":
        r.update(achieved=k["TFLOPs"], peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s", frac=k["compute_frac"],
                 hbm_frac=k["hbm_frac"])
    else:
        r.update(achieved=k["GBps"], peak=HBM_PEAK_GBS, unit="GB/s", frac=k["hbm_frac"], mfma_frac=k["compute_frac"])
    return r


def run_layer(args, name, cpu_baseline):
    """One fmoe_layer_forward per step on a single-layer workload."""
    import numpy as np
    import torch
    from paper_2511_17885_amd import binding, workloads as W

    def c5_layer_full():
        w5 = W.config5(n_layers=1)
        w5.k_visual, w5.retention, w5.name = 6, 1.0, w5.name + "_full_activation"
        return w5

    wl = {"c1": W.config1, "c2": W.config2, "c3": W.config3, "c4": W.config4,
          "c5_layer": lambda: W.config5(n_layers=1), "c5_layer_full": c5_layer_full}[name]()
    is_bf16 = wl.dtype == W.BF16
    td = torch.bfloat16 if is_bf16 else torch.float32
    es = 2 if is_bf16 else 4
    # every copy holds the same layer: the steps differ only in where their weights live (c2's 164 MB of
    # touched weights would otherwise partly stay in the 256 MB memory-side cache from step to step,
    # which no layer of a model's forward pass enjoys; the larger layers exceed that cache on their own)
    NL = args.weight_copies if args.weight_copies is not None else (4 if name == "c2" else 1)
    NL = max(1, min(NL, 64))
    lw = wl.weights
    ctxs = [_make_ctx(binding, wl, lw, td, ffn_shape=args.ffn_shape) for _ in range(NL)]
    m = ctxs[0]
    x, vis, cu = _dev(wl.x, td), _dev(wl.is_visual), _dev(wl.cu_seqlens)
    pp = binding.prune_params(retention=wl.retention, window=wl.window, gamma=args.gamma)
    T, B = wl.T, wl.B
    out = torch.empty((T, wl.d), dtype=td, device="cuda")
    kept = torch.empty(T, dtype=torch.int32, device="cuda")
    new_cu = torch.empty(B + 1, dtype=torch.int32, device="cuda")
    for c in ctxs:
        c.workspace(T, B)
    calls = [0]

    def step():
        c = ctxs[calls[0] % NL]
        calls[0] += 1
        c.layer_forward(x, vis, cu, pp, out=out, kept_idx=kept, new_cu=new_cu)
        return c

    mean_ms, median_ms = _time_steps(torch, step, args.steps, args.warmup)

    for c in ctxs:
        c.profile_enable(True)
    acc = {}
    nprof = max(1, min(args.profile_steps, args.steps))
    nprof = (nprof + NL - 1) // NL * NL          # every copy the same number of times
    for _ in range(nprof):
        c = step()
        for k, v in c.profile_read().items():
            acc[k] = acc.get(k, 0.0) + v
    for c in ctxs:
        c.profile_enable(False)
    kms = {k: v / nprof for k, v in acc.items()}

    n_kept = int(new_cu[-1].item())
    _, idx, _ = m.route(x, vis, want_probs=False)
    offs, _, _ = m.permute(idx.contiguous(), kept, n_kept)
    offs = offs.cpu().numpy()
    M = int(offs[-1])
    touched = int((np.diff(offs) > 0).sum())
    Kmax = max(wl.k_text, wl.k_visual)
    n_vis = int(wl.is_visual.sum())
    work = _layer_work(wl.d, wl.F, wl.E, wl.n_shared, wl.F_shared, es, Kmax, T, n_vis, n_kept, M, touched,
                       wl.retention < 1.0, wl.window, False, is_bf16)
    launches = {k: 1 for k in kms}
    work = _named_work(work, kms)
    kernels = _kernel_table(kms, launches, work)
    rows_per_expert = M / max(touched, 1)
    res = {
        "value": round(T / (mean_ms * 1e-3), 1), "ms_per_step": round(mean_ms, 5),
        "ms_per_step_median": round(median_ms, 5),
        "config": {"workload": wl.name, "tokens": T, "visual": n_vis, "d_model": wl.d, "experts": wl.E,
                   "d_ffn": wl.F, "shared_experts": wl.n_shared, "k_text": wl.k_text, "k_visual": wl.k_visual,
                   "retention": wl.retention, "window": wl.window, "kept_tokens": n_kept, "routed_rows": M,
                   "experts_touched": touched, "weight_copies": NL,
                   **({"gamma": args.gamma} if args.gamma > 0 else {})},
        "dtype": "bf16" if is_bf16 else "f32",
        "roofline": _roofline(kernels, work, launches, name if args.gamma == 0 else None,
                              "mfma" if rows_per_expert >= 315 else "hbm"),
        "kernel_sum_us": round(sum(kms.values()) * 1e3, 2), "kernels": kernels,
    }
    if cpu_baseline:
        import oracle
        t0 = time.time()
        passes = 0
        while passes == 0 or (time.time() - t0 < 10.0 and passes < 1000):   # about 10 s of CPU work
            oracle.layer_forward(wl.x, wl.is_visual, wl.cu_seqlens, lw, k_text=wl.k_text,
                                 k_visual=wl.k_visual, is_bf16=is_bf16, retention=wl.retention,
                                 window=wl.window, gamma=args.gamma)
            passes += 1
        dt = time.time() - t0
        res["cpu_baseline"] = {"value": round(passes * T / dt, 1), "unit": "tokens/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "seconds": round(dt, 2),
                               "sample": f"{passes} passes of the full layer over the whole {wl.name} batch ({T} tokens each)"}
    for c in ctxs:
        c.close()
    del ctxs, x, out
    torch.cuda.empty_cache()
    return res


def run_stack(args, cpu_baseline):
    """One fmoe_stack_forward per step on the full-size config-5 stack."""
    import numpy as np
    import torch
    from paper_2511_17885_amd import binding, workloads as W

    wl = W.config5()
    td, es = torch.bfloat16, 2
    n_layers = len(wl.layers)
    t0 = time.time()
    layers = []
    with cf.ThreadPoolExecutor(max_workers=3) as ex:   # layers are drawn from independent seeded streams
        for l, lw in enumerate(ex.map(lambda l: wl.layers[l], range(n_layers))):
            kt, kv = wl.k_schedule[l]
            layers.append(_make_ctx(binding, wl, lw, td, kt, kv, ffn_shape=args.ffn_shape))
            del lw
    setup_s = time.time() - t0
    sched = {wl.prune_after_layer: binding.prune_params(retention=wl.retention, window=wl.window, prune_mode=2)}
    stack = binding.FMoEStack(layers, wl.k_schedule, prune_schedule=sched)
    x, vis, cu = _dev(wl.x, td), _dev(wl.is_visual), _dev(wl.cu_seqlens)
    T, B = wl.T, wl.B
    bounds = wl.cu_seqlens
    nv = [int(wl.is_visual[s:e].sum()) for s, e in zip(bounds[:-1], bounds[1:])]
    nt = [int(e - s) - v for s, e, v in zip(bounds[:-1], bounds[1:], nv)]
    out = torch.empty((T, wl.d), dtype=td, device="cuda")
    kept = torch.empty(T, dtype=torch.int32, device="cuda")
    new_cu = torch.empty(B + 1, dtype=torch.int32, device="cuda")

    def step():
        return stack.forward(x, vis, cu, nv, nt, out=out, kept_idx=kept, new_cu=new_cu)

    mean_ms, median_ms = _time_steps(torch, step, args.steps, args.warmup)

    # ---- instrumentation pass: HIP events around every kernel of every layer, on the launch stream
    for c in layers:
        c.profile_enable(True)
    acc, cnt = {}, {}
    layer_kernels = [set() for _ in layers]   # which kernels each layer launched (the GEMM shape is per call)
    nprof = max(1, min(args.profile_steps, args.steps))
    for _ in range(nprof):
        step()
        for l, c in enumerate(layers):
            for k, v in c.profile_read().items():
                acc[k] = acc.get(k, 0.0) + v
                cnt[k] = cnt.get(k, 0) + 1
                layer_kernels[l].add(k)
    for c in layers:
        c.profile_enable(False)
    kms = {k: v / nprof for k, v in acc.items()}
    launches = {k: round(v / nprof) for k, v in cnt.items()}

    # ---- algorithmic work per step: every token lists exactly k experts, so the routed rows of a layer
    # follow from the token counts (host bookkeeping of the budget rule); at these sizes every expert
    # is touched in every layer
    n_out = int(new_cu[-1].item())
    nv_kept = binding.kept_visual_lens(nv, wl.retention)
    assert n_out == sum(nv_kept) + sum(nt)
    work = {}
    per_layer = []
    cur_nv, n_text = sum(nv), sum(nt)
    for l in range(n_layers):
        kt, kv = wl.k_schedule[l]
        stage = l == wl.prune_after_layer
        T_in, nv_in = cur_nv + n_text, cur_nv
        if stage:
            cur_nv = sum(nv_kept)
        n_kept = cur_nv + n_text
        M = n_text * kt + cur_nv * kv
        per_layer.append({"layer": l, "tokens_in": T_in, "kept_tokens": n_kept, "routed_rows": M,
                          "rows_per_expert": round(M / wl.E, 1), "k": [kt, kv]})
        w = _layer_work(wl.d, wl.F, wl.E, wl.n_shared, wl.F_shared, es, max(kt, kv), T_in, nv_in, n_kept, M, wl.E,
                        stage, wl.window, True, True)
        for k, v in _named_work(w, layer_kernels[l]).items():
            e = work.setdefault(k, dict(bytes=0.0, flops=0.0, peak=v["peak"]))
            e["bytes"] += v["bytes"]
            e["flops"] += v["flops"]
    kernels = _kernel_table(kms, launches, work)
    res = {
        "value": round(T * n_layers / (mean_ms * 1e-3), 1), "ms_per_step": round(mean_ms, 5),
        "ms_per_step_median": round(median_ms, 5),
        "config": {"workload": "c5_stack", "name": wl.name, "value_definition": "input tokens x layers / stack time",
                   "tokens": T, "sequences": B, "sequence_lengths": [int(v) for v in np.diff(bounds)],
                   "layers": n_layers, "d_model": wl.d, "experts": wl.E, "d_ffn": wl.F,
                   "shared_experts": wl.n_shared, "k_schedule": "6/6 in layers 0-1, 6/3 from layer 2",
                   "prune": f"once, in layer {wl.prune_after_layer}, retention {wl.retention}, window {wl.window}",
                   "tokens_out": n_out, "weights_GB": round(sum(
                       (3 * wl.E * wl.F + 3 * wl.n_shared * wl.F_shared + wl.E) * wl.d * 2 for _ in range(n_layers)) / 1e9, 2),
                   "per_layer": per_layer, "setup_seconds": round(setup_s, 1)},
        "dtype": "bf16",
        "roofline": _roofline(kernels, work, launches, "c5_stack", "mfma"),
        "kernel_sum_us": round(sum(kms.values()) * 1e3, 2), "kernels": kernels,
    }

    if cpu_baseline:
        # the oracle on the whole 12-layer schedule, over the shortest sequence of the batch (a bounded
        # sample: the full batch would take the host several minutes); weights drawn again layer by layer
        # outside the timed sections
        import oracle
        b = int(np.argmin(np.diff(bounds)))
        s, e = int(bounds[b]), int(bounds[b + 1])
        xs, vs = wl.x[s:e], wl.is_visual[s:e]
        cs = np.array([0, e - s], np.int32)
        spent = 0.0
        for l in range(n_layers):
            lw = wl.layers[l]
            kt, kv = wl.k_schedule[l]
            stage = l == wl.prune_after_layer
            t1 = time.time()
            o = oracle.layer_forward(xs, vs, cs, lw, k_text=kt, k_visual=kv, is_bf16=True, add_residual=True,
                                     do_prune=stage, retention=wl.retention if stage else 1.0, window=wl.window)
            spent += time.time() - t1
            if stage:
                vs, cs = vs[o["kept_idx"]], o["new_cu_seqlens"]
            xs = o["out"]
            del lw
        res["cpu_baseline"] = {"value": round((e - s) * n_layers / spent, 1), "unit": "tokens/s",
                               "cores": oracle.num_threads(), "kind": "oracle", "seconds": round(spent, 2),
                               "sample": f"the whole {n_layers}-layer schedule on the shortest sequence of the batch "
                                         f"({e - s} of {T} tokens); same definition: input tokens x layers / time"}
    for c in layers:
        c.close()
    del layers, stack, x, out
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c5_stack",
                    choices=["c5_stack", "c1", "c2", "c3", "c4", "c5_layer", "c5_layer_full"],
                    help="c5_stack (default): the full-size 12-layer ragged stack, the largest configuration that "
                         "fits one GPU; the others are single layers (c5_layer: one layer of the ragged batch "
                         "with pruning, c5_layer_full: the same with top-6 for every token and no pruning)")
    ap.add_argument("--no-context", action="store_true",
                    help="headline run only: skip the single-layer context workloads c2, c3, c4 (use this under "
                         "rocprofv3, so that the kernel averages are those of the headline workload alone)")
    ap.add_argument("--context-steps", type=int, default=100)
    ap.add_argument("--gamma", type=float, default=0.0,
                    help="merge rate of Sec. 3.2.3 (single-layer workloads; the metric is quoted at 0)")
    ap.add_argument("--weight-copies", type=int, default=None,
                    help="single-layer workloads: cycle the steps over this many copies of the layer's weights, "
                         "each in device memory of its own (default 4 for c2, 1 elsewhere)")
    ap.add_argument("--ffn-shape", type=int, default=0, choices=[0, 1, 2],
                    help="shape of the bf16 expert GEMM kernel: 0 chosen by size (default), 1 weight-stream, 2 dense")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-steps", type=int, default=20)
    ap.add_argument("--copy-calib", action="store_true",
                    help="also run a plain 256 MiB device copy (scale for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives are part of it); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    torch.cuda.set_device(0)
    cpu = not args.no_cpu_baseline
    if args.workload == "c5_stack":
        res = run_stack(args, cpu)
    else:
        res = run_layer(args, args.workload, cpu)

    context = None
    if args.workload == "c5_stack" and not args.no_context:
        context = {}
        steps, warm = args.steps, args.warmup
        args.steps, args.warmup = args.context_steps, max(args.warmup, 10)
        for name in ("c2", "c3", "c4"):
            r = run_layer(args, name, cpu)
            context[name] = {k: r[k] for k in ("value", "ms_per_step", "ms_per_step_median", "config", "roofline",
                                               "kernel_sum_us", "kernels", "cpu_baseline") if k in r}
            context[name]["unit"] = "tokens/s"
            context[name]["steps"] = args.steps
        args.steps, args.warmup = steps, warm

    if args.copy_calib:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    line = {
        "metric": "MoE-layer prefill tokens/s (visual-reduced top-k + pruning)",
        "value": res["value"], "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
        "ms_per_step_median": res["ms_per_step_median"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": res["dtype"], "data": "synthetic", "config": res["config"],
        "roofline": res["roofline"], "cpu_baseline": res.get("cpu_baseline"),
        "kernel_sum_us": res["kernel_sum_us"], "kernels": res["kernels"],
        **({"context": context} if context is not None else {}),
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
