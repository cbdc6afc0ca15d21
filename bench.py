#!/usr/bin/env python3
"""Benchmark of the MoE-layer prefill path on one MI355X.

A "step" is one fmoe_layer_forward call: router softmax, modality-dependent top-k, routing-aware
visual-token pruning, permutation by expert, SwiGLU grouped GEMM, gate-weighted combine, over one
batch of synthetic tokens that is already resident in HBM.  Metric: input tokens per second.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2]

Prints ONE JSON line.  Besides the contract fields it carries
  roofline      the dominant kernel (routed gate/up grouped GEMM): algorithmic bytes per launch
                over its HIP-event duration, against the 8 TB/s HBM peak,
  kernels       the same for every kernel of the step (instrumentation pass after the timed one),
  cpu_baseline  the CPU oracle timed on the host cores on the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
MFMA_F32_PEAK_TFLOPS = 157.3
VALU_F32_PEAK_TFLOPS = 157.3
# HBM bytes per launch of the dominant kernel on workload c2 from two rocprofv3 --pmc runs
# (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, KiB; the factors are what a 256 MiB device copy reads on the
# same counters) -- profiles/ffn_stream_c2_hbm_traffic.md.  Other workloads: not measured.
MEASURED_TRAFFIC_BYTES = {"c2": int((84611.9 * 2.0 + 7616.0) * 1024)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5_layer", "c5_layer_full"],
                    help="c2 is the configuration the metric is quoted on; the others are context "
                         "(c5_layer: one layer of the ragged 8-sequence batch with pruning, "
                         "c5_layer_full: the same layer with top-6 for every token and no pruning)")
    ap.add_argument("--gamma", type=float, default=0.0,
                    help="merge rate of Sec. 3.2.3 (context runs; the metric is quoted at 0, i.e. without merging)")
    ap.add_argument("--weight-copies", type=int, default=None,
                    help="cycle the steps over this many copies of the layer's weights, each in device memory of "
                         "its own (same values, same result).  Default 4 for workload c2, whose 164 MB of touched "
                         "weights would otherwise partly stay in the 256 MB memory-side cache from one step to "
                         "the next, which no layer of a real model's forward pass enjoys; 1 elsewhere (those "
                         "layers exceed that cache on their own)")
    ap.add_argument("--also-same-copy", action="store_true",
                    help="after the timed region, time the same number of steps on one copy of the weights only "
                         "and add the result as 'same_weights_every_step' (off by default: a kernel trace of the "
                         "run would otherwise average launches with and without cache-resident weights)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-steps", type=int, default=30)
    ap.add_argument("--copy-calib", action="store_true",
                    help="also run a plain 256 MiB device copy (scale for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives are part of it); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2511_17885_amd import binding, workloads as W

    torch.cuda.set_device(0)
    def c5_layer_full():
        w5 = W.config5(n_layers=1)
        w5.k_visual, w5.retention, w5.name = 6, 1.0, w5.name + "_full_activation"
        return w5

    wl = {"c1": W.config1, "c2": W.config2, "c3": W.config3, "c4": W.config4,
          "c5_layer": lambda: W.config5(n_layers=1), "c5_layer_full": c5_layer_full}[args.workload]()
    is_bf16 = wl.dtype == W.BF16
    td = torch.bfloat16 if is_bf16 else torch.float32
    es = 2 if is_bf16 else 4

    def dev(a, t=None):
        if a is None:
            return None
        r = torch.from_numpy(np.ascontiguousarray(a)).cuda()
        return r.to(t).contiguous() if t is not None else r

    def make_ctx(w):
        c = binding.FMoE(d_model=wl.d, n_experts=wl.E, d_ffn=wl.F, n_shared=wl.n_shared,
                         d_ffn_shared=wl.F_shared if wl.n_shared else 0, k_text=wl.k_text,
                         k_visual=wl.k_visual, dtype=wl.dtype)
        c.set_weights(dev(w.router_w, td), dev(w.router_bias), dev(w.w_gate, td), dev(w.w_up, td),
                      dev(w.w_down, td), dev(w.ws_gate, td), dev(w.ws_up, td), dev(w.ws_down, td))
        return c

    # every copy holds the same layer: the steps differ only in where their weights live
    NL = args.weight_copies if args.weight_copies is not None else (4 if args.workload == "c2" else 1)
    NL = max(1, min(NL, 64))
    lw = wl.weights
    ctxs = [make_ctx(lw) for _ in range(NL)]
    m = ctxs[0]
    x, vis, cu = dev(wl.x, td), dev(wl.is_visual), dev(wl.cu_seqlens)
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

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(args.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    ms_per_step = ev0.elapsed_time(ev1) / args.steps
    same_layer_ms = None
    if NL > 1 and args.also_same_copy:   # for comparison: the same copy of the weights every step
        for _ in range(args.warmup):
            m.layer_forward(x, vis, cu, pp, out=out, kept_idx=kept, new_cu=new_cu)
        ev0.record()
        for _ in range(args.steps):
            m.layer_forward(x, vis, cu, pp, out=out, kept_idx=kept, new_cu=new_cu)
        ev1.record()
        torch.cuda.synchronize()
        same_layer_ms = ev0.elapsed_time(ev1) / args.steps

    # ---- instrumentation pass: HIP events around every kernel, on the launch stream
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

    # ---- algorithmic work per launch, from the shapes and the routing result of this input
    n_kept = int(new_cu[-1].item())
    # (expert_offsets lives in the workspace; recompute the routing through the entry points)
    probs, idx, gate = m.route(x, vis, want_probs=False)
    offs, _, _ = m.permute(idx.contiguous(), kept, n_kept)
    offs = offs.cpu().numpy()
    M = int(offs[-1])
    touched = int((np.diff(offs) > 0).sum())
    d, F, E, Ns, Fs, Kmax = wl.d, wl.F, wl.E, wl.n_shared, wl.F_shared, max(wl.k_text, wl.k_visual)
    n_vis = int(wl.is_visual.sum())
    work = {
        "route_kernel": dict(bytes=T * d * es + n_vis * E * 4 + T * Kmax * 8 + E * d * 4,
                             flops=2.0 * T * d * E, peak_tflops=MFMA_F32_PEAK_TFLOPS),
        # one launch covers the routed experts and the shared group
        "ffn_stream_kernel<true>": dict(
            bytes=(touched * 2 * F * d + M * d + M * F + Ns * 2 * Fs * d + n_kept * d * (1 if Ns else 0)
                   + n_kept * Ns * Fs) * es,
            flops=4.0 * M * d * F + 4.0 * n_kept * d * Fs * Ns,
            peak_tflops=MFMA_BF16_PEAK_TFLOPS if is_bf16 else MFMA_F32_PEAK_TFLOPS),
        "ffn_stream_kernel<false>": dict(
            bytes=(touched * d * F + M * F + M * d + Ns * d * Fs + n_kept * Ns * Fs
                   + n_kept * d * (1 if Ns else 0)) * es,
            flops=2.0 * M * d * F + 2.0 * n_kept * d * Fs * Ns,
            peak_tflops=MFMA_BF16_PEAK_TFLOPS if is_bf16 else MFMA_F32_PEAK_TFLOPS),
        "combine_kernel": dict(bytes=M * d * es + Ns * n_kept * d * es + n_kept * d * es
                               + n_kept * Kmax * 8, flops=2.0 * M * d, peak_tflops=VALU_F32_PEAK_TFLOPS),
        "window_score_kernel": dict(bytes=n_vis * E * 4 + (n_vis // wl.window) * 4, flops=6.0 * n_vis * E,
                                    peak_tflops=VALU_F32_PEAK_TFLOPS),
        "permute_count_kernel": dict(bytes=n_kept * Kmax * 8, flops=0.0, peak_tflops=VALU_F32_PEAK_TFLOPS),
        "permute_scatter_kernel": dict(bytes=n_kept * Kmax * 12 + M * 4, flops=0.0,
                                       peak_tflops=VALU_F32_PEAK_TFLOPS),
    }
    kernels = {}
    for name, ms in kms.items():
        ent = {"us": round(ms * 1e3, 2)}
        w = work.get(name)
        if w and ms > 0:
            gbs = w["bytes"] / (ms * 1e-3) / 1e9
            tfl = w["flops"] / (ms * 1e-3) / 1e12
            ent.update(algo_bytes=int(w["bytes"]), GBps=round(gbs, 1), hbm_frac=round(gbs / HBM_PEAK_GBS, 4),
                       TFLOPs=round(tfl, 2), compute_frac=round(tfl / w["peak_tflops"], 4))
        kernels[name] = ent

    dom = "ffn_stream_kernel<true>"   # gate/up projections + SwiGLU of all experts, routed and shared
    dom_ms = kms.get(dom, 0.0)
    roofline = None
    if dom_ms > 0:
        ach = work[dom]["bytes"] / (dom_ms * 1e-3) / 1e9
        roofline = {"kernel": dom, "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": MEASURED_TRAFFIC_BYTES.get(args.workload),
                    "algo_bytes_per_launch": int(work[dom]["bytes"]), "us_per_launch": round(dom_ms * 1e3, 2),
                    "mfma_frac": kernels[dom].get("compute_frac")}

    if args.copy_calib:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        t0 = time.time()
        passes = 0
        while passes == 0 or (time.time() - t0 < 10.0 and passes < 1000):   # about 10 s of CPU work
            oracle.layer_forward(wl.x, wl.is_visual, wl.cu_seqlens, lw, k_text=wl.k_text,
                                 k_visual=wl.k_visual, is_bf16=is_bf16, retention=wl.retention,
                                 window=wl.window, gamma=args.gamma)
            passes += 1
        dt = time.time() - t0
        cpu = {"value": round(passes * T / dt, 1), "unit": "tokens/s", "cores": oracle.num_threads(),
               "kind": "oracle", "seconds": round(dt, 2),
               "sample": f"{passes} passes of the full layer over the whole {wl.name} batch ({T} tokens each)"}

    line = {
        "metric": "MoE-layer prefill tokens/s (visual-reduced top-k + pruning)",
        "value": round(T / (ms_per_step * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if is_bf16 else "f32", "data": "synthetic",
        "config": {"workload": wl.name, "tokens": T, "visual": n_vis, "d_model": d, "experts": E,
                   "d_ffn": F, "shared_experts": Ns, "k_text": wl.k_text, "k_visual": wl.k_visual,
                   "retention": wl.retention, "window": wl.window, "kept_tokens": n_kept,
                   "routed_rows": M, "experts_touched": touched, "weight_copies": NL,
                   **({"gamma": args.gamma} if args.gamma > 0 else {})},
        "roofline": roofline, "cpu_baseline": cpu,
        **({"same_weights_every_step": {"ms_per_step": round(same_layer_ms, 5),
                                      "value": round(T / (same_layer_ms * 1e-3), 1)}} if same_layer_ms else {}),
        "kernel_sum_us": round(sum(kms.values()) * 1e3, 2), "kernels": kernels,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
