"""Benchmark of the stage hot path on one MI355X.

A step = stage_zero_grads + stage_run_schedule(M, K, early-backward) over one batch
of synthetic micro-batches already resident in HBM, + stream sync.  Workload: the
BERT-Large-shaped stage (6 layers, hidden 1024, 16 heads, FFN 4096, seq 512,
micro-batch 4, M = 8, K = 4, bf16 storage with fp32 accumulation).

Prints one JSON line: stage samples/s (value), algorithmic TFLOP/s and its fraction
of the bf16 MFMA peak, peak activation bytes for K-slot early-backward against
M-slot GPipe order, the roofline of the dominant kernel (the MFMA GEMM, timed with
HIP events on the stage's stream in a separate profiled pass over the same steps)
and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA

# HBM-side bytes per gemm_mfma_kernel launch (average over the 528 launches of a step), from the
# rocprofv3 FETCH_SIZE / WRITE_SIZE passes summarised in profiles/gemm_mfma_bert_large_pmc_traffic.md,
# each counter scaled by what it reads for the library's copy kernel of known size (1.990 / 1.000).
# Counters cannot be read from inside this process, so the figure is carried here per workload.
GEMM_TRAFFIC_BYTES_PER_LAUNCH = {"bert_large": 64959032}


def stage_flops(cfg, M):
    """Algorithmic flops of one iteration: per layer and micro-batch the forward is
    24 T H^2 (four linear layers at F = 4H; in general 8 T H^2 + 4 T H F) + 4 T s H
    (QK^T and PV); the backward is twice that."""
    T, H, F, s = cfg.tokens, cfg.hidden, cfg.ffn, cfg.seq
    fwd = 8.0 * T * H * H + 4.0 * T * H * F + 4.0 * T * s * H
    head = 0.0
    if cfg.has_mlm_head:  # transform and vocabulary projection on the ceil(0.15 T) predicted rows
        import math
        n = math.ceil(0.15 * T)
        head = 2.0 * n * H * H + 2.0 * n * H * cfg.vocab
    return 3.0 * (fwd * cfg.n_layers + head) * M


def cpu_baseline(cfg, seed, M_sample, K_sample):
    import numpy as np
    from oracle import stage_oracle as O
    from paper_2007_01045_amd import inputs as I
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    theta = I.make_params(cfg, seed).astype(np.float64)
    st = O.Stage(I.param_layout(cfg), theta, cfg.n_layers, cfg.n_heads, cfg.ln_eps, cfg.has_embedding,
                 cfg.has_mlm_head, 1.0)
    mbs = [I.make_microbatch(cfg, seed, m) for m in range(M_sample)]
    xs = [mb["ids"] if cfg.has_embedding else mb["x"].astype(np.float64) for mb in mbs]
    dys = None if cfg.has_mlm_head else [mb["dy"].astype(np.float64) for mb in mbs]
    tg = [mb["targets"] for mb in mbs] if cfg.has_mlm_head else None
    t0 = time.perf_counter()
    O.run_schedule(st, M_sample, K_sample, O.EARLY_BACKWARD, xs, dys, tg)
    dt = time.perf_counter() - t0
    return {"value": M_sample * cfg.micro_batch / dt, "unit": "samples/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{M_sample} of the {cfg.M} micro-batches (K={K_sample}) of the same stage, float64 numpy, "
                      f"{dt:.1f} s", "tflops": stage_flops(cfg, M_sample) / dt / 1e12}


def pipeline_study(cfg, seed, S=4, layers_per_stage=3, M=16):
    """S stages of the workload's layer shape run as a pipeline on S equal partitions of the compute units
    (one virtual device each): task times F_i, B_i alone, the latency model from them, and the measured
    iteration in the early-backward order (K_i = S - i) and in the GPipe order (all M resident)."""
    import numpy as np
    import torch

    from paper_2007_01045_amd import binding as B
    from paper_2007_01045_amd import inputs as I

    part = I.StageConfig(layers_per_stage, cfg.hidden, cfg.n_heads, cfg.ffn, cfg.seq, cfg.micro_batch, M, S, cfg.dtype,
                         ln_eps=cfg.ln_eps, name="pipeline_part")
    T, H = part.tokens, part.hidden
    K = B.pipeline_warmup_depths(S, M, B.POLICY_A)
    pr = B.PipelineRunner([B.config_for(part, M, flags=B.FLAG_ONE_STREAM) for _ in range(S)],
                          [I.make_params(part, seed + i) for i in range(S)], M, parts=S)
    try:
        r0 = pr.runners[0]
        mbs = [I.make_microbatch(part, seed, m) for m in range(M)]
        xs = [r0.to_dev(mb["x"].reshape(T, H)) for mb in mbs]
        dys = [r0.to_dev(mb["dy"].reshape(T, H)) for mb in mbs]
        ys = [r0.empty_act() for _ in range(M)]
        dxs = [r0.empty_act() for _ in range(M)]
        torch.cuda.synchronize()

        def once(m, k, order):
            pr.run(m, k, order, xs[:m], dys[:m], None, ys[:m], dxs[:m])
            tl = pr.timeline(m)
            dur = {key: v[1] - v[0] for key, v in tl.items()}
            return max(v[1] for v in tl.values()), dur

        alone = [once(1, [1] * S, B.ORDER_EARLY_BACKWARD)[1] for _ in range(8)][3:]
        F = [float(np.median([d[("F", i, 0)] for d in alone])) for i in range(S)]
        Bt = [float(np.median([d[("B", i, 0)] for d in alone])) for i in range(S)]
        out = {"stages": S, "layers_per_stage": layers_per_stage, "M": M, "K": K, "compute_units_per_stage": 256 // S,
               "F_ms_alone": F, "B_ms_alone": Bt, "pivot_stage": B.pipeline_pivot_stage(M, F, Bt),
               "model_ms_from_alone": B.pipeline_latency_model(M, F, Bt)}
        for name, order, k in (("early_backward", B.ORDER_EARLY_BACKWARD, K), ("gpipe_order", B.ORDER_GPIPE, None)):
            runs = [once(M, k, order) for _ in range(4)][1:]
            span, dur = sorted(runs, key=lambda r: r[0])[len(runs) // 2]
            Fi = [float(np.mean([dur[("F", i, m)] for m in range(M)])) for i in range(S)]
            Bi = [float(np.mean([dur[("B", i, m)] for m in range(M)])) for i in range(S)]
            busy = [M * (Fi[i] + Bi[i]) for i in range(S)]
            out[name] = {"measured_ms": span, "model_ms_from_in_situ_task_times": B.pipeline_latency_model(M, Fi, Bi),
                         "F_ms_in_situ": Fi, "B_ms_in_situ": Bi, "bubble_frac_per_stage": [1.0 - b / span for b in busy],
                         "peak_resident": [int(B.stage_stats(r.h).peak_live_slots) for r in pr.runners]}
            for r in pr.runners:
                B.stage_reset_stats(r.h)
        return out
    finally:
        pr.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="bert_large")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-pipeline", action="store_true")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--seed", type=int, default=None)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs one pipeline stage on ONE GPU; --gpus must be 1 "
              "(no collectives or sharding are part of it)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2007_01045_amd import binding as B
    from paper_2007_01045_amd import inputs as I

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    B.load()           # raises if the HIP library has not been built: there is no fallback
    cfg = I.CONFIGS[args.workload]
    seed = I.DEFAULT_SEED if args.seed is None else args.seed
    M, K, T, H = cfg.M, cfg.K, cfg.tokens, cfg.hidden
    theta = I.make_params(cfg, seed)
    mbs = [I.make_microbatch(cfg, seed, m) for m in range(M)]

    def make_io(r):
        emb, head = cfg.has_embedding, cfg.has_mlm_head
        xs = [r.to_dev(mb["ids"].reshape(T).astype(np.int32)) if emb else r.to_dev(mb["x"].reshape(T, H)) for mb in mbs]
        dys = None if head else [r.to_dev(mb["dy"].reshape(T, H)) for mb in mbs]
        auxs = [r.to_dev(mb["targets"].reshape(T).astype(np.int32)) for mb in mbs] if head else None
        ys = [torch.zeros(1, dtype=torch.float32, device="cuda") if head else r.empty_act() for _ in range(M)]
        dxs = None if emb else [r.empty_act() for _ in range(M)]
        ptr = lambda ts: None if ts is None else [t.data_ptr() for t in ts]
        return xs, dys, ys, dxs, auxs, (ptr(xs), ptr(dys), ptr(ys), ptr(dxs), ptr(auxs))

    results = {}
    peak_bytes = {}
    runner = None
    # GPipe order with M slots; early-backward order with K slots; and the latter with re-computation
    # (a resident micro-batch keeps its input only and the backward task re-runs the forward)
    for order_name, order, slots, flags in (("gpipe", B.ORDER_GPIPE, M, 0),
                                            ("early_backward_recompute", B.ORDER_EARLY_BACKWARD, K, B.FLAG_RECOMPUTE),
                                            ("early_backward", B.ORDER_EARLY_BACKWARD, K, 0)):
        r = B.StageRunner(B.config_for(cfg, slots, flags=flags), theta)
        xs, dys, ys, dxs, auxs, (px, pdy, py, pdx, paux) = make_io(r)

        def step():
            B.stage_zero_grads(r.h)
            B.stage_run_schedule(r.h, M, K, order, px, pdy, py, pdx, paux)

        for _ in range(args.warmup):
            step()
        B.stage_sync(r.h)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        B.stage_sync(r.h)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        results[order_name] = dt / args.steps
        st = B.stage_stats(r.h)
        peak_bytes[order_name] = int(st.peak_activation_bytes)
        if order_name == "early_backward":
            runner = (r, step)
        else:
            del xs, dys, ys, dxs, auxs
            r.close()
            del r
            torch.cuda.empty_cache()

    # the early-backward iteration again as ONE HIP graph (captured once on a stream of its own, then
    # replayed): what is left when the host issues one launch per iteration instead of one per kernel
    if not args.no_graph:
        with torch.cuda.stream(torch.cuda.Stream()):
            rg = B.StageRunner(B.config_for(cfg, K), theta)
            gio = make_io(rg)
            gp = gio[-1]
            B.stage_zero_grads(rg.h)
            B.stage_run_schedule(rg.h, M, K, B.ORDER_EARLY_BACKWARD, gp[0], gp[1], gp[2], gp[3], gp[4])
            B.stage_sync(rg.h)
            B.stage_graph_capture(rg.h, M, K, B.ORDER_EARLY_BACKWARD, gp[0], gp[1], gp[2], gp[3], gp[4], zero_grads_first=True)
            for _ in range(args.warmup):
                B.stage_graph_launch(rg.h)
            B.stage_sync(rg.h)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                B.stage_graph_launch(rg.h)
            B.stage_sync(rg.h)
            torch.cuda.synchronize()
            results["graph"] = (time.perf_counter() - t0) / args.steps
            del gio
            rg.close()
            del rg
        torch.cuda.empty_cache()

    # per-kernel-class times: the same steps again with HIP events around every launch
    r, step = runner
    B.stage_profile_enable(r.h, True)
    prof_steps = min(args.steps, 5)
    for _ in range(prof_steps):
        step()
    prof = B.stage_profile_read(r.h)
    B.stage_profile_enable(r.h, False)
    gemm = [prof[k] for k in ("gemm_fwd", "gemm_dgrad", "gemm_wgrad")]
    g_ms = sum(p["ms"] for p in gemm)
    g_fl = sum(p["flops"] for p in gemm)
    g_n = sum(p["launches"] for p in gemm)
    achieved = g_fl / (g_ms * 1e-3) / 1e12 if g_ms > 0 else 0.0
    classes = {k: {"launches_per_step": v["launches"] / prof_steps, "ms_per_step": v["ms"] / prof_steps,
                   "tflops": (v["flops"] / (v["ms"] * 1e-3) / 1e12) if v["ms"] > 0 and v["flops"] > 0 else None}
               for k, v in prof.items() if v["launches"]}
    # the Apply step that closes a training iteration: one fused Adam pass over the stage's parameters
    # (reads g, w, m, v in fp32; writes w, m, v, the weight in the stage's dtype and the zeroed g)
    r.init_adam()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(2):
        r.apply_adam(1e-4, grad_scale=1.0 / (M * cfg.micro_batch), zero_grads=True)
    e0.record()
    n_apply = 10
    for _ in range(n_apply):
        r.apply_adam(1e-4, grad_scale=1.0 / (M * cfg.micro_batch), zero_grads=True)
    e1.record()
    torch.cuda.synchronize()
    apply_ms = e0.elapsed_time(e1) / n_apply
    apply_bytes = r.sizes.n_params * (16 + 12 + 4 + (2 if cfg.dtype == "bf16" else 4))
    r.close()

    sec = results["early_backward"]
    flops = stage_flops(cfg, M)
    out = {
        "metric": "stage samples/sec + MFMA util (%) + peak activation bytes vs GPipe order",
        "value": M * cfg.micro_batch / sec, "unit": "samples/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: L={cfg.n_layers} H={cfg.hidden} A={cfg.n_heads} F={cfg.ffn} "
                               f"s={cfg.seq} b={cfg.micro_batch} M={M} K={K}, early-backward order",
                   "seed": seed},
        "tflops_algorithmic": flops / sec / 1e12,
        "mfma_peak_frac_algorithmic": flops / sec / 1e12 / PEAK_BF16_TFLOPS,
        "gpipe_order": {"samples_per_s": M * cfg.micro_batch / results["gpipe"], "ms_per_step": results["gpipe"] * 1e3},
        "peak_activation_bytes": {"early_backward_K_slots": peak_bytes["early_backward"],
                                  "gpipe_M_slots": peak_bytes["gpipe"],
                                  "ratio": peak_bytes["early_backward"] / peak_bytes["gpipe"]},
        "roofline": {"bound": "mfma", "kernel": "gemm_mfma_kernel (all linear-layer products: fwd, dgrad, wgrad)",
                     "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS,
                     "traffic": GEMM_TRAFFIC_BYTES_PER_LAUNCH.get(cfg.name),
                     "launches_per_step": g_n / prof_steps, "avg_launch_us": g_ms * 1e3 / max(g_n, 1)},
        "recompute": {"samples_per_s": M * cfg.micro_batch / results["early_backward_recompute"],
                      "ms_per_step": results["early_backward_recompute"] * 1e3,
                      "peak_activation_bytes": peak_bytes["early_backward_recompute"],
                      "throughput_vs_stored": sec / results["early_backward_recompute"],
                      "memory_vs_stored": peak_bytes["early_backward_recompute"] / peak_bytes["early_backward"],
                      "memory_vs_gpipe_order": peak_bytes["early_backward_recompute"] / peak_bytes["gpipe"]},
        "hip_graph_replay": None if args.no_graph else
        {"samples_per_s": M * cfg.micro_batch / results["graph"], "ms_per_step": results["graph"] * 1e3,
         "note": "one hipGraphLaunch per iteration (one backward lane inside the graph)"},
        "apply_adam": {"ms": apply_ms, "params": int(r.sizes.n_params), "bytes": int(apply_bytes),
                       "GB/s": apply_bytes / (apply_ms * 1e-3) / 1e9, "hbm_peak_frac": apply_bytes / (apply_ms * 1e-3) / 8e12},
        "kernel_classes": classes,
    }
    if not args.no_pipeline and not cfg.has_embedding and not cfg.has_mlm_head:
        out["pipeline_on_partitions"] = pipeline_study(cfg, seed)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, seed, min(4, M), 2)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
