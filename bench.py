"""Benchmark of the stage hot path on one MI355X.

A step = stage_zero_grads + stage_run_schedule(M, K, early-backward) over one batch
of synthetic micro-batches already resident in HBM, + stream sync.  Workload: the
BERT-Large-shaped stage (6 layers, hidden 1024, 16 heads, FFN 4096, seq 512,
micro-batch 4, M = 8, K = 4, bf16 storage with fp32 accumulation).

Prints one JSON line: stage samples/s (value: K back-to-back steps between two
synchronisations; beside it the median of individually synchronised steps), algorithmic
TFLOP/s and its fraction of the bf16 MFMA peak, peak activation bytes for K-slot
early-backward against M-slot GPipe order, the roofline of the dominant kernel (the MFMA
GEMM) and a per-kernel table, both timed with HIP events around every launch in a separate
pass that runs the same steps on ONE stream (no kernel of another stream shares the
compute units, so a kernel's time is its own), the other named stage configurations, and
the CPU oracle timed on the same workload.

`--serial` runs only the one-stream iteration (what the per-kernel table times), for a
profiler: `rocprofv3 --kernel-trace --stats -- python3 bench.py --serial --steps 5`.
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

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E

# HBM-side bytes per gemm_mfma_kernel launch (average over the 528 launches of a step), from the
# rocprofv3 FETCH_SIZE / WRITE_SIZE passes summarised in profiles/gemm_mfma_bert_large_pmc_traffic.md,
# each counter scaled by what it reads for the library's copy kernel of known size.  Counters cannot
# be read from inside this process, so the figure is carried here per workload, with the commit of
# the library it was measured on: it is a record of that build, not a live measurement.
GEMM_TRAFFIC = {"bert_large": {"bytes_per_launch": 66187701,
                               "source": "profiles/gemm_mfma_bert_large_pmc_traffic.md", "library_commit": "e1f1768"}}


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
    what = "the whole iteration" if M_sample == cfg.M else f"{M_sample} of the {cfg.M} micro-batches"
    return {"value": M_sample * cfg.micro_batch / dt, "unit": "samples/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{what} of the same stage (M={M_sample}, K={K_sample}, early-backward order), float64 numpy, "
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


def make_io(r, cfg, mbs, M):
    import numpy as np
    import torch
    T, H = cfg.tokens, cfg.hidden
    emb, head = cfg.has_embedding, cfg.has_mlm_head
    xs = [r.to_dev(mb["ids"].reshape(T).astype(np.int32)) if emb else r.to_dev(mb["x"].reshape(T, H)) for mb in mbs]
    dys = None if head else [r.to_dev(mb["dy"].reshape(T, H)) for mb in mbs]
    auxs = [r.to_dev(mb["targets"].reshape(T).astype(np.int32)) for mb in mbs] if head else None
    ys = [torch.zeros(1, dtype=torch.float32, device="cuda") if head else r.empty_act() for _ in range(M)]
    dxs = None if emb else [r.empty_act() for _ in range(M)]
    ptr = lambda ts: None if ts is None else [t.data_ptr() for t in ts]
    return (xs, dys, ys, dxs, auxs), (ptr(xs), ptr(dys), ptr(ys), ptr(dxs), ptr(auxs))


def time_iteration(cfg, theta, mbs, order, slots, flags, steps, warmup, synced=0, keep=False):
    """Mean seconds per step over `steps` back-to-back steps between two synchronisations; median of
    `synced` individually synchronised steps (None if 0); peak activation bytes; the runner if keep."""
    import numpy as np
    import torch
    from paper_2007_01045_amd import binding as B
    M, K = cfg.M, cfg.K
    r = B.StageRunner(B.config_for(cfg, slots, flags=flags, loss_scale=1.0 / (M * cfg.tokens)), theta)
    bufs, (px, pdy, py, pdx, paux) = make_io(r, cfg, mbs, M)

    def step():
        B.stage_zero_grads(r.h)
        B.stage_run_schedule(r.h, M, K, order, px, pdy, py, pdx, paux)

    for _ in range(warmup):
        step()
    B.stage_sync(r.h)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    B.stage_sync(r.h)
    torch.cuda.synchronize()
    mean = (time.perf_counter() - t0) / steps
    med = None
    if synced:
        ts = []
        for _ in range(synced):
            t0 = time.perf_counter()
            step()
            B.stage_sync(r.h)
            torch.cuda.synchronize()
            ts.append(time.perf_counter() - t0)
        med = float(np.median(ts))
    peak = int(B.stage_stats(r.h).peak_activation_bytes)
    if keep:
        return mean, med, peak, (r, step, bufs)
    del bufs
    r.close()
    del r
    torch.cuda.empty_cache()
    return mean, med, peak, None


def algorithmic_bytes(cls, cfg):
    """HBM bytes one launch of an HBM-bound kernel class has to move (unit = T*H elements)."""
    T, H = cfg.tokens, cfg.hidden
    e = 2 if cfg.dtype == "bf16" else 4
    u = T * H
    if cls == "ln_fwd":     # reads the fp32 pre-LN sum, writes y (and its fp32 copy for the next residual add) + stats
        return u * (4 + e + 4) + 8 * T if cfg.dtype == "bf16" else u * 8 + 8 * T
    if cls == "ln_bwd":     # reads dy and the pre-LN sum, writes dz and one partial-sum triple per block of 8 rows
        return u * (e + 4 + e) + ((T + 7) // 8) * 3 * H * 4 if cfg.dtype == "bf16" else u * 12 + ((T + 7) // 8) * 3 * H * 4
    return None


def serial_kernel_table(cfg, theta, mbs, steps):
    """The iteration on ONE stream with HIP events around every launch: per (class, shape) the launches per step,
    the average duration alone, and its fraction of the roofline that bounds it."""
    from paper_2007_01045_amd import binding as B
    mean, _, _, (r, step, bufs) = time_iteration(cfg, theta, mbs, B.ORDER_EARLY_BACKWARD, cfg.K, B.FLAG_ONE_STREAM,
                                                 steps, 2, keep=True)
    B.stage_profile_enable(r.h, True)
    for _ in range(steps):
        step()
    recs = B.stage_profile_launches(r.h)
    B.stage_profile_read(r.h)
    B.stage_profile_enable(r.h, False)
    r.close()
    groups = {}
    for x in recs:
        key = (x["cls"], x["M"], x["N"], x["K"], x["batch"])
        g = groups.setdefault(key, [0, 0.0, 0.0])
        g[0] += 1
        g[1] += x["ms"]
        g[2] += x["flops"]
    table = []
    for (cls, Mm, N, Kk, batch), (n, ms, fl) in sorted(groups.items(), key=lambda kv: -kv[1][1]):
        us = ms / n * 1e3
        row = {"class": cls, "launches_per_step": n / steps, "avg_us": us, "ms_per_step": ms / steps}
        if Mm:
            row["shape"] = f"{batch}x[{Mm}x{N}x{Kk}]" if batch > 1 else f"{Mm}x{N}x{Kk}"
        if fl > 0:
            row.update(gflop_per_launch=fl / n / 1e9, tflops=fl / (ms * 1e-3) / 1e12,
                       frac_of_mfma_peak=fl / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS)
        else:
            by = algorithmic_bytes(cls, cfg)
            if by:
                row.update(mbytes_per_launch=by / 1e6, gbs=by / (us * 1e-6) / 1e9,
                           frac_of_hbm_peak=by / (us * 1e-6) / 1e9 / PEAK_HBM_GBS)
        table.append(row)
    gem = [x for x in recs if x["cls"].startswith("gemm")]
    g_ms, g_fl = sum(x["ms"] for x in gem), sum(x["flops"] for x in gem)
    return {"ms_per_step_one_stream": mean * 1e3, "table": table,
            "gemm": {"launches_per_step": len(gem) / steps, "avg_launch_us": g_ms * 1e3 / max(len(gem), 1),
                     "tflops": g_fl / (g_ms * 1e-3) / 1e12 if g_ms > 0 else 0.0}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="bert_large")
    ap.add_argument("--serial", action="store_true", help="only the one-stream iteration with the per-kernel table")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-pipeline", action="store_true")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true")
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
    M, K = cfg.M, cfg.K
    theta = I.make_params(cfg, seed)
    mbs = [I.make_microbatch(cfg, seed, m) for m in range(M)]
    name = (f"{cfg.name}: L={cfg.n_layers} H={cfg.hidden} A={cfg.n_heads} F={cfg.ffn} s={cfg.seq} "
            f"b={cfg.micro_batch} M={M} K={K}")

    if args.serial:
        out = serial_kernel_table(cfg, theta, mbs, min(args.steps, 5))
        out["config"] = {"workload": name + ", early-backward order, one stream", "seed": seed}
        print(json.dumps(out))
        return

    # GPipe order with M slots; early-backward order with K slots with re-computation (a resident micro-batch
    # keeps its input only and the backward task re-runs the forward); early-backward order with K slots
    sec_gp, _, peak_gp, _ = time_iteration(cfg, theta, mbs, B.ORDER_GPIPE, M, 0, args.steps, args.warmup)
    sec_rc, _, peak_rc, _ = time_iteration(cfg, theta, mbs, B.ORDER_EARLY_BACKWARD, K, B.FLAG_RECOMPUTE, args.steps,
                                           args.warmup)
    sec, med, peak_eb, (r, step, bufs) = time_iteration(cfg, theta, mbs, B.ORDER_EARLY_BACKWARD, K, 0, args.steps,
                                                        args.warmup, synced=max(10, min(args.steps, 20)), keep=True)

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
    n_params = int(r.sizes.n_params)
    apply_bytes = n_params * (16 + 12 + 4 + (2 if cfg.dtype == "bf16" else 4))
    del bufs, step
    r.close()
    del r
    torch.cuda.empty_cache()

    # the early-backward iteration again as ONE HIP graph (captured once on a stream of its own, then
    # replayed): what is left when the host issues one launch per iteration instead of one per kernel
    sec_graph = None
    if not args.no_graph:
        with torch.cuda.stream(torch.cuda.Stream()):
            rg = B.StageRunner(B.config_for(cfg, K, loss_scale=1.0 / (M * cfg.tokens)), theta)
            gbufs, gp = make_io(rg, cfg, mbs, M)
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
            sec_graph = (time.perf_counter() - t0) / args.steps
            del gbufs
            rg.close()
            del rg
        torch.cuda.empty_cache()

    # per-kernel times: the same iteration on one stream with HIP events around every launch
    serial = serial_kernel_table(cfg, theta, mbs, min(args.steps, 5))
    torch.cuda.empty_cache()
    achieved = serial["gemm"]["tflops"]
    classes = {}
    for row in serial["table"]:
        c = classes.setdefault(row["class"], {"launches_per_step": 0.0, "ms_per_step": 0.0})
        c["launches_per_step"] += row["launches_per_step"]
        c["ms_per_step"] += row["ms_per_step"]

    flops = stage_flops(cfg, M)
    samples = M * cfg.micro_batch
    traffic = GEMM_TRAFFIC.get(cfg.name)
    out = {
        "metric": "stage samples/sec + MFMA util (%) + peak activation bytes vs GPipe order",
        "value": samples / sec, "unit": "samples/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": name + ", early-backward order", "seed": seed},
        "ms_per_step_median_synced": med * 1e3,
        "tflops_algorithmic": flops / sec / 1e12,
        "mfma_peak_frac_algorithmic": flops / sec / 1e12 / PEAK_BF16_TFLOPS,
        "gpipe_order": {"samples_per_s": samples / sec_gp, "ms_per_step": sec_gp * 1e3,
                        "note": "the same tasks, all forwards listed before all backwards: no backward may start "
                                "before the last forward has finished, so forwards never run beside backwards; the "
                                "difference to the early-backward figure is this executor's overlap, not a property "
                                "of the schedules (on one stage both do the same work)"},
        "peak_activation_bytes": {"early_backward_K_slots": peak_eb, "gpipe_M_slots": peak_gp,
                                  "ratio": peak_eb / peak_gp},
        "roofline": {"bound": "mfma", "kernel": "gemm_mfma_kernel (all linear-layer products: fwd, dgrad, wgrad)",
                     "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS,
                     "traffic": traffic["bytes_per_launch"] if traffic else None,
                     "traffic_source": (f"{traffic['source']}, measured on the library at commit "
                                        f"{traffic['library_commit']}") if traffic else None,
                     "launches_per_step": serial["gemm"]["launches_per_step"],
                     "avg_launch_us": serial["gemm"]["avg_launch_us"],
                     "timed": "HIP events around every launch of the iteration run on ONE stream (no kernel of "
                              "another stream on the compute units); `value` is the four-stream iteration"},
        "recompute": {"samples_per_s": samples / sec_rc, "ms_per_step": sec_rc * 1e3,
                      "peak_activation_bytes": peak_rc, "throughput_vs_stored": sec / sec_rc,
                      "memory_vs_stored": peak_rc / peak_eb, "memory_vs_gpipe_order": peak_rc / peak_gp},
        "hip_graph_replay": None if sec_graph is None else
        {"samples_per_s": samples / sec_graph, "ms_per_step": sec_graph * 1e3,
         "note": "one hipGraphLaunch per iteration (one backward lane inside the graph)"},
        "apply_adam": {"ms": apply_ms, "params": n_params, "bytes": int(apply_bytes),
                       "GB/s": apply_bytes / (apply_ms * 1e-3) / 1e9, "hbm_peak_frac": apply_bytes / (apply_ms * 1e-3) / 8e12},
        "one_stream": {"ms_per_step": serial["ms_per_step_one_stream"], "kernel_classes": classes,
                       "kernels": serial["table"]},
    }
    if not args.no_other_workloads and cfg.name == "bert_large":
        others = {}
        for wl in ("bert48_quarter", "first_stage", "last_stage"):
            c2 = I.CONFIGS[wl]
            th2 = I.make_params(c2, seed)
            mb2 = [I.make_microbatch(c2, seed, m) for m in range(c2.M)]
            s2, _, pk2, _ = time_iteration(c2, th2, mb2, B.ORDER_EARLY_BACKWARD, c2.K, 0, 10, 2)
            # GPipe order's peak is M slots of the same size: stated from the slot size, not run (M = 32 slots of
            # the last stage would need no more than 17 GB, but timing it adds nothing to the memory figure)
            slot = pk2 // c2.K
            others[wl] = {"workload": f"L={c2.n_layers} H={c2.hidden} F={c2.ffn} s={c2.seq} b={c2.micro_batch} "
                                      f"M={c2.M} K={c2.K}" + (" +embeddings" if c2.has_embedding else "") +
                                      (" +MLM head" if c2.has_mlm_head else ""),
                          "samples_per_s": c2.M * c2.micro_batch / s2, "ms_per_step": s2 * 1e3,
                          "tflops_algorithmic": stage_flops(c2, c2.M) / s2 / 1e12,
                          "mfma_peak_frac_algorithmic": stage_flops(c2, c2.M) / s2 / 1e12 / PEAK_BF16_TFLOPS,
                          "peak_activation_bytes": pk2, "peak_vs_gpipe_order_M_slots": pk2 / (slot * c2.M)}
            del th2, mb2
            torch.cuda.empty_cache()
        out["other_workloads"] = others
    if not args.no_pipeline and not cfg.has_embedding and not cfg.has_mlm_head:
        out["pipeline_on_partitions"] = pipeline_study(cfg, seed)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, seed, M, K)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
