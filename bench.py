#!/usr/bin/env python3
"""Benchmark of the GSWA hot path on one MI355X.

A step is one pass of the whole hot path over one synthetic batch of the lightweight-SR
shape: two consecutive GSWA layers (shift 0, then shift 4), forward and backward, bf16
storage with fp32 accumulation, B=32, 64x64 map, C=60, 6 heads, window 8.  Inputs are
resident in HBM before the timed region.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--groups G] [--workload c2|c3|c4|c5_m8|c5_m16|agile_h4_qk16|agile_h4_qk32|agile_h6_qk24|agile_infer|astl_c2|astl_agile|astl_c3]
"""
import argparse
import json
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0

# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# (profiles/fused_kernels_c2_groups2_hbm_counters.txt), valid only for the kernel source they
# were taken on: {(workload, groups, kernel): (sha256 of the kernel source, bytes per launch)}
MEASURED_TRAFFIC = {
    ("c2", 2, "fused_bwd"): ("543025eaca5637d323d8b5d5adeea5f256205d5adcce7374e0e0048c8723f94e", 77146317),
}


def measured_traffic(workload, groups, kernel):
    import hashlib
    import os
    entry = MEASURED_TRAFFIC.get((workload, groups, kernel))
    if not entry or not entry[0]:
        return None
    src = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2409_06206_amd", "csrc",
                       kernel + ".hip")
    if not os.path.exists(src):
        return None
    digest = hashlib.sha256(open(src, "rb").read()).hexdigest()
    return entry[1] if digest == entry[0] else None


FLAGS = 0  # extra descriptor flags for every layer (--force-staged)
BATCH = 0  # batch size override (--batch); 0 = the workload's own
CHECKPOINT_EVERY = 0  # layers per recomputed block of a stack workload (--checkpoint-every)


def build_case(name, groups):
    import torch
    from paper_2409_06206_amd import runner, synth
    cfg = dict(synth.CONFIGS[name])
    if BATCH:
        cfg["B"] = BATCH
    x, dy = synth.activations(cfg["B"], cfg["H"], cfg["W"], cfg["C"], synth.ACT_SEED)
    layers = []
    if cfg.get("stack"):
        # one call runs the whole sequence of layers (alternating shift) in each direction
        S = runner.DeviceStack(cfg["B"], cfg["H"], cfg["W"], cfg["C"], cfg["heads"], groups, cfg["window"],
                               cfg["stack_shift"], cfg["dtype"], cfg["hidden"], cfg["stack"], CHECKPOINT_EVERY,
                               flags=FLAGS, dqk=cfg.get("dqk", 0))
        S.set_params([synth.astl_params(cfg["C"], cfg["heads"], groups, cfg["window"], cfg["hidden"],
                                        synth.LAYER_SEED0 + li, dqk=cfg.get("dqk", 0)) for li in range(cfg["stack"])])
        S.set_inputs(x, dy)
        torch.cuda.synchronize()
        return cfg, [S]
    for li, shift in enumerate(cfg["layers"]):
        if cfg.get("block"):
            L = runner.DeviceBlock(cfg["B"], cfg["H"], cfg["W"], cfg["C"], cfg["heads"], groups, cfg["window"],
                                   shift, cfg["dtype"], cfg["hidden"], flags=FLAGS, dqk=cfg.get("dqk", 0))
            L.set_params(synth.astl_params(cfg["C"], cfg["heads"], groups, cfg["window"], cfg["hidden"],
                                           synth.LAYER_SEED0 + li, dqk=cfg.get("dqk", 0)))
        else:
            L = runner.DeviceLayer(cfg["B"], cfg["H"], cfg["W"], cfg["C"], cfg["heads"], groups,
                                   cfg["window"], shift, cfg["dtype"], FLAGS, dqk=cfg.get("dqk", 0))
            L.set_params(synth.layer_params(cfg["C"], cfg["heads"], groups, cfg["window"],
                                            synth.LAYER_SEED0 + li, dqk=cfg.get("dqk", 0)))
        layers.append(L)
    layers[0].set_inputs(x)
    layers[-1].dy = runner.to_device(dy, cfg["dtype"])
    # chain: layer l+1 reads layer l's y; layer l's dy is layer l+1's dx
    for a, b in zip(layers[:-1], layers[1:]):
        b.x = a.y
        a.dy = b.dx
    torch.cuda.synchronize()
    return cfg, layers


def step(layers, backward=True):
    for L in layers:
        L.forward(keep=backward)
    if backward:
        for L in reversed(layers):
            L.backward()


def time_steps(layers, steps, warmup, backward=True):
    import torch
    for _ in range(warmup):
        step(layers, backward)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step(layers, backward)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def time_graph_replays(layers, steps, warmup, backward=True):
    """The same step captured once into a HIP graph (every launch of the library goes to the stream
    it is given, nothing allocates or synchronises) and replayed: launch cost leaves the host."""
    import torch
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(layers, backward)          # first calls set kernel attributes: not capturable
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(layers, backward)
    for _ in range(warmup):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def profile_steps(layers, steps, backward=True):
    """Per-kernel average durations from HIP events recorded on the launch stream."""
    import torch
    from paper_2409_06206_amd import gswa
    gswa.gswa_profile_enable(True)
    gswa.gswa_profile_collect()
    t0 = time.perf_counter()
    per = {}
    for _ in range(steps):
        step(layers, backward)
        res, dropped = gswa.gswa_profile_collect()   # waits for the step's events
        assert dropped == 0
        for k, (ms, n) in res.items():
            a = per.setdefault(k, [0.0, 0])
            a[0] += ms
            a[1] += n
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps
    gswa.gswa_profile_enable(False)
    return {k: {"total_ms_per_step": v[0] / steps, "launches_per_step": v[1] / steps,
                "avg_us": 1e3 * v[0] / v[1]} for k, v in per.items()}, wall


FORWARD_KERNELS = {"qkv_linear", "attn_fwd", "attn_core_fwd", "window_fwd", "proj_linear", "fused_fwd", "fused_attn_fwd", "proj_gemm",
                   "pack_fwd", "mlp_fwd", "fc1_linear", "fc2_linear", "gelu_fwd"}


def algorithmic_bytes_per_launch(kernel, cfg, launches_per_layer, training=True):
    """Bytes the METHOD has to move for the work one launch of `kernel` covers.

    Per token the layer must read x and write y in forward (2*C*e), write one saved [T,C]
    tensor when training, and in backward read x, dy and the saved tensor and write dx
    (4*C*e); weights are negligible.  A kernel that is launched n times per layer and pass
    (once per head group or head chunk) is charged 1/n of the pass per launch.
    """
    T = cfg["B"] * cfg["H"] * cfg["W"]
    e = 2 if cfg["dtype"] == "bf16" else 4
    fwd = (3 if training else 2) * cfg["C"] * e * T
    bwd = 4 * cfg["C"] * e * T
    return (fwd if kernel in FORWARD_KERNELS else bwd) / max(launches_per_layer, 1.0)


def synth_groups(name):
    from paper_2409_06206_amd import synth
    return synth.CONFIGS[name]["groups"]


def model_flops_per_token(cfg, groups, backward=True):
    C, N, heads = cfg["C"], cfg["window"] ** 2, cfg["heads"]
    qk = heads * (cfg.get("dqk", 0) or C // heads)       # channels of q (and of k) over all heads
    fwd = 2 * (C / groups) * (2 * qk + C) + 2 * N * (qk + C) + 2 * C * C
    if cfg.get("block"):
        fwd += 4 * C * cfg["hidden"]     # the two fully connected layers of Eq. 5
    return (3 if backward else 1) * fwd


def cpu_baseline(name, groups, min_seconds=10.0, max_reps=60):
    """The CPU oracle, as it stands, on the same layer pair."""
    from oracle import gswa_oracle
    from paper_2409_06206_amd import synth
    cfg = dict(synth.CONFIGS[name])
    if BATCH:
        cfg["B"] = BATCH
    x, dy = synth.activations(cfg["B"], cfg["H"], cfg["W"], cfg["C"], synth.ACT_SEED)
    x = synth.quantize(x, cfg["dtype"])
    dy = synth.quantize(dy, cfg["dtype"])
    dqk = cfg.get("dqk", 0)
    kw = dict(heads=cfg["heads"], groups=groups, window=cfg["window"], dqk=dqk)
    params = []
    for li in range(len(cfg["layers"])):
        p = synth.layer_params(cfg["C"], cfg["heads"], groups, cfg["window"], synth.LAYER_SEED0 + li,
                               dqk=dqk)
        p = {k: synth.quantize(v, cfg["dtype"]) for k, v in p.items()}
        params.append((p["w_qkv"], p["b_qkv"], p["w_proj"], p["b_proj"], p["table"]))
    if cfg.get("block"):
        return cpu_baseline_block(name, cfg, groups, x, dy, min_seconds, max_reps)
    reps, t0 = 0, time.perf_counter()
    while reps < max_reps and (reps == 0 or time.perf_counter() - t0 < min_seconds):
        acts = [x]
        for a, s in zip(params, cfg["layers"]):
            acts.append(gswa_oracle.forward(acts[-1], *a, shift=s, **kw))
        g = dy
        for a, s, xin in zip(reversed(params), reversed(cfg["layers"]), reversed(acts[:-1])):
            g = gswa_oracle.backward(xin, g, *a, shift=s, **kw)[0]
        reps += 1
    dt = (time.perf_counter() - t0) / reps
    tokens = cfg["B"] * cfg["H"] * cfg["W"] * len(cfg["layers"])
    return {"value": tokens / dt, "unit": "tokens/s", "cores": gswa_oracle.threads(), "kind": "oracle",
            "sample": f"full {name} layer pair (B={cfg['B']}), fwd+bwd, fp64 C oracle with OpenMP, "
                      f"{reps} repetition(s), {dt:.2f} s each"}


def cpu_baseline_block(name, cfg, groups, x, dy, min_seconds, max_reps):
    """The whole-layer CPU oracle (numpy fp64 around the C attention oracle) on the same layer pair."""
    from oracle import astl_oracle, gswa_oracle
    from paper_2409_06206_amd import synth
    dqk = cfg.get("dqk", 0)
    kw = dict(heads=cfg["heads"], groups=groups, window=cfg["window"], dqk=dqk)
    params = []
    for li in range(len(cfg["layers"])):
        p = synth.astl_params(cfg["C"], cfg["heads"], groups, cfg["window"], cfg["hidden"],
                              synth.LAYER_SEED0 + li, dqk=dqk)
        params.append({k: synth.quantize(v, cfg["dtype"]) for k, v in p.items()})
    reps, t0 = 0, time.perf_counter()
    while reps < max_reps and (reps == 0 or time.perf_counter() - t0 < min_seconds):
        acts = [x]
        for p, s in zip(params, cfg["layers"]):
            acts.append(astl_oracle.forward(acts[-1], p, shift=s, **kw))
        g = dy
        for p, s, xin in zip(reversed(params), reversed(cfg["layers"]), reversed(acts[:-1])):
            g = astl_oracle.backward(xin, g, p, shift=s, **kw)[0]
        reps += 1
    dt = (time.perf_counter() - t0) / reps
    tokens = cfg["B"] * cfg["H"] * cfg["W"] * len(cfg["layers"])
    return {"value": tokens / dt, "unit": "tokens/s", "cores": gswa_oracle.threads(), "kind": "oracle",
            "sample": f"full {name} layer pair (B={cfg['B']}), fwd+bwd, fp64 oracle (numpy around the C "
                      f"attention oracle with OpenMP), {reps} repetition(s), {dt:.2f} s each"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--groups", type=int, default=2)
    ap.add_argument("--workload", default="c2", choices=["c2", "c3", "c4", "c5_m8", "c5_m16", "agile_h4_qk16", "agile_h4_qk32", "agile_h6_qk24", "agile_infer",
                                                              "astl_c2", "astl_agile", "astl_c3", "astl_infer", "astl_stack36",
                                                              "astl_agile_stack36"],
                    help="c2 is the benchmark line; the others are the remaining benchmark shapes "
                         "(c5_*: forward only)")
    ap.add_argument("--batch", type=int, default=0,
                    help="batch size other than the workload's own (a different workload: say so when quoting it)")
    ap.add_argument("--force-staged", action="store_true",
                    help="time the one-kernel-per-step path where a fused kernel exists")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step captured into one HIP graph and replayed (reported as "
                         "whole_step.graph_ms_per_step; `value` stays the eager figure)")
    ap.add_argument("--checkpoint-every", type=int, default=0,
                    help="stack workloads: keep only every k-th layer input and recompute blocks of k layers "
                         "in the backward pass (0 = keep everything)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-group-sweep", action="store_true")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after the run, copy a 128 MiB tensor three times (known-size reference "
                         "dispatch for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)")

    import torch
    from paper_2409_06206_amd import gswa
    gswa.lib()
    global FLAGS, BATCH, CHECKPOINT_EVERY
    CHECKPOINT_EVERY = max(0, args.checkpoint_every)
    if args.force_staged:
        FLAGS = gswa.GSWA_FORCE_STAGED
    BATCH = max(0, args.batch)
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    from paper_2409_06206_amd import synth as _synth
    backward = not (args.workload.startswith("c5") or _synth.CONFIGS[args.workload].get("forward_only"))
    if args.groups not in synth_groups(args.workload):
        sys.exit(f"groups={args.groups} is not one of the benchmark's values for {args.workload}")
    cfg, layers = build_case(args.workload, args.groups)
    T = cfg["B"] * cfg["H"] * cfg["W"]
    n_layers = cfg.get("stack") or len(layers)
    tokens_per_step = T * n_layers
    sec = time_steps(layers, args.steps, args.warmup, backward)

    graph_sec = time_graph_replays(layers, args.steps, args.warmup, backward) if args.graph else None
    prof, prof_wall = profile_steps(layers, min(args.steps, 20), backward)
    dom = max(prof, key=lambda k: prof[k]["total_ms_per_step"])
    dom_bytes = algorithmic_bytes_per_launch(dom, cfg, prof[dom]["launches_per_step"] / n_layers, backward)
    dom_s = prof[dom]["avg_us"] * 1e-6
    achieved = dom_bytes / dom_s / 1e9
    roofline = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                "traffic": measured_traffic(args.workload, args.groups, dom),
                "avg_launch_us": prof[dom]["avg_us"], "algorithmic_bytes_per_launch": dom_bytes}
    e = 2 if cfg["dtype"] == "bf16" else 4
    # whole layers keep two [T, C] tensors for the backward pass instead of one
    per_token = (9 if backward else 2) if cfg.get("block") else (7 if backward else 2)
    step_bytes = per_token * cfg["C"] * e * tokens_per_step
    step_flops = model_flops_per_token(cfg, args.groups, backward) * tokens_per_step

    sweep = {}
    if not args.no_group_sweep and not cfg.get("stack"):
        for G in cfg["groups"]:
            if G == args.groups:
                ls, s_ = layers, sec
            else:
                _, ls = build_case(args.workload, G)
                s_ = time_steps(ls, max(5, args.steps // 5), 3, backward)
            L0 = ls[0]
            sweep[str(G)] = {"tokens_per_s": tokens_per_step / s_, "ms_per_step": 1e3 * s_,
                             "saved_bytes_per_layer": L0.saved_bytes,
                             "workspace_bytes": max(L0.fwd_ws_bytes, L0.bwd_ws_bytes),
                             "peak_saved_act_bytes": L0.saved_bytes + max(L0.fwd_ws_bytes, L0.bwd_ws_bytes)}
            if ls is not layers:
                del ls
                torch.cuda.empty_cache()

    out = {
        "metric": "GSWA fwd+bwd tokens/sec (1 GPU); % of HBM/MFMA roofline; peak saved-act bytes",
        "value": tokens_per_step / sec, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": 1e3 * sec, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": f"{args.workload}: {n_layers} {'whole (LN, GSWA, MLP, skips)' if cfg.get('block') else 'GSWA'} layer(s), shifts {list(cfg['layers'])[:4]}"
                               f"{'...' if len(layers) > 4 else ''}"
                               f"{' one stack call per pass, shifts 0/%d alternating, checkpoint_every=%d' % (cfg['stack_shift'], CHECKPOINT_EVERY) if cfg.get('stack') else ''}, "
                               f"{'fwd+bwd' if backward else 'forward only'}, "
                               f"B={cfg['B']} {cfg['H']}x{cfg['W']} C={cfg['C']} heads={cfg['heads']} "
                               f"window={cfg['window']} groups={args.groups}"
                               f"{' q/k channels per head=%d' % cfg['dqk'] if cfg.get('dqk') else ''}",
                   "groups": args.groups, "tokens_per_step": tokens_per_step},
        "roofline": roofline,
        "whole_step": {"algorithmic_GBps": step_bytes / sec / 1e9, "hbm_frac": step_bytes / sec / 1e9 / HBM_PEAK_GBS,
                       "model_TFLOPs": step_flops / sec / 1e12,
                       "mfma_frac": step_flops / sec / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                       "profiled_ms_per_step": 1e3 * prof_wall,
                       "graph_ms_per_step": None if graph_sec is None else 1e3 * graph_sec},
        "kernels": prof,
        "peak_saved_act_bytes": layers[0].saved_bytes + max(layers[0].fwd_ws_bytes, layers[0].bwd_ws_bytes),
        "by_groups": sweep,
    }
    if args.calibration_copy:
        a = torch.empty(32 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline and backward and (args.workload == "c2" or args.workload.startswith("agile") or cfg.get("block")) and not cfg.get("stack"):
        out["cpu_baseline"] = cpu_baseline(args.workload, args.groups)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
