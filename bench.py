#!/usr/bin/env python3
"""Benchmark of the GSWA hot path on one MI355X.

A step is one pass of the whole hot path over one synthetic batch.  The default workload is the
largest of the benchmark's configurations, the deep-feature stack (c4): 36 consecutive GSWA
layers (shifts alternating 0/4, independently seeded weights), forward through all of them and
backward through all of them, bf16 storage with fp32 accumulation, B=32, 64x64 map, C=180,
6 heads in 2 groups, window 8.  Inputs are resident in HBM before the timed region.  Prints one
JSON line; `by_workload` carries the remaining benchmark configurations (c2 and c3 at every
group count, the two large-image inference shapes), each with its own roofline entry and CPU
baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--groups G] [--workload c2|c3|c4|c5_m8|c5_m16|agile_h4_qk16|agile_h4_qk32|agile_h6_qk24|agile_infer|astl_c2|astl_agile|astl_c3]
"""
import argparse
import json
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0

# HBM bytes per launch of a workload's dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# (profiles/wide_layers_hbm_counters.txt, profiles/fused_kernels_c2_groups2_hbm_counters.txt; mean over
# the launch kinds of that kernel), valid only for the kernel source they were taken on:
# {(workload, groups, kernel): (source file, sha256 of it, bytes per launch)}
MEASURED_TRAFFIC = {
    ("c4", 2, "wide_attn_bwd"): ("wide_bwd.hip", "9049b09287411286713757e150239f25eb4b0fc83b84015ac04c6c9f78170307", 229576312),
    ("c3", 2, "wide_attn_bwd"): ("wide_bwd.hip", "9049b09287411286713757e150239f25eb4b0fc83b84015ac04c6c9f78170307", 116065640),
    ("c2", 2, "fused_bwd"): ("fused_bwd.hip", "8aefb5890a71d6f6e8172a7992c221f0116de8d79eace3ae9662cfa534bd9b74", 74163908),
    ("c5_m8", 2, "fused_fwd"): ("wide_fwd.hip", "2741dc20c76eea55b1b9254b569d5d7423fdfab82ee26444cc861f11740d1a99", 225001912),
    ("c5_m16", 2, "fused_attn_fwd"): ("fused_fwd.hip", "fb20eb1f46acd89fc3898bd81bb6dcaaef9a8566d74eb9b3c773e5ab64968f98", 181130520),
}


def measured_traffic(workload, groups, kernel):
    import hashlib
    import os
    entry = MEASURED_TRAFFIC.get((workload, groups, kernel))
    if not entry:
        return None
    src = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2409_06206_amd", "csrc", entry[0])
    if not os.path.exists(src):
        return None
    digest = hashlib.sha256(open(src, "rb").read()).hexdigest()
    return entry[2] if digest == entry[1] else None


FLAGS = 0  # extra descriptor flags for every layer (--force-staged)
BATCH = 0  # batch size override (--batch); 0 = the workload's own
CHECKPOINT_EVERY = 0  # layers per recomputed block of a stack workload (--checkpoint-every)
BAND_WINDOWS = 0      # window rows per band of a forward-only stack workload (--band-windows)


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
                               flags=FLAGS, dqk=cfg.get("dqk", 0), band_windows=BAND_WINDOWS,
                               inference_only=bool(cfg.get("forward_only")))
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


def time_steps(layers, steps, warmup, backward=True, want_median=False):
    """Seconds per step over exactly `steps` steps between two synchronisations (wall clock), and
    the median of the per-step durations taken from events recorded on the launch stream."""
    import torch
    for _ in range(warmup):
        step(layers, backward)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        step(layers, backward)
        ev[i + 1].record()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / steps
    if not want_median:
        return sec
    per = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
    return sec, 1e-3 * per[len(per) // 2]


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


def cpu_baseline(name, groups, min_seconds=4.0, max_reps=20, batch=None, n_layers=None, threads=None,
                 backward=True):
    """The CPU oracle, as it stands, on a bounded sample of the workload: the first `n_layers` layers
    (default: all) at batch `batch` (default: the workload's).  Windows are independent and every
    window costs the same, so the oracle's time is linear in the number of windows and layers; a
    sample is therefore stated in tokens/s, the unit of the GPU figure."""
    from oracle import gswa_oracle
    from paper_2409_06206_amd import synth
    cfg = dict(synth.CONFIGS[name])
    if BATCH:
        cfg["B"] = BATCH
    full_B, full_layers = cfg["B"], len(cfg["layers"])
    if batch:
        cfg["B"] = min(batch, cfg["B"])
    shifts = list(cfg["layers"])[:n_layers or None]
    x, dy = synth.activations(cfg["B"], cfg["H"], cfg["W"], cfg["C"], synth.ACT_SEED)
    x = synth.quantize(x, cfg["dtype"])
    dy = synth.quantize(dy, cfg["dtype"])
    dqk = cfg.get("dqk", 0)
    kw = dict(heads=cfg["heads"], groups=groups, window=cfg["window"], dqk=dqk)
    if cfg.get("block"):
        return cpu_baseline_block(name, cfg, groups, x, dy, min_seconds, max_reps)
    params = []
    for li in range(len(shifts)):
        p = synth.layer_params(cfg["C"], cfg["heads"], groups, cfg["window"], synth.LAYER_SEED0 + li,
                               dqk=dqk)
        p = {k: synth.quantize(v, cfg["dtype"]) for k, v in p.items()}
        params.append((p["w_qkv"], p["b_qkv"], p["w_proj"], p["b_proj"], p["table"]))
    all_threads = gswa_oracle.threads()
    if threads:
        gswa_oracle.set_threads(threads)
    try:
        reps, t0 = 0, time.perf_counter()
        while reps < max_reps and (reps == 0 or time.perf_counter() - t0 < min_seconds):
            acts = [x]
            for a, s in zip(params, shifts):
                # a stack of bare attention layers is chained as the GPU harness chains it
                acts.append(gswa_oracle.forward(acts[-1], *a, shift=s, **kw))
            if backward:
                g = dy
                for a, s, xin in zip(reversed(params), reversed(shifts), reversed(acts[:-1])):
                    g = gswa_oracle.backward(xin, g, *a, shift=s, **kw)[0]
            reps += 1
        dt = (time.perf_counter() - t0) / reps
        used = gswa_oracle.threads()
    finally:
        if threads:
            gswa_oracle.set_threads(all_threads)
    tokens = cfg["B"] * cfg["H"] * cfg["W"] * len(shifts)
    what = "full" if (cfg["B"] == full_B and len(shifts) == full_layers) else "sample of"
    return {"value": tokens / dt, "unit": "tokens/s", "cores": used, "kind": "oracle",
            "sample": f"{what} {name}: {len(shifts)} of {full_layers} layer(s) at B={cfg['B']} of {full_B}, "
                      f"{'fwd+bwd' if backward else 'forward only'}, fp64 C oracle with OpenMP, {reps} repetition(s), "
                      f"{dt:.2f} s each; the oracle's time is linear in windows and layers, so tokens/s carries over "
                      f"to the full workload"}


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


def is_forward_only(name):
    from paper_2409_06206_amd import synth
    return name.startswith("c5") or bool(synth.CONFIGS[name].get("forward_only"))


def workload_text(name, cfg, groups, n_layers, backward):
    return (f"{name}: {n_layers} {'whole (LN, GSWA, MLP, skips)' if cfg.get('block') else 'GSWA'} layer(s), "
            f"shifts {list(cfg['layers'])[:4]}{'...' if n_layers > 4 else ''}"
            f"{' one stack call per pass, shifts 0/%d alternating, checkpoint_every=%d' % (cfg['stack_shift'], CHECKPOINT_EVERY) if cfg.get('stack') else ''}"
            f"{' in bands of %d window rows' % BAND_WINDOWS if cfg.get('stack') and BAND_WINDOWS else ''}, "
            f"{'fwd+bwd' if backward else 'forward only'}, "
            f"B={cfg['B']} {cfg['H']}x{cfg['W']} C={cfg['C']} heads={cfg['heads']} "
            f"window={cfg['window']} groups={groups}"
            f"{' q/k channels per head=%d' % cfg['dqk'] if cfg.get('dqk') else ''}")


def measure(name, groups, steps, warmup, profile_n=20, graph=False):
    """Times one workload: wall-clock mean over exactly `steps` steps, the median step from events,
    per-kernel event averages, and the roofline entry of the kernel with the largest total time."""
    import torch
    backward = not is_forward_only(name)
    cfg, layers = build_case(name, groups)
    T = cfg["B"] * cfg["H"] * cfg["W"]
    n_layers = cfg.get("stack") or len(layers)
    tokens = T * n_layers
    sec, med = time_steps(layers, steps, warmup, backward, want_median=True)
    graph_sec = time_graph_replays(layers, steps, warmup, backward) if graph else None
    prof, prof_wall = profile_steps(layers, min(steps, profile_n), backward)
    dom = max(prof, key=lambda k: prof[k]["total_ms_per_step"])
    dom_bytes = algorithmic_bytes_per_launch(dom, cfg, prof[dom]["launches_per_step"] / n_layers, backward)
    achieved = dom_bytes / (prof[dom]["avg_us"] * 1e-6) / 1e9
    roofline = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                "traffic": measured_traffic(name, groups, dom),
                "avg_launch_us": prof[dom]["avg_us"], "algorithmic_bytes_per_launch": dom_bytes}
    e = 2 if cfg["dtype"] == "bf16" else 4
    # whole layers keep two [T, C] tensors for the backward pass instead of one
    per_token = (9 if backward else 2) if cfg.get("block") else (7 if backward else 2)
    step_bytes = per_token * cfg["C"] * e * tokens
    step_flops = model_flops_per_token(cfg, groups, backward) * tokens
    L0 = layers[0]
    res = {
        "cfg": cfg, "layers": layers, "backward": backward, "n_layers": n_layers, "tokens": tokens,
        "sec": sec, "median_sec": med, "roofline": roofline, "kernels": prof,
        "whole_step": {"algorithmic_GBps": step_bytes / sec / 1e9, "hbm_frac": step_bytes / sec / 1e9 / HBM_PEAK_GBS,
                       "model_TFLOPs": step_flops / sec / 1e12,
                       "mfma_frac": step_flops / sec / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                       "profiled_ms_per_step": 1e3 * prof_wall,
                       "graph_ms_per_step": None if graph_sec is None else 1e3 * graph_sec},
        "saved_bytes_per_layer": L0.saved_bytes,
        "workspace_bytes": max(L0.fwd_ws_bytes, L0.bwd_ws_bytes),
        "peak_saved_act_bytes": L0.saved_bytes + max(L0.fwd_ws_bytes, L0.bwd_ws_bytes),
    }
    return res


# CPU-baseline samples of the benchmark workloads: (batch, layers) of the slice the oracle is timed on
CPU_SAMPLE = {"c2": (None, None), "c3": (None, None), "c4": (2, 4), "c5_m8": (None, None), "c5_m16": (None, None)}


def other_workloads(headline, steps, warmup, want_cpu):
    """Every benchmark configuration other than the headline, each at every group count it names:
    ms per step (median of `steps` timed steps after `warmup`), tokens/s, the roofline entry of its
    dominant kernel, the bytes the library asks for, and the CPU oracle on a bounded sample."""
    import torch
    out = {}
    for name in ("c2", "c3", "c4", "c5_m8", "c5_m16"):
        if name == headline:
            continue
        for G in synth_groups(name):
            n_steps = steps if name != "c4" else max(10, steps // 5)
            r = measure(name, G, n_steps, warmup, profile_n=10)
            entry = {"workload": workload_text(name, r["cfg"], G, r["n_layers"], r["backward"]),
                     "ms_per_step": 1e3 * r["median_sec"], "mean_ms_per_step": 1e3 * r["sec"],
                     "tokens_per_s": r["tokens"] / r["median_sec"], "steps": n_steps, "warmup": warmup,
                     "roofline": r["roofline"], "whole_step": r["whole_step"],
                     "kernels_avg_us": {k: round(v["avg_us"], 2) for k, v in r["kernels"].items()},
                     "saved_bytes_per_layer": r["saved_bytes_per_layer"], "workspace_bytes": r["workspace_bytes"],
                     "peak_saved_act_bytes": r["peak_saved_act_bytes"]}
            if want_cpu and G == (2 if 2 in synth_groups(name) else synth_groups(name)[0]):
                b, nl = CPU_SAMPLE[name]
                entry["cpu_baseline"] = cpu_baseline(name, G, min_seconds=2.0, max_reps=5, batch=b, n_layers=nl,
                                                     backward=r["backward"])
            out[f"{name}_g{G}"] = entry
            del r
            torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--groups", type=int, default=2)
    ap.add_argument("--workload", default="c4", choices=["c2", "c3", "c4", "c5_m8", "c5_m16", "agile_h4_qk16", "agile_h4_qk32", "agile_h6_qk24", "agile_infer",
                                                              "astl_c2", "astl_agile", "astl_c3", "astl_infer", "astl_stack36",
                                                              "astl_agile_stack36", "astl_infer_stack6", "astl_infer_stack6_2k"],
                    help="c4 (the 36-layer stack, the largest benchmark configuration) is the headline; a default "
                         "run also carries c2, c3 and c5_* in by_workload (c5_*: forward only)")
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
    ap.add_argument("--band-windows", type=int, default=0,
                    help="forward-only stack workloads: inference band by band, this many window rows per band "
                         "(0 = the whole map per layer call)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-group-sweep", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="leave out by_workload (the benchmark configurations other than --workload)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after the run, copy a 128 MiB tensor three times (known-size reference "
                         "dispatch for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)")

    import torch
    from paper_2409_06206_amd import gswa
    gswa.lib()
    global FLAGS, BATCH, CHECKPOINT_EVERY, BAND_WINDOWS
    CHECKPOINT_EVERY = max(0, args.checkpoint_every)
    BAND_WINDOWS = max(0, args.band_windows)
    if args.force_staged:
        FLAGS = gswa.GSWA_FORCE_STAGED
    BATCH = max(0, args.batch)
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    if args.groups not in synth_groups(args.workload):
        sys.exit(f"groups={args.groups} is not one of the benchmark's values for {args.workload}")
    r = measure(args.workload, args.groups, args.steps, args.warmup, graph=args.graph)
    cfg, layers, backward, sec = r["cfg"], r["layers"], r["backward"], r["sec"]
    n_layers, tokens_per_step = r["n_layers"], r["tokens"]

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
        "warmup": args.warmup, "ms_per_step": 1e3 * sec, "median_ms_per_step": 1e3 * r["median_sec"],
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": workload_text(args.workload, cfg, args.groups, n_layers, backward),
                   "groups": args.groups, "tokens_per_step": tokens_per_step},
        "roofline": r["roofline"],
        "whole_step": r["whole_step"],
        "kernels": r["kernels"],
        "saved_bytes_per_layer": r["saved_bytes_per_layer"],
        "workspace_bytes": r["workspace_bytes"],
        "peak_saved_act_bytes": r["peak_saved_act_bytes"],
        "peak_bytes_whole_workload": (n_layers * r["saved_bytes_per_layer"] + r["workspace_bytes"])
                                     if not cfg.get("stack") else r["peak_saved_act_bytes"],
        "by_groups": sweep,
    }
    if args.calibration_copy:
        a = torch.empty(32 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
    del r, layers
    torch.cuda.empty_cache()
    want_cpu = not args.no_cpu_baseline
    plain = args.workload in CPU_SAMPLE
    if want_cpu and not cfg.get("stack") and (plain or (backward and (args.workload.startswith("agile") or cfg.get("block")))):
        b, nl = CPU_SAMPLE.get(args.workload, (None, None))
        out["cpu_baseline"] = cpu_baseline(args.workload, args.groups, batch=b, n_layers=nl, backward=backward)
        if plain:
            # the same sample on one thread, so that the per-core rate is visible
            one = cpu_baseline(args.workload, args.groups, min_seconds=0.0, max_reps=1, batch=1 if b else 2,
                               n_layers=2, threads=1, backward=backward)
            out["cpu_baseline"]["single_thread"] = {"value": one["value"], "unit": one["unit"], "cores": one["cores"],
                                                    "sample": one["sample"]}
    if plain and not args.no_other_workloads and not BATCH and not FLAGS:
        out["by_workload"] = other_workloads(args.workload, 50, 10, want_cpu)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
