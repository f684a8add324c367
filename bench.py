#!/usr/bin/env python3
"""Benchmark of the convolution hot path on one MI355X.

A step is one forward+backward pass of the five-convolution stack (conv1..conv5
with ReLU / max-pool glue) over one synthetic mini-batch shard of N samples,
N = 128 by default: the per-GPU share of the paper's two-GPU data-parallel run.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--batch N]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3      # MI355X dense fp32 matrix peak (published)


def cpu_baseline(threads_hint=None, budget_images=None):
    """Time the CPU oracle, as it stands, on a bounded sample of the same stack:
    every conv pass of the step at the real layer shapes, on a few images."""
    import numpy as np
    import oracle
    from paper_1312_5853_amd import synth
    from paper_1312_5853_amd.stack import conv_flops

    threads = oracle.num_threads()
    n = budget_images or max(1, min(4 * threads, 64))      # about 10-30 s of oracle time
    Ls = synth.LAYERS
    flops = 0.0
    t0 = time.perf_counter()
    for name, passes, reps in (("conv1", ("f", "w"), 1), ("conv2", ("f", "d", "w"), 2),
                               ("conv3", ("f", "d", "w"), 1), ("conv4", ("f", "d", "w"), 1),
                               ("conv5", ("f", "d", "w"), 1)):
        L = Ls[name]
        x, w, dy = synth.layer_tensors(name, n)
        x, w, dy = x.astype(np.float64), w.astype(np.float64), dy.astype(np.float64)
        for _ in range(reps):
            if "f" in passes:
                oracle.conv_fwd(x, w, L["stride"], L["pad"])
            if "d" in passes:
                oracle.conv_bwd_data(dy, w, L["H"], L["W"], L["stride"], L["pad"])
            if "w" in passes:
                oracle.conv_bwd_filter(x, dy, L["R"], L["S"], L["stride"], L["pad"])
            flops += len(passes) * conv_flops(n, L)
    dt = time.perf_counter() - t0
    return {
        "value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
        "sample": "all 16 conv passes of one stack step at the real layer shapes on %d images "
                  "(%.1f GFLOP, %.1f s, input generation included)" % (n, flops / 1e9, dt),
        "seconds": dt,
    }


PEAK_BF16_MFMA_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak (published)


def bf16_layers(N, hp, synth, conv_flops, torch, reps=10):
    """Per-pass timings of conv3..conv5 with bf16 inputs and fp32 accumulation/output (HIP events)."""
    out = {}
    for layer in ("conv3", "conv4", "conv5"):
        L = synth.LAYERS[layer]
        x, w, dy = (torch.from_numpy(synth.to_bf16_grid(a)).cuda().to(torch.bfloat16)
                    for a in synth.layer_tensors(layer, N))
        y = torch.empty(dy.shape, device="cuda")
        dx = torch.empty(x.shape, device="cuda")
        dw = torch.empty(w.shape, device="cuda")
        calls = {
            "fwd": lambda: hp.conv_fwd(x, w, L["stride"], L["pad"], y=y),
            "dgrad": lambda: hp.conv_bwd_data(dy, w, L["H"], L["W"], L["stride"], L["pad"], dx=dx),
            "wgrad": lambda: hp.conv_bwd_filter(x, dy, L["R"], L["S"], L["stride"], L["pad"], dw=dw),
        }
        for name, fn in calls.items():
            for _ in range(3):
                fn()
            s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            s.record()
            for _ in range(reps):
                fn()
            e.record()
            torch.cuda.synchronize()
            ms = s.elapsed_time(e) / reps
            tf = conv_flops(N, L) / ms / 1e9
            out["%s.%s" % (layer, name)] = {"ms": round(ms, 4), "tflops": round(tf, 1),
                                            "frac_bf16_peak": round(tf / PEAK_BF16_MFMA_TFLOPS, 4)}
    return out


def two_column_layers(N, hp, synth, conv_flops, torch, reps=10):
    """conv4 / conv5 as the paper's two model-parallel columns without cross-connection (groups = 2: 192 -> 192 and
    192 -> 128 per column), fp32, per-pass timings of the grouped calls (HIP events)."""
    out = {}
    for layer in ("conv4", "conv5"):
        L = synth.LAYERS[layer]
        x, w, dy = (torch.from_numpy(a).cuda() for a in synth.layer_tensors(layer, N))
        w = w[:, :L["C"] // 2].contiguous()                      # [K, C/2, R, S]: each filter reads its column only
        y, dx, dw = torch.empty_like(dy), torch.empty_like(x), torch.empty_like(w)
        calls = {
            "fwd": lambda: hp.conv_fwd_grouped(x, w, L["stride"], L["pad"], 2, y=y),
            "dgrad": lambda: hp.conv_bwd_data_grouped(dy, w, L["H"], L["W"], L["stride"], L["pad"], 2, dx=dx),
            "wgrad": lambda: hp.conv_bwd_filter_grouped(x, dy, L["R"], L["S"], L["stride"], L["pad"], 2, dw=dw),
        }
        for name, fn in calls.items():
            for _ in range(3):
                fn()
            s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            s.record()
            for _ in range(reps):
                fn()
            e.record()
            torch.cuda.synchronize()
            ms = s.elapsed_time(e) / reps
            tf = conv_flops(N, L) / 2 / ms / 1e9                 # half the multiply-adds of the full-width layer
            out["%s.%s" % (layer, name)] = {"ms": round(ms, 4), "tflops": round(tf, 1),
                                            "frac_peak": round(tf / PEAK_FP32_MFMA_TFLOPS, 4)}
    return out


PEAK_HBM_TBS = 8.0                 # MI355X HBM3E peak (published)


def whole_network(N, hp, torch, steps):
    """The fully connected layers (fp32 MFMA GEMMs), the SGD update, and one whole training step of the network on
    one shard (conv stack + fc6-fc8 + update): per-call timings with HIP events and the step's wall time."""
    from paper_1312_5853_amd.stack import FullNetwork, FC_LAYERS, fc_flops, stack_flops
    net = FullNetwork(N)
    out = {}

    def timed(fn, reps=10):
        for _ in range(3):
            fn()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        for _ in range(reps):
            fn()
        e.record()
        torch.cuda.synchronize()
        return s.elapsed_time(e) / reps

    net.forward()
    for idx, (name, i, o) in enumerate(FC_LAYERS):
        x = net.a5.view(N, -1) if idx == 0 else net.fc_y[FC_LAYERS[idx - 1][0]]
        w, b, dy = net.fc_w[name], net.fc_b[name], torch.randn((N, o), device="cuda")
        dx = torch.empty((N, i), device="cuda")
        calls = {"fwd": lambda: hp.fc_fwd(x, w, b, relu=True, y=net.fc_y[name], ws=net.ws),
                 "dgrad": lambda: hp.fc_bwd_data(dy, w, dx=dx, ws=net.ws),
                 "wgrad": lambda: hp.fc_bwd_filter(x, dy, dw=net.fc_dw[name], ws=net.ws)}
        for pname, fn in calls.items():
            ms = timed(fn)
            tf = 2.0 * N * i * o / ms / 1e9
            out["%s.%s" % (name, pname)] = {"ms": round(ms, 4), "tflops": round(tf, 1),
                                            "frac_peak": round(tf / PEAK_FP32_MFMA_TFLOPS, 4)}
    nparam = sum(p.numel() for p, _ in net.params)
    ms = timed(net.update)
    out["sgd_update"] = {"ms": round(ms, 4), "params": nparam, "launches": len(net.params),
                         "hbm_tb_per_s": round(nparam * 20 / ms / 1e9, 3),       # w, dw, v read; w, v written
                         "frac_hbm_peak": round(nparam * 20 / ms / 1e9 / PEAK_HBM_TBS, 4)}
    for _ in range(3):
        net.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        net.step()
    torch.cuda.synchronize()
    step_ms = (time.perf_counter() - t0) * 1e3 / steps
    gf = (stack_flops(N) + fc_flops(N)) / 1e9
    out["step"] = {"ms": round(step_ms, 4), "images_per_s": round(N / step_ms * 1e3, 1), "gflop": round(gf, 2),
                   "tflops": round(gf / step_ms, 2),
                   "what": "conv1-5 + glue, fc6-fc8 with bias/ReLU, SGD update with momentum and weight decay; "
                           "seeded gradient instead of a loss, no dropout / response normalisation"}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=128)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stack-only", action="store_true",
                    help="only the fp32 stack step (no two-column, bf16 or CPU blocks): the run the profiles are taken on")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build targets one GPU (one data-parallel shard / one model-parallel "
                 "column per call); --gpus %d is not supported, run with --gpus 1" % args.gpus)

    import torch
    from paper_1312_5853_amd import binding as hp
    from paper_1312_5853_amd import build as hp_build
    from paper_1312_5853_amd.stack import ConvStack, stack_flops, conv_flops
    from paper_1312_5853_amd import synth

    if not os.path.exists(hp.LIB_PATH):
        hp_build.build()
    hp.lib()
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")

    N = args.batch
    stack = ConvStack(N)
    flops = stack_flops(N)

    for _ in range(args.warmup):
        stack.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        stack.step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # the same step replayed from a HIP graph (no per-call host work): K replays
    graph_ms = None
    try:
        graph = stack.capture()
        for _ in range(2):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        del graph
    except RuntimeError as e:           # an extra figure only: the headline numbers do not depend on it
        sys.stderr.write("bench.py: HIP graph replay skipped (%s)\n" % e)
        torch.cuda.synchronize()

    # second timed region: HIP events (on the launch stream) around every conv call
    stack.timers = {}
    acc = {}
    reps = max(3, min(args.steps, 10))
    for _ in range(reps):
        stack.step()
        torch.cuda.synchronize()
        for key, (s, e) in stack.timers.items():
            acc[key] = acc.get(key, 0.0) + s.elapsed_time(e)
    stack.timers = None
    per_pass = {}
    conv_ms = 0.0
    def pass_flops(layer):
        """Nominal FLOPs of one pass of a stack layer (conv2 = both model-parallel columns in one grouped call)."""
        return conv_flops(N, synth.LAYERS[layer]) * (2 if layer == "conv2" else 1)

    for (layer, p), tot in sorted(acc.items()):
        ms = tot / reps
        f = pass_flops(layer)
        conv_ms += ms
        per_pass["%s.%s" % (layer, p)] = {"ms": round(ms, 4), "tflops": round(f / ms / 1e9, 2),
                                           "frac_peak": round(f / ms / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4)}

    # dominant kernel: the 128x128-tile implicit-GEMM kernel that runs forward of conv2 (both columns in one
    # launch), conv3, conv4, conv5 and backward-data of conv3, conv4, conv5 (7 launches per step)
    dom_keys = [k for k in acc if k[1] in ("fwd", "dgrad") and k[0] != "conv1"]
    dom_keys = [k for k in dom_keys if not (k[0] == "conv2" and k[1] == "dgrad")]
    dom_flops = sum(pass_flops(k[0]) for k in dom_keys)
    dom_ms = sum(acc[k] for k in dom_keys) / reps
    achieved = dom_flops / dom_ms / 1e9
    roofline = {
        "bound": "mfma", "kernel": "colgemm_fast_kernel<2,2,2,2,16> (fwd of conv2-5, dgrad of conv3-5)",
        "achieved": round(achieved, 2), "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
        "frac": round(achieved / PEAK_FP32_MFMA_TFLOPS, 4),
        # HBM bytes per launch of this kernel from rocprofv3 FETCH_SIZE (x2.00) + WRITE_SIZE (x1.00), factors from a
        # 256 MiB copy; collected offline (profiles/stack_n128_fp32_hbm_traffic.txt), valid for the default N = 128
        "traffic": 140.4e6 if N == 128 else None,
        "launches_per_step": len(dom_keys), "avg_launch_ms": round(dom_ms / len(dom_keys), 4),
        "flops_per_launch": dom_flops / len(dom_keys),
    }

    def bf16_block():
        out = bf16_layers(N, hp, synth, conv_flops, torch)
        # the same step with bf16 tensors end to end (fp32 accumulation, fp32 filter gradients)
        bstack = ConvStack(N, dtype="bf16")
        for _ in range(3):
            bstack.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            bstack.step()
        torch.cuda.synchronize()
        bf16_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        out["stack_ms_per_step"] = round(bf16_ms, 4)
        out["stack_tflops"] = round(flops / bf16_ms / 1e9, 2)
        return out

    def extra(fn):
        """The blocks beside the headline step: a failure in one of them is reported in its place."""
        try:
            return fn()
        except Exception as e:          # noqa: BLE001 - the headline figures above stand on their own
            torch.cuda.synchronize()
            return {"error": "%s: %s" % (type(e).__name__, e)}

    columns, bf16, network = None, None, None
    if not args.stack_only:
        del stack
        network = extra(lambda: whole_network(N, hp, torch, args.steps))
        columns = extra(lambda: two_column_layers(N, hp, synth, conv_flops, torch))
        bf16 = extra(bf16_block)

    value = flops / ms_per_step / 1e9
    out = {
        "metric": "conv-stack TFLOP/s at N=%d (conv1-5 fwd+dgrad+wgrad, fp32 MFMA, ReLU/pool glue in the step)" % N,
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "5-conv AlexNet stack fwd+bwd, N=%d, fp32 (conv2 as two model-parallel columns)" % N,
                   "batch": N, "conv_gflop_per_step": round(flops / 1e9, 2)},
        "frac_fp32_mfma_peak": round(value / PEAK_FP32_MFMA_TFLOPS, 4),
        "hip_graph_ms_per_step": None if graph_ms is None else round(graph_ms, 4),
        "conv_only_ms": round(conv_ms, 4),
        "conv_only_frac_peak": round(flops / conv_ms / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4),
        "per_pass": per_pass,
        "roofline": roofline,
        "two_column_conv4_conv5_fp32": columns,
        "bf16_in_fp32_acc": bf16,
        "whole_network_fp32": network,
        "context": "paper: 10.5 days per 100 epochs on one NVIDIA TITAN at batch 256 (whole network with data "
                   "loading: about 141 images/s; context for whole_network_fp32.step, not for value)",
    }
    if not args.no_cpu_baseline and not args.stack_only:
        out["cpu_baseline"] = extra(cpu_baseline)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
