#!/usr/bin/env python3
"""Benchmark of the convolution hot path on one MI355X.

A step is one forward+backward pass of the five-convolution stack (conv1..conv5
with ReLU / max-pool glue) over one synthetic mini-batch shard of N samples,
N = 128 by default: the per-GPU share of the paper's two-GPU data-parallel run.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--batch N]

Beside the headline (K wall-clock-timed steps) the line carries, all from this
one run: per-pass figures of the step (median and minimum of 50 event-timed
launches after 10 warm-ups), the per-configuration figures of the workload list
(`per_config`), the register-resident MFMA rate this GPU sustains
(`mfma_ceiling_tflops`, a second denominator next to the published peak), and the
CPU oracle timed on the host cores (`cpu_baseline`).  Any block that fails makes
the exit status non-zero.
"""
import argparse
import json
import os
import re
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3      # MI355X dense fp32 matrix peak (published)
PEAK_BF16_MFMA_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak (published)
PEAK_HBM_TBS = 8.0                 # MI355X HBM3E peak (published)
TIMED_LAUNCHES = 50                # per-pass protocol: 10 warm-ups, then the median / minimum of 50 launches
WARMUP_LAUNCHES = 10


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def mfma_ceiling():
    """The stand-alone register-resident fp32 MFMA loop (built next to the library): what the matrix cores of this
    GPU sustain with no memory traffic.  Runs as a child process, before this process touches the GPU."""
    exe = os.path.join(ROOT, "paper_1312_5853_amd", "mfma_ceiling")
    res = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    if res.returncode != 0:
        raise RuntimeError("mfma_ceiling failed: %s" % res.stderr.strip())
    out = {}
    for line in res.stdout.splitlines():
        m = re.match(r"(burst|sustained|bf16_sustained_random_operands|bf16_sustained_constant_operands)\s.*"
                     r"TFLOP/s=([0-9.]+)", line)
        if m:
            out[m.group(1)] = float(m.group(2))
        m = re.match(r"rate_(\S+)\s+bytes_per_clk_per_cu=([0-9.]+)", line)
        if m:
            out.setdefault("bytes_per_clk_per_cu", {})[m.group(1)] = float(m.group(2))
    if "sustained" not in out:
        raise RuntimeError("mfma_ceiling printed no figure: %r" % res.stdout)
    return out


def cpu_baseline(N):
    """The CPU oracle, as it stands, on the same workload as the GPU step: every conv pass of one stack step at the
    real layer shapes on N images (fewer on a host with few threads, so that it stays within about half a minute)."""
    import numpy as np
    import oracle
    from paper_1312_5853_amd import synth
    from paper_1312_5853_amd.stack import conv_flops

    threads = oracle.num_threads()
    n = max(1, min(N, 8 * threads))
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
        "sample": "all 16 conv passes of one stack step at the real layer shapes on %d images%s "
                  "(%.1f GFLOP, %.1f s, input generation included)"
                  % (n, "" if n == N else " (the GPU step runs on %d)" % N, flops / 1e9, dt),
        "seconds": dt, "cpu_model": cpu_model(),
    }


def tiny_oracle_seconds():
    """Workload 0 (the small 5x5 layer): the oracle's three passes in seconds, single-threaded and on all threads."""
    import numpy as np
    import oracle
    from paper_1312_5853_amd import synth
    L = synth.LAYERS["tiny"]
    x, w, dy = (a.astype(np.float64) for a in synth.layer_tensors("tiny", 4))
    all_threads = oracle.num_threads()
    out = {}
    for label, threads in (("oracle_seconds_1_thread", 1), ("oracle_seconds_all_threads", all_threads)):
        oracle.set_num_threads(threads)
        best = None
        for _ in range(3):
            t0 = time.perf_counter()
            oracle.conv_fwd(x, w, L["stride"], L["pad"])
            oracle.conv_bwd_data(dy, w, L["H"], L["W"], L["stride"], L["pad"])
            oracle.conv_bwd_filter(x, dy, L["R"], L["S"], L["stride"], L["pad"])
            dt = time.perf_counter() - t0
            best = dt if best is None else min(best, dt)
        out[label] = round(best, 6)
    oracle.set_num_threads(all_threads)
    out["threads"] = all_threads
    out["cpu_model"] = cpu_model()
    return out


class Timer:
    """Per-launch time of `fn`: WARMUP_LAUNCHES untimed launches, then TIMED_LAUNCHES samples; a sample is GROUP
    launches back to back between one pair of HIP events on torch's current stream (the stream the binding launches
    on), divided by GROUP -- an event pair costs several microseconds of idle GPU, which single-launch samples would
    add to calls of 50-100 us.  Reports the median and the minimum of the samples."""
    GROUP = 4

    def __init__(self, torch):
        self.torch = torch

    def __call__(self, fn, reps=TIMED_LAUNCHES, warmup=WARMUP_LAUNCHES):
        torch = self.torch
        for _ in range(warmup):
            fn()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for s, e in ev:
            s.record()
            for _ in range(self.GROUP):
                fn()
            e.record()
        torch.cuda.synchronize()
        ms = sorted(s.elapsed_time(e) / self.GROUP for s, e in ev)
        return {"ms": round(ms[len(ms) // 2], 4), "ms_min": round(ms[0], 4)}


def with_rates(t, flops, peak, key="frac_peak"):
    tf = flops / t["ms"] / 1e9
    t["tflops"] = round(tf, 1)
    t[key] = round(tf / peak, 4)
    return t


def layer_passes(layer, N, dtype, passes, hp, synth, conv_flops, torch, timer):
    """One layer of the workload list as single calls (dense tensors): dtype "f32", or "bf16" = bf16 inputs with
    fp32 accumulation and fp32 outputs."""
    L = synth.LAYERS[layer]
    x, w, dy = synth.layer_tensors(layer, N)
    if dtype == "bf16":
        x, w, dy = (hp.convert_f32_to_bf16(torch.from_numpy(a).cuda()) for a in (x, w, dy))
        peak, key = PEAK_BF16_MFMA_TFLOPS, "frac_bf16_peak"
    else:
        x, w, dy = (torch.from_numpy(a).cuda() for a in (x, w, dy))
        peak, key = PEAK_FP32_MFMA_TFLOPS, "frac_peak"
    y = torch.empty(dy.shape, device="cuda")
    dx = torch.empty(x.shape, device="cuda")
    dw = torch.empty(w.shape, device="cuda")
    calls = {
        "fwd": lambda: hp.conv_fwd(x, w, L["stride"], L["pad"], y=y),
        "dgrad": lambda: hp.conv_bwd_data(dy, w, L["H"], L["W"], L["stride"], L["pad"], dx=dx),
        "wgrad": lambda: hp.conv_bwd_filter(x, dy, L["R"], L["S"], L["stride"], L["pad"], dw=dw),
    }
    return {p: with_rates(timer(calls[p]), conv_flops(N, L), peak, key) for p in passes}


def two_column_layers(N, hp, synth, conv_flops, torch, timer):
    """conv4 / conv5 as the paper's two model-parallel columns without cross-connection (groups = 2: 192 -> 192 and
    192 -> 128 per column), fp32, per-pass timings of the grouped calls."""
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
            # half the multiply-adds of the full-width layer
            out["%s.%s" % (layer, name)] = with_rates(timer(fn), conv_flops(N, L) / 2, PEAK_FP32_MFMA_TFLOPS)
    return out


def stack_ms(N, dtype, steps, torch, ConvStack):
    """Wall-clock ms per step of the stack at batch N (3 warm-up steps, `steps` timed)."""
    st = ConvStack(N, dtype=dtype)
    for _ in range(3):
        st.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        st.step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def whole_network(N, hp, torch, steps, timer):
    """The fully connected layers (fp32 MFMA GEMMs), the SGD update, and one whole training step of the network on
    one shard (conv stack + fc6-fc8 + update): per-call timings with HIP events and the step's wall time."""
    from paper_1312_5853_amd.stack import FullNetwork, FC_LAYERS, fc_flops, stack_flops
    net = FullNetwork(N)
    out = {}
    net.forward()
    for idx, (name, i, o) in enumerate(FC_LAYERS):
        x = net.a5.view(N, -1) if idx == 0 else net.fc_y[FC_LAYERS[idx - 1][0]]
        w, b, dy = net.fc_w[name], net.fc_b[name], torch.randn((N, o), device="cuda")
        dx = torch.empty((N, i), device="cuda")
        calls = {"fwd": lambda: hp.fc_fwd(x, w, b, relu=True, y=net.fc_y[name], ws=net.ws),
                 "dgrad": lambda: hp.fc_bwd_data(dy, w, dx=dx, ws=net.ws),
                 "wgrad": lambda: hp.fc_bwd_filter(x, dy, dw=net.fc_dw[name], ws=net.ws)}
        for pname, fn in calls.items():
            out["%s.%s" % (name, pname)] = with_rates(timer(fn), 2.0 * N * i * o, PEAK_FP32_MFMA_TFLOPS)
    nparam = sum(p.numel() for p, _ in net.params)
    t = timer(net.update)
    t.update({"params": nparam, "tensors": len(net.params), "launches": 1,
              "hbm_tb_per_s": round(nparam * 20 / t["ms"] / 1e9, 3),       # w, dw, v read; w, v written
              "frac_hbm_peak": round(nparam * 20 / t["ms"] / 1e9 / PEAK_HBM_TBS, 4)})
    out["sgd_update"] = t
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


def traffic_from_profile(N):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary (FETCH_SIZE x2.00 +
    WRITE_SIZE x1.00, factors from a 256 MiB copy; taken at the default N = 128): counters cannot be read inside
    this run, so the figure is the profile's, named here with its file."""
    if N != 128:
        return None
    path = os.path.join(ROOT, "profiles", "stack_n128_fp32_hbm_traffic.txt")
    try:
        m = re.search(r"dominant kernel: ([0-9.]+) MB per launch", open(path).read())
    except OSError:
        return None
    return float(m.group(1)) * 1e6 if m else None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=128)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stack-dtype", choices=("f32", "bf16"), default="f32",
                    help="with --stack-only: element type of the profiled step (bf16 = bf16 tensors end to end); the "
                         "default run always reports the fp32 step as `value`")
    ap.add_argument("--stack-only", action="store_true",
                    help="only the fp32 stack step (no per-config, two-column, bf16 or CPU blocks): the run the "
                         "profiles are taken on")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build targets one GPU (one data-parallel shard / one model-parallel "
                 "column per call); --gpus %d is not supported, run with --gpus 1" % args.gpus)

    from paper_1312_5853_amd import build as hp_build
    from paper_1312_5853_amd import binding as hp
    if not os.path.exists(hp.LIB_PATH):
        hp_build.build()

    failures = []
    torch = None                        # imported below, after the child process of the ceiling probe has run

    def extra(name, fn):
        """The blocks beside the headline step: a failure is reported in the block's place and fails the run."""
        try:
            return fn()
        except Exception as e:          # noqa: BLE001 - reported, and the exit status says so
            failures.append(name)
            try:
                torch.cuda.synchronize()
            except Exception:           # noqa: BLE001
                pass
            return {"error": "%s: %s" % (type(e).__name__, e)}

    # before this process initialises the GPU: the MFMA ceiling probe runs as a child process
    ceiling = None
    if not args.stack_only:
        ceiling = extra("mfma_ceiling", mfma_ceiling)

    import torch
    from paper_1312_5853_amd.stack import ConvStack, stack_flops, conv_flops
    from paper_1312_5853_amd import synth

    hp.lib()
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    timer = Timer(torch)

    N = args.batch
    if args.stack_dtype != "f32" and not args.stack_only:
        sys.exit("bench.py: --stack-dtype is a profiling option of --stack-only")
    stack = ConvStack(N, dtype=args.stack_dtype)
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

    # second timed region: HIP events (on the launch stream) around every conv call of the step, one sample per
    # step and call; the step has been warm for args.warmup + args.steps steps by now
    stack.timers = {}
    samples = {}
    reps = TIMED_LAUNCHES if not args.stack_only else max(3, min(args.steps, 10))
    for _ in range(reps):
        stack.step()
        torch.cuda.synchronize()
        for key, (s, e) in stack.timers.items():
            samples.setdefault(key, []).append(s.elapsed_time(e))
    stack.timers = None

    def pass_flops(layer):
        """Nominal FLOPs of one pass of a stack layer (conv2 = both model-parallel columns in one grouped call)."""
        return conv_flops(N, synth.LAYERS[layer]) * (2 if layer == "conv2" else 1)

    per_pass = {}
    conv_ms = 0.0
    med = {}
    for (layer, p), vals in sorted(samples.items()):
        vals = sorted(vals)
        med[(layer, p)] = vals[len(vals) // 2]
        conv_ms += med[(layer, p)]
        per_pass["%s.%s" % (layer, p)] = with_rates({"ms": round(med[(layer, p)], 4), "ms_min": round(vals[0], 4)},
                                                    pass_flops(layer),
                                                    PEAK_BF16_MFMA_TFLOPS if args.stack_dtype == "bf16"
                                                    else PEAK_FP32_MFMA_TFLOPS)

    # dominant kernel.  fp32: the 128x128-tile implicit-GEMM kernel that runs forward of conv2 (both columns in one
    # launch), conv3, conv4, conv5 and backward-data of conv3, conv4, conv5 (7 launches per step).  bf16 profiling
    # run: the direct-to-LDS kernel (forward and backward-data of conv3, conv4, conv5; 6 launches per step).
    bf16_run = args.stack_dtype == "bf16"
    dom_keys = [k for k in samples if k[1] in ("fwd", "dgrad") and k[0] != "conv1"]
    dom_keys = [k for k in dom_keys if not (k[0] == "conv2" and (k[1] == "dgrad" or bf16_run))]
    dom_flops = sum(pass_flops(k[0]) for k in dom_keys)
    dom_ms = sum(sum(samples[k]) for k in dom_keys) / reps          # mean launch duration over the timed region
    achieved = dom_flops / dom_ms / 1e9
    peak = PEAK_BF16_MFMA_TFLOPS if bf16_run else PEAK_FP32_MFMA_TFLOPS
    roofline = {
        "bound": "mfma",
        "kernel": ("colgemm_bf16_dma_kernel (fwd and dgrad of conv3-5)" if bf16_run else
                   "colgemm_fast_kernel<2,2,2,2,16> (fwd of conv2-5, dgrad of conv3-5)"),
        "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
        "frac": round(achieved / peak, 4),
        "traffic": None if bf16_run else traffic_from_profile(N),
        "traffic_source": "profiles/stack_n128_fp32_hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)",
        "launches_per_step": len(dom_keys), "avg_launch_ms": round(dom_ms / len(dom_keys), 4),
        "flops_per_launch": dom_flops / len(dom_keys), "timed_launches_each": reps,
    }
    if isinstance(ceiling, dict) and "sustained" in ceiling and not bf16_run:
        roofline["frac_of_measured_mfma_ceiling"] = round(achieved / ceiling["sustained"], 4)

    def bf16_block():
        out = {}
        for layer in ("conv3", "conv4", "conv5"):
            for p, t in layer_passes(layer, N, "bf16", ("fwd", "dgrad", "wgrad"), hp, synth, conv_flops, torch,
                                     timer).items():
                out["%s.%s" % (layer, p)] = t
        # the same step with bf16 tensors end to end (fp32 accumulation, fp32 filter gradients)
        bf16_ms = stack_ms(N, "bf16", args.steps, torch, ConvStack)
        out["stack_ms_per_step"] = round(bf16_ms, 4)
        out["stack_tflops"] = round(flops / bf16_ms / 1e9, 2)
        out["stack_frac_bf16_peak"] = round(flops / bf16_ms / 1e9 / PEAK_BF16_MFMA_TFLOPS, 4)
        return out

    def per_config_block():
        """The workload list, configuration by configuration (median / minimum of 50 launches each)."""
        out = {}
        tiny = layer_passes("tiny", 4, "f32", ("fwd", "dgrad", "wgrad"), hp, synth, conv_flops, torch, timer)
        tiny.update(tiny_oracle_seconds())
        out["0_tiny_N4_fp32"] = tiny
        out["1_conv1_N128_fp32"] = layer_passes("conv1", 128, "f32", ("fwd", "wgrad"), hp, synth, conv_flops, torch,
                                                timer)
        out["2_conv2_column_N128_fp32"] = layer_passes("conv2", 128, "f32", ("fwd", "dgrad", "wgrad"), hp, synth,
                                                       conv_flops, torch, timer)
        for dt, tag in (("f32", "fp32"), ("bf16", "bf16_in_fp32_acc")):
            blk = {}
            for layer in ("conv3", "conv4", "conv5"):
                for p, t in layer_passes(layer, 256, dt, ("fwd", "dgrad", "wgrad"), hp, synth, conv_flops, torch,
                                         timer).items():
                    blk["%s.%s" % (layer, p)] = t
            out["3_conv3_5_N256_%s" % tag] = blk
        steps = {}
        for n in (64, 128, 256):
            for dt, peak in (("f32", PEAK_FP32_MFMA_TFLOPS), ("bf16", PEAK_BF16_MFMA_TFLOPS)):
                ms = ms_per_step if (n == N and dt == "f32") else stack_ms(n, dt, max(5, args.steps // 2), torch,
                                                                           ConvStack)
                tf = stack_flops(n) / ms / 1e9
                steps["N%d_%s" % (n, dt)] = {"ms_per_step": round(ms, 4), "tflops": round(tf, 2),
                                             "frac_peak": round(tf / peak, 4)}
        out["4_stack_step"] = steps
        return out

    columns, bf16, network, per_config = None, None, None, None
    if not args.stack_only:
        del stack
        network = extra("whole_network_fp32", lambda: whole_network(N, hp, torch, args.steps, timer))
        columns = extra("two_column_conv4_conv5_fp32",
                        lambda: two_column_layers(N, hp, synth, conv_flops, torch, timer))
        bf16 = extra("bf16_in_fp32_acc", bf16_block)
        per_config = extra("per_config", per_config_block)

    value = flops / ms_per_step / 1e9
    out = {
        "metric": "conv-stack TFLOP/s at N=%d (conv1-5 fwd+dgrad+wgrad, %s, ReLU/pool glue in the step)"
                  % (N, "fp32 MFMA" if args.stack_dtype == "f32" else "bf16 tensors, fp32 accumulation"),
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.stack_dtype, "data": "synthetic",
        "config": {"workload": "5-conv AlexNet stack fwd+bwd, N=%d, %s (conv2 as two model-parallel columns)"
                               % (N, "fp32" if args.stack_dtype == "f32" else "bf16"),
                   "batch": N, "conv_gflop_per_step": round(flops / 1e9, 2)},
        "frac_fp32_mfma_peak": round(value / PEAK_FP32_MFMA_TFLOPS, 4) if args.stack_dtype == "f32" else None,
        "mfma_ceiling_tflops": ceiling,
        "frac_of_measured_mfma_ceiling": (round(value / ceiling["sustained"], 4)
                                          if isinstance(ceiling, dict) and "sustained" in ceiling else None),
        "hip_graph_ms_per_step": None if graph_ms is None else round(graph_ms, 4),
        "conv_only_ms": round(conv_ms, 4),
        "conv_only_frac_peak": round(flops / conv_ms / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4),
        "timing_protocol": "value: wall clock over `steps` steps after `warmup`; per-pass / per_config figures: HIP "
                           "events on the launch stream, %d warm-up launches, then median (ms) and minimum (ms_min) "
                           "of %d samples of %d back-to-back launches each (per_pass: one launch per sample, inside "
                           "the running step); helper launches of a call (operand preparation, split sums) are "
                           "inside its time" % (WARMUP_LAUNCHES, TIMED_LAUNCHES, Timer.GROUP),
        "per_pass": per_pass,
        "roofline": roofline,
        "per_config": per_config,
        "two_column_conv4_conv5_fp32": columns,
        "bf16_in_fp32_acc": bf16,
        "whole_network_fp32": network,
        "context": "paper: 10.5 days per 100 epochs on one NVIDIA TITAN at batch 256 (whole network with data "
                   "loading: about 141 images/s; context for whole_network_fp32.step, not for value)",
    }
    if not args.no_cpu_baseline and not args.stack_only:
        out["cpu_baseline"] = extra("cpu_baseline", lambda: cpu_baseline(N))
    print(json.dumps(out))
    if failures:
        sys.stderr.write("bench.py: failed blocks: %s\n" % ", ".join(failures))
        sys.exit(1)


if __name__ == "__main__":
    main()
