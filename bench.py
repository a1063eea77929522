#!/usr/bin/env python3
"""Benchmark of the approximate-activation layer step on one MI355X.

A step is one forward + one backward pass of the whole hot path over the ImageNet deep-stage
bottleneck stack (12 x [1x1 1024->256, 3x3 256->256, 1x1 256->1024] BN-ReLU-conv layers at 14x14,
N=64, identity skip around every block, K=4, fp32) on seeded synthetic tensors that are already
resident in HBM.  Prints one JSON line: layer train-step images/sec (images x layers / second), the
roofline figures of the dominant kernel, the same step on the 56x56 bottleneck and on the CIFAR
stage as sub-results, the rates of the HBM-bound passes on a 205 MB tensor next to measured
read / write / copy ceilings, and the CPU oracle's throughput on a bounded sample of the workload.
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
MFMA_FP32_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix
MFMA_BF16_PEAK_TFLOPS = 2500.0 # MI355X dense bf16 matrix


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--K", type=int, default=4)
    ap.add_argument("--workload", default="config5", choices=["config1", "config2", "config3a", "config3b",
                                                              "config4", "config5"])
    ap.add_argument("--math", default="fp32", choices=["fp32", "bf16"],
                    help="operand type of the conv contractions (bf16 = ABL_MATH_BF16 variant)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="record the step into a HIP graph once and time replays (pays for launch-bound workloads)")
    ap.add_argument("--kernel-reps", type=int, default=20)
    ap.add_argument("--no-sub", action="store_true", help="skip the sub-results on the other workloads")
    return ap.parse_args()


def get_workload(name):
    from paper_1901_07988_amd import synth
    if name == "config1":
        return synth.config1()
    if name == "config2":
        return synth.config2()
    if name in ("config3a", "config3b"):
        return synth.config3()[0 if name == "config3a" else 1]
    if name == "config4":
        return synth.config4()
    return synth.config5()


def time_events(fn, reps, nset=1):
    """Average duration in ms of `fn(i % nset)` launched `reps` times back to back on the current stream.
    The timed launches follow some 25 ms of the same launches: after an idle gap (the set-up between
    two stages) the clocks need that long to come back up, and a matrix-core-bound kernel timed in a
    short burst right after it reads 8-10 % slow (measured: 137 us in a burst of 20 after idling,
    124 us from the hundredth launch on, 125.5 us inside the layer step)."""
    import torch
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(nset):
        fn(i)
    torch.cuda.synchronize()
    start.record()
    for i in range(3):
        fn(i % nset)
    stop.record()
    torch.cuda.synchronize()
    est = max(start.elapsed_time(stop) / 3, 1e-3)
    for i in range(min(400, int(25.0 / est))):
        fn(i % nset)
    start.record()
    for i in range(reps):
        fn(i % nset)
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / reps


# HBM bytes per launch (fetch + write) from two rocprofv3 --pmc runs, FETCH_SIZE and WRITE_SIZE in KiB per
# dispatch, each scaled by what the same counter reads for the plain streaming kernels of the same run
# (abl_hbm_probe on 205 MB: FETCH_SIZE reads 1/2.000 of the bytes, WRITE_SIZE 1/1.000).  The runs, their
# commands and the per-kernel tables are under profiles/*_hbm_traffic.txt; counters cannot be read inside
# a timed run, so the figures of the single-launch stages are kept here, by workload and layer shape.
S3 = "64x14x14x256x256x3x3x1x1"
MEASURED_TRAFFIC = {
    ("config5", 4, "fp32"): {
        (S3, "bn_conv_fwd"): 46.50e6,            # x 12.8 MB + the weights once per XCD (8 x 2.4 MB) + y + codes
        (S3, "conv_fwd"): 45.09e6,
        (S3, "conv_dgrad_bn_reduce"): 46.81e6,
        ("64x14x14x1024x256x1x1x1x0", "bn_conv_fwd"): 86.82e6,
        ("64x14x14x1024x256x1x1x1x0", "conv_dgrad_bn_reduce"): 79.86e6,
    },
    ("config4", 4, "fp32"): {
        ("64x56x56x64x64x3x3x1x1", "bn_conv_fwd"): 143.07e6,
        ("64x56x56x64x64x3x3x1x1", "conv_fwd"): 120.12e6,
        ("64x56x56x64x64x3x3x1x1", "conv_dgrad_bn_reduce"): 119.33e6,
        ("64x56x56x256x64x1x1x1x0", "bn_conv_fwd"): 288.55e6,
    },
    ("config2", 4, "fp32"): {
        ("128x32x32x16x16x3x3x1x1", "bn_conv_fwd"): 23.77e6,         # in the stack: half the layers also read a shortcut
        ("128x32x32x16x16x3x3x1x1", "conv_bwd_bn_reduce"): 25.79e6,  # includes 4.7 MB of per-tile dW copies
    },
}


def kernel_breakdown(G, B, s, K, reps, flags=0, in_place=False):
    """Per-kernel timing of one layer shape with HIP events on the stream the kernels run on
    (torch's current stream, which is the one handed to the library).  Where the shape has the
    fused kernels (3x3 'same' stride-1 layers) these are the kernels the layer step runs; the
    separate stages are timed as well.  Returns {stage: dict(ms, bytes, flops, launches, step)} with
    ALGORITHMIC bytes / flops per call; step=True marks the stages that make up one layer step.
    in_place: every layer of this shape in the stack runs in place on the shared buffer (the middle
    layers of a residual group), where the forward with the fused prologue cannot be used: the step
    then consists of the normalise-ReLU-pack pass and the plain forward."""
    import torch
    t = s.as_tuple()
    M, C, E = s.M, s.Cin, s.E
    Eo = s.N * s.Ho * s.Wo * s.Cout
    wbytes = 4 * s.R * s.S * s.Cin * s.Cout
    P = B.abl_packed_bytes(t, K)
    flops = 2.0 * s.N * s.Ho * s.Wo * s.Cin * s.Cout * s.R * s.S
    f32 = dict(dtype=torch.float32, device="cuda")
    # Several sets of operands, used in turn, so that a kernel does not find its own previous output
    # in the L2 caches (in the layer step its operands were last touched by other kernels).
    nset = max(1, min(8, (96 << 20) // (8 * E + 8 * Eo)))
    w = torch.randn(s.R * s.S * s.Cin * s.Cout, **f32) * 0.1
    dw = torch.empty_like(w)
    gamma, beta = torch.ones(C, **f32), torch.zeros(C, **f32)
    dg, db = torch.empty(C, **f32), torch.empty(C, **f32)
    stats = G.zeros_bytes(B.abl_stats_bytes(t))
    scratch = G.zeros_bytes(B.abl_scratch_bytes(t, K))
    sets = []
    for _ in range(nset):
        d = dict(x=torch.randn(E, **f32), dy=torch.randn(Eo, **f32), y=torch.empty(Eo, **f32),
                 a3=torch.empty(E, **f32), dx=torch.empty(E, **f32), packed=G.zeros_bytes(P))
        B.abl_bn_stats(d["x"], M, C, gamma, beta, K, scratch, stats)
        B.abl_bn_relu_pack(d["x"], M, C, K, stats, d["a3"], d["packed"])
        sets.append(d)
    d = sets[0]
    fwd_fused = fused = True
    try:
        B.abl_bn_conv_fwd(t, K, d["x"], stats, w, None, d["y"], d["packed"], flags=flags)
    except B.AblError:
        fwd_fused = False
    try:
        B.abl_conv_dgrad_bn_reduce(t, K, d["dy"], w, d["packed"], stats, scratch, d["dx"], flags=flags)
    except B.AblError:
        fused = False
    bwd_fused = fused
    if fused:
        try:
            B.abl_conv_bwd_bn_reduce(t, K, d["dy"], w, d["packed"], stats, scratch, d["dx"], dw, flags=flags)
        except B.AblError:
            bwd_fused = False
    conv_bytes = 4 * E + 4 * Eo + wbytes
    S = sets
    fwd_fused_step = fwd_fused and not in_place and B.abl_forward_is_fused(t, K, flags)
    # name: (call on operand set i, algorithmic bytes, flops, launches, part of the layer step)
    stages = {
        "bn_stats": (lambda i: B.abl_bn_stats(S[i]["x"], M, C, gamma, beta, K, scratch, stats), 4 * E, 0, 2, not fused),
        "bn_relu_pack": (lambda i: B.abl_bn_relu_pack(S[i]["x"], M, C, K, stats, S[i]["a3"], S[i]["packed"]),
                         8 * E + P, 0, 1, not fwd_fused_step),
        "conv_fwd": (lambda i: B.abl_conv_fwd(t, S[i]["a3"], w, None, S[i]["y"], flags=flags), conv_bytes, flops, 1,
                     not fwd_fused_step),
        "conv_dgrad": (lambda i: B.abl_conv_dgrad(t, S[i]["dy"], w, S[i]["dx"], flags=flags), conv_bytes, flops, 1,
                       not fused),
        "conv_wgrad_packed": (lambda i: B.abl_conv_wgrad_packed(t, K, S[i]["packed"], stats, S[i]["dy"], scratch, dw,
                                                                flags=flags), P + 4 * Eo + wbytes, flops, 2,
                              not bwd_fused),
        "bn_bwd": (lambda i: B.abl_bn_bwd(S[i]["packed"], stats, S[i]["dx"], M, C, K, scratch, S[i]["a3"], dg, db),
                   2 * P + 12 * E, 0, 3, not fused),
        "pack": (lambda i: B.abl_pack(S[i]["x"], M, C, K, stats, S[i]["packed"]), 4 * E + P, 0, 1, False),
        "unpack": (lambda i: B.abl_unpack(S[i]["packed"], M, C, K, stats, S[i]["a3"]), 4 * E + P, 0, 1, False),
    }
    if fwd_fused:
        stages["bn_conv_fwd"] = (lambda i: B.abl_bn_conv_fwd(t, K, S[i]["x"], stats, w, None, S[i]["y"], S[i]["packed"],
                                                             flags=flags), conv_bytes + P, flops, 1, fwd_fused_step)
    if fused:
        stages["conv_dgrad_bn_reduce"] = (
            lambda i: B.abl_conv_dgrad_bn_reduce(t, K, S[i]["dy"], w, S[i]["packed"], stats, scratch, S[i]["dx"],
                                                 flags=flags), conv_bytes + P, flops, 1, not bwd_fused)
    if bwd_fused:
        # both contractions of the backward in one kernel; its per-tile copies of dW are summed by the
        # launch that also finishes the BN-backward sums, so the kernel is timed without that sum
        stages["conv_bwd_bn_reduce"] = (
            lambda i: B.abl_conv_bwd_bn_reduce(t, K, S[i]["dy"], w, S[i]["packed"], stats, scratch, S[i]["dx"], None,
                                               flags=flags), conv_bytes + P + wbytes, 2 * flops, 1, True)
    out = {}
    for name, (fn, nbytes, fl, launches, in_step) in stages.items():
        ms = time_events(fn, reps, nset)
        out[name] = dict(ms=ms, bytes=nbytes, flops=fl, launches=launches, step=in_step,
                         gbs=nbytes / ms / 1e6, tflops=fl / ms / 1e9)
    return out


def hbm_bound_passes(G, B, K, reps):
    """The HBM-bound passes of the method on a tensor large enough to be bound by memory and not by
    the launch - the input of the first ImageNet bottleneck layer, [64*56*56, 256] fp32 (205 MB) - next
    to what plain read-only / write-only / copy kernels reach on the same tensor (abl_hbm_probe).
    Three operand sets are used in turn (1.3 GB in all), so nothing is found in a cache."""
    import torch
    M, C = 64 * 56 * 56, 256
    E = M * C
    t = (64, 56, 56, C, 64, 1, 1, 1, 0)
    P = B.abl_packed_bytes(t, K)
    f32 = dict(dtype=torch.float32, device="cuda")
    gamma, beta = torch.ones(C, **f32), torch.zeros(C, **f32)
    dg, db = torch.empty(C, **f32), torch.empty(C, **f32)
    stats = G.zeros_bytes(B.abl_stats_bytes(t))
    scratch = G.zeros_bytes(B.abl_bn_scratch_bytes(M, C))
    nset = 3
    S = [dict(x=torch.randn(E, **f32), a3=torch.empty(E, **f32), packed=G.zeros_bytes(P)) for _ in range(nset)]
    B.abl_bn_stats(S[0]["x"], M, C, gamma, beta, K, scratch, stats)
    for d in S:
        B.abl_bn_relu_pack(d["x"], M, C, K, stats, d["a3"], d["packed"])
    nb = 4 * E
    probes = {
        "read": (lambda i: B.abl_hbm_probe(0, S[i]["x"], scratch, nb), nb),
        "write": (lambda i: B.abl_hbm_probe(1, None, S[i]["a3"], nb), nb),
        "copy": (lambda i: B.abl_hbm_probe(2, S[i]["x"], S[i]["a3"], nb), 2 * nb),
    }
    ceil = {k: nbytes / time_events(fn, reps, nset) / 1e6 for k, (fn, nbytes) in probes.items()}
    # name: (call, algorithmic bytes, launches, which ceiling its traffic mix is compared with)
    stages = {
        "bn_stats": (lambda i: B.abl_bn_stats(S[i]["x"], M, C, gamma, beta, K, scratch, stats), 4 * E, 2, "read"),
        "pack": (lambda i: B.abl_pack(S[i]["x"], M, C, K, stats, S[i]["packed"]), 4 * E + P, 1, "read"),
        "unpack": (lambda i: B.abl_unpack(S[i]["packed"], M, C, K, stats, S[i]["a3"]), 4 * E + P, 1, "write"),
        "bn_relu_pack": (lambda i: B.abl_bn_relu_pack(S[i]["x"], M, C, K, stats, S[i]["a3"], S[i]["packed"]),
                         8 * E + P, 1, "copy"),
        # Eq. 6-7 sums (read dA3 + codes), second pass, Eq. 8 (read dA3 + codes, write dx): three launches
        "bn_bwd": (lambda i: B.abl_bn_bwd(S[i]["packed"], stats, S[i]["x"], M, C, K, scratch, S[i]["a3"], dg, db),
                   12 * E + 2 * P, 3, "copy"),
    }
    out = {"shape": "[%d, %d] fp32" % (M, C), "hbm_peak_gbs": HBM_PEAK_GBS,
           "ceiling_gbs": {k: round(v, 1) for k, v in ceil.items()}}
    for name, (fn, nbytes, launches, kind) in stages.items():
        gbs = nbytes / time_events(fn, reps, nset) / 1e6
        out[name] = {"gbs": round(gbs, 1), "frac_of_peak": round(gbs / HBM_PEAK_GBS, 3),
                     "frac_of_%s_ceiling" % kind: round(gbs / ceil[kind], 3), "launches": launches}
    return out


def mfma_ceilings(G, B, reps=5):
    """TFLOP/s that a loop of independent matrix instructions on register operands reaches
    (abl_mfma_probe): the practical ceiling of the contractions next to the published peak."""
    out = G.zeros_bytes(B.abl_mfma_probe_out_bytes())
    res = {}
    for name, mode, iters in (("fp32_16x16x4", 0, 1000), ("bf16_16x16x32", 1, 2000)):
        ms = time_events(lambda i: B.abl_mfma_probe(mode, iters, out), reps)
        res[name] = round(B.abl_mfma_probe_flops(mode, iters) / ms / 1e9, 1)
    return res


def omp_threads(set_to=None):
    """Size of the OpenMP team the oracle's loops run with (optionally change it first)."""
    import ctypes
    try:
        gomp = ctypes.CDLL("libgomp.so.1")
    except OSError:
        return None
    if set_to is not None:
        gomp.omp_set_num_threads(int(set_to))
    return int(gomp.omp_get_max_threads())


def oracle_step_seconds(o, np, x, layers, dy, K, skip_every):
    ol = [(o.Shape(*s.as_tuple()), w, g, b) for s, w, g, b in layers]
    t0 = time.time()
    _, saved = o.stack_forward(x, ol, K, np.float32, skip_every)
    o.stack_backward(saved, ol, dy, np.float32, skip_every)
    return time.time() - t0


def cpu_baseline(wl, K):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: the whole step where
    that takes seconds, else the first group of layers (one bottleneck block), scaled by the number
    of identical groups."""
    import numpy as np
    from oracle import abl_oracle as o
    from paper_1901_07988_amd import synth
    o.build()
    x, layers, dy = synth.draw_stack(wl)
    n, L = wl.shapes[0].N, len(layers)
    g = wl.skip_every
    periodic = g > 0 and L > g and L % g == 0 and all(wl.shapes[i] == wl.shapes[i % g] for i in range(L))
    flops = sum(6.0 * s.N * s.Ho * s.Wo * s.Cin * s.Cout * s.R * s.S for s in wl.shapes)
    threads = omp_threads()
    if periodic and flops > 200e9:
        # dy of the sample: the seeded gradient at the top of the stack has the block's output shape
        dt_block = oracle_step_seconds(o, np, x, layers[:g], dy, K, g)
        dt = dt_block * (L // g)
        sample = ("forward+backward of the first block (%d layers, N=%d) of the same workload: %.1f s, times the %d "
                  "identical blocks" % (g, n, dt_block, L // g))
    else:
        dt = oracle_step_seconds(o, np, x, layers, dy, K, g)
        sample = "1 full step (forward+backward, all %d layers, N=%d) of the same workload, %.1f s" % (L, n, dt)
    out = {"value": n * L / dt, "unit": "images/sec per layer step", "cores": threads, "kind": "oracle",
           "sample": sample}
    # one core on the smallest configuration (a single 3x3 16->16 layer at 32x32, N=8)
    w1 = synth.config1()
    x1, l1, dy1 = synth.draw_stack(w1)
    omp_threads(set_to=1)
    dt1 = min(oracle_step_seconds(o, np, x1, l1, dy1, K, 0) for _ in range(3))
    omp_threads(set_to=threads)
    out["config1_single_thread"] = {"value": w1.shapes[0].N / dt1, "unit": "images/sec per layer step", "cores": 1,
                                    "sample": "forward+backward of %s, best of 3, %.1f ms" % (w1.name, dt1 * 1e3)}
    return out


def time_stack(G, B, synth, wl, K, flags, steps, warmup, graph=False):
    """ms per step (forward + backward of the whole stack, inputs resident in HBM) and the StackRun."""
    import torch
    x, layers, dy = synth.draw_stack(wl)
    run = G.StackRun(layers, K, wl.skip_every, flags=flags)
    xd = G.dev(x).view(-1)
    dyd = G.dev(dy).view(-1)
    n_in, n_out = xd.numel(), dyd.numel()

    def step():
        run.buf_s[:n_in].copy_(xd)        # the batch arrives in the residual-stream buffer
        run.forward()
        run.buf_s[:n_out].copy_(dyd)      # the loss gradient arrives in the same buffer
        run.backward()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    timed_step = step
    if graph:
        # the library enqueues kernels only (no allocation, no synchronisation, no memset nodes), so
        # the whole step can be recorded once; tests/test_gpu_graph.py checks replays against eager
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            step()
        timed_step = g.replay
        for _ in range(2):
            timed_step()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        timed_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    return dt / steps * 1e3, run


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_1901_07988_amd import binding as B
    from paper_1901_07988_amd import synth
    from paper_1901_07988_amd import runtime as G

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    wl = get_workload(args.workload)
    K = args.K
    flags = B.ABL_MATH_BF16 if args.math == "bf16" else 0
    ms_per_step, run = time_stack(G, B, synth, wl, K, flags, args.steps, args.warmup, args.graph)
    N, L = wl.shapes[0].N, len(wl.shapes)
    value = N * L / (ms_per_step * 1e-3)
    stored = run.stored_bytes()
    del run
    torch.cuda.empty_cache()

    # per-kernel timing of every distinct layer shape, for the roofline block: the dominant kernel is
    # the one with the largest share of the step among the kernels the layer step runs
    shapes = {}
    for s in wl.shapes:
        shapes[s] = shapes.get(s, 0) + 1
    # layers that the stack runs in place (include/abl.h, abl_stack_forward: the middle layers of a
    # complete residual group; of an odd chain outside the groups, the first)
    g = wl.skip_every
    n_grouped = (L // g) * g if g > 0 else 0
    in_place_layer = [(g > 0 and i < n_grouped and 0 < i % g < g - 1) or
                      (i == n_grouped and (L - n_grouped) % 2 == 1) for i in range(L)]
    in_place_shape = {s: all(in_place_layer[i] for i, t in enumerate(wl.shapes) if t == s) for s in shapes}
    per_step = {}
    breakdown = {}
    details = {}
    for s, count in shapes.items():
        bd = kernel_breakdown(G, B, s, K, args.kernel_reps, flags, in_place_shape[s])
        details[s] = bd
        breakdown["x".join(map(str, s.as_tuple()))] = {k: round(v["ms"] * 1e3, 2) for k, v in bd.items()}
        for k, v in bd.items():
            if v["step"]:
                per_step[(s, k)] = (v["ms"] * count, v)
    # a stage that is one launch is preferred when it is within 25% of a several-launch one, so that
    # the figure is that of a single kernel
    (dom_shape, dom_name), (_, dom) = max(per_step.items(),
                                          key=lambda kv: kv[1][0] * (1.0 if kv[1][1]["launches"] == 1 else 0.75))
    mfma_peak = MFMA_BF16_PEAK_TFLOPS if args.math == "bf16" else MFMA_FP32_PEAK_TFLOPS
    flops_bound_ms = dom["flops"] / (mfma_peak * 1e9)
    bytes_bound_ms = dom["bytes"] / (HBM_PEAK_GBS * 1e6)
    if dom["flops"] > 0 and flops_bound_ms >= bytes_bound_ms:
        roof = {"bound": "mfma", "achieved": dom["tflops"], "peak": mfma_peak, "unit": "TFLOP/s",
                "frac": dom["tflops"] / mfma_peak}
    else:
        roof = {"bound": "hbm", "achieved": dom["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": dom["gbs"] / HBM_PEAK_GBS}
    wl_key = args.workload
    dom_shape_str = "x".join(map(str, dom_shape.as_tuple()))
    traffic = MEASURED_TRAFFIC.get((wl_key, K, args.math), {}).get((dom_shape_str, dom_name))
    roof.update({"traffic": traffic, "kernel": dom_name, "shape": dom_shape_str,
                 "avg_us": dom["ms"] * 1e3, "launches_per_call": dom["launches"],
                 "algorithmic_bytes": dom["bytes"], "algorithmic_flops": dom["flops"],
                 "hbm_frac_of_same_kernel": dom["gbs"] / HBM_PEAK_GBS})
    roof["measured_mfma_ceiling_tflops"] = mfma_ceilings(G, B)
    # every contraction of the step against the fp32 (or bf16) matrix peak
    roof["contractions_frac_of_mfma_peak"] = {
        "x".join(map(str, s.as_tuple())): {k: round(v["tflops"] / mfma_peak, 3) for k, v in bd.items()
                                             if v["step"] and v["flops"] > 0}
        for s, bd in details.items()}

    exact_bytes = sum(4 * s.E for s in wl.shapes)
    result = {
        "metric": "layer train-step images/sec at K=%d" % K,
        "value": value,
        "unit": "images/sec per layer step (N x layers / step time)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if args.math == "fp32" else "bf16 operands, f32 accumulate (contractions); f32 elsewhere",
        "data": "synthetic",
        "config": {"workload": wl.name, "K": K, "layers": L, "batch": N, "skip_every": wl.skip_every,
                   "launch": "hip graph replay" if args.graph else "eager",
                   "stack_images_per_sec": N / (ms_per_step * 1e-3)},
        "roofline": roof,
        "stage_us": breakdown,
        "activation_bytes": {"stored": stored, "exact_fp32": exact_bytes, "ratio": stored / exact_bytes},
    }
    bd0 = details[max(shapes, key=shapes.get)]
    result["pack_unpack_gbs"] = {"pack": bd0["pack"]["gbs"], "unpack": bd0["unpack"]["gbs"],
                                 "bn_relu_pack": bd0["bn_relu_pack"]["gbs"]}
    del details
    torch.cuda.empty_cache()
    if args.kernel_reps > 0:
        result["hbm_bound_passes_large"] = hbm_bound_passes(G, B, K, max(3, min(args.kernel_reps, 24)))
        torch.cuda.empty_cache()
    if not args.no_sub:
        # the same step on the other ImageNet-shaped workload and on the CIFAR stage
        subs = []
        for name, steps in (("config4", 30), ("config2", 100)):
            if name == args.workload:
                continue
            w2 = get_workload(name)
            ms2, run2 = time_stack(G, B, synth, w2, K, flags, steps, 5)
            n2, l2 = w2.shapes[0].N, len(w2.shapes)
            subs.append({"workload": w2.name, "K": K, "steps": steps, "ms_per_step": ms2,
                         "value": n2 * l2 / (ms2 * 1e-3), "unit": result["unit"]})
            del run2
            torch.cuda.empty_cache()
        if args.math == "fp32" and args.workload != "config4":
            # the bf16-operand variant (32-deep bf16 matrix instruction, fp32 accumulation) on config 4
            w2 = get_workload("config4")
            ms2, run2 = time_stack(G, B, synth, w2, K, B.ABL_MATH_BF16, 30, 5)
            subs.append({"workload": w2.name + " --math bf16", "K": K, "steps": 30, "ms_per_step": ms2,
                         "value": w2.shapes[0].N * len(w2.shapes) / (ms2 * 1e-3), "unit": result["unit"],
                         "dtype": "bf16 operands, f32 accumulate (contractions); f32 elsewhere"})
            del run2
            torch.cuda.empty_cache()
        if args.math == "fp32" and args.workload != "config4":
            # ... and on the timed workload itself
            ms2, run2 = time_stack(G, B, synth, wl, K, B.ABL_MATH_BF16, args.steps, args.warmup)
            subs.append({"workload": wl.name + " --math bf16", "K": K, "steps": args.steps, "ms_per_step": ms2,
                         "value": N * L / (ms2 * 1e-3), "unit": result["unit"],
                         "dtype": "bf16 operands, f32 accumulate (contractions); f32 elsewhere"})
            del run2
            torch.cuda.empty_cache()
        if K == 4 and args.math == "fp32":
            # the same workload with 8-bit codes (twice the stored bytes, same kernels)
            ms2, run2 = time_stack(G, B, synth, wl, 8, flags, args.steps, args.warmup)
            subs.append({"workload": wl.name + " K=8", "K": 8, "steps": args.steps, "ms_per_step": ms2,
                         "value": N * L / (ms2 * 1e-3), "unit": result["unit"],
                         "stored_over_exact": run2.stored_bytes() / exact_bytes})
            del run2
            torch.cuda.empty_cache()
        result["sub_results"] = subs
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, K)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
