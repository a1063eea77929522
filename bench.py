#!/usr/bin/env python3
"""Benchmark of the approximate-activation layer step on one MI355X.

A step is one forward + one backward pass of the whole hot path over the CIFAR-ResNet-shaped
residual stage (18 stacked 3x3 BN-ReLU-conv layers, N=128, 16 channels, 32x32, identity skip
every 2 layers, K=4) on seeded synthetic tensors that are already resident in HBM.  Prints one
JSON line: layer train-step images/sec (images x layers / second), the roofline figures of the
dominant kernel and the CPU oracle's throughput on the same workload.
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
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--K", type=int, default=4)
    ap.add_argument("--workload", default="config2", choices=["config1", "config2", "config3a", "config3b",
                                                              "config4", "config5"])
    ap.add_argument("--math", default="fp32", choices=["fp32", "bf16"],
                    help="operand type of the conv contractions (bf16 = ABL_MATH_BF16 variant)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="record the step into a HIP graph once and time replays (pays for launch-bound workloads)")
    ap.add_argument("--kernel-reps", type=int, default=50)
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
    """Average duration in ms of `fn(i % nset)` launched `reps` times back to back on the current stream."""
    import torch
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(nset):
        fn(i)
    torch.cuda.synchronize()
    start.record()
    for i in range(reps):
        fn(i % nset)
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / reps


# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch), each divided by
# what the same counter reads for a plain device copy of known size (FETCH_SIZE reads 1/1.994 of the
# bytes, WRITE_SIZE 1/1.000), for the kernels of the default workload (3x3 16->16, 32x32, N=128, K=4).
# The runs and their commands are summarised under profiles/.
MEASURED_TRAFFIC = {
    ("config2", 4, "fp32"): {
        "bn_conv_fwd": 23.77e6,            # in the stack: half the layers also read a shortcut
        "conv_bwd_bn_reduce": 25.74e6,     # includes 4.7 MB of per-tile dW copies
    },
}


def kernel_breakdown(G, B, s, K, reps, flags=0):
    """Per-kernel timing of one layer shape with HIP events on the stream the kernels run on
    (torch's current stream, which is the one handed to the library).  Where the shape has the
    fused kernels (3x3 'same' stride-1 layers) these are the kernels the layer step runs; the
    separate stages are timed as well.  Returns {stage: dict(ms, bytes, flops, launches, step)} with
    ALGORITHMIC bytes / flops per call; step=True marks the stages that make up one layer step."""
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
    # name: (call on operand set i, algorithmic bytes, flops, launches, part of the layer step)
    stages = {
        "bn_stats": (lambda i: B.abl_bn_stats(S[i]["x"], M, C, gamma, beta, K, scratch, stats), 4 * E, 0, 2, not fused),
        "bn_relu_pack": (lambda i: B.abl_bn_relu_pack(S[i]["x"], M, C, K, stats, S[i]["a3"], S[i]["packed"]),
                         8 * E + P, 0, 1, not fwd_fused),
        "conv_fwd": (lambda i: B.abl_conv_fwd(t, S[i]["a3"], w, None, S[i]["y"], flags=flags), conv_bytes, flops, 1,
                     not fwd_fused),
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
                                                             flags=flags), conv_bytes + P, flops, 1, True)
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


def pack_unpack_large(G, B, K, reps):
    """Pack / unpack / fused normalise-ReLU-pack rates on a tensor large enough to be bound by HBM and
    not by the launch: the input of the first ImageNet bottleneck layer, [64*56*56, 256] fp32 (205 MB)."""
    import torch
    M, C = 64 * 56 * 56, 256
    E = M * C
    t = (64, 56, 56, C, 64, 1, 1, 1, 0)
    P = B.abl_packed_bytes(t, K)
    f32 = dict(dtype=torch.float32, device="cuda")
    gamma, beta = torch.ones(C, **f32), torch.zeros(C, **f32)
    stats = G.zeros_bytes(B.abl_stats_bytes(t))
    scratch = G.zeros_bytes(B.abl_bn_scratch_bytes(M, C))
    S = [dict(x=torch.randn(E, **f32), a3=torch.empty(E, **f32), packed=G.zeros_bytes(P)) for _ in range(2)]
    B.abl_bn_stats(S[0]["x"], M, C, gamma, beta, K, scratch, stats)
    for d in S:
        B.abl_bn_relu_pack(d["x"], M, C, K, stats, d["a3"], d["packed"])
    stages = {
        "pack": (lambda i: B.abl_pack(S[i]["x"], M, C, K, stats, S[i]["packed"]), 4 * E + P),
        "unpack": (lambda i: B.abl_unpack(S[i]["packed"], M, C, K, stats, S[i]["a3"]), 4 * E + P),
        "bn_relu_pack": (lambda i: B.abl_bn_relu_pack(S[i]["x"], M, C, K, stats, S[i]["a3"], S[i]["packed"]), 8 * E + P),
    }
    out = {"shape": "[%d, %d] fp32" % (M, C)}
    for name, (fn, nbytes) in stages.items():
        out[name] = nbytes / time_events(fn, reps, 2) / 1e6
    return out


def cpu_baseline(wl, K):
    """The CPU oracle, as it stands, on one full step of the same workload."""
    import numpy as np
    from oracle import abl_oracle as o
    from paper_1901_07988_amd import synth
    o.build()
    x, layers, dy = synth.draw_stack(wl)
    ol = [(o.Shape(*s.as_tuple()), w, g, b) for s, w, g, b in layers]
    t0 = time.time()
    _, saved = o.stack_forward(x, ol, K, np.float32, wl.skip_every)
    o.stack_backward(saved, ol, dy, np.float32, wl.skip_every)
    dt = time.time() - t0
    n = wl.shapes[0].N
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": n * len(layers) / dt, "unit": "images/sec per layer step", "cores": cores, "kind": "oracle",
            "sample": "1 full step (forward+backward, all %d layers, N=%d) of the same workload, %.1f s"
                      % (len(layers), n, dt)}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_1901_07988_amd import binding as B
    from paper_1901_07988_amd import synth
    from paper_1901_07988_amd import runtime as G

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    wl = get_workload(args.workload)
    K = args.K
    x, layers, dy = synth.draw_stack(wl)
    flags = B.ABL_MATH_BF16 if args.math == "bf16" else 0
    run = G.StackRun(layers, K, wl.skip_every, flags=flags)
    xd = G.dev(x).view(-1)
    dyd = G.dev(dy).view(-1)
    n_in, n_out = xd.numel(), dyd.numel()

    def step():
        run.buf_s[:n_in].copy_(xd)        # the batch arrives in the residual-stream buffer
        run.forward()
        run.buf_s[:n_out].copy_(dyd)      # the loss gradient arrives in the same buffer
        run.backward()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    timed_step = step
    if args.graph:
        # the library enqueues kernels only (no allocation, no synchronisation, no memset nodes), so
        # the whole step can be recorded once; tests/test_gpu_graph.py checks replays against eager
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        timed_step = graph.replay
        for _ in range(2):
            timed_step()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        timed_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    N, L = wl.shapes[0].N, len(layers)
    value = N * L / (dt / args.steps)

    # per-kernel timing of every distinct layer shape, for the roofline block: the dominant kernel is
    # the one with the largest share of the step among the kernels the layer step runs
    shapes = {}
    for s in wl.shapes:
        shapes[s] = shapes.get(s, 0) + 1
    per_step = {}
    breakdown = {}
    details = {}
    for s, count in shapes.items():
        bd = kernel_breakdown(G, B, s, K, args.kernel_reps, flags)
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
    traffic = MEASURED_TRAFFIC.get((args.workload, K, args.math), {}).get(dom_name)
    roof.update({"traffic": traffic, "kernel": dom_name, "shape": "x".join(map(str, dom_shape.as_tuple())),
                 "avg_us": dom["ms"] * 1e3, "launches_per_call": dom["launches"],
                 "algorithmic_bytes": dom["bytes"], "algorithmic_flops": dom["flops"],
                 "hbm_frac_of_same_kernel": dom["gbs"] / HBM_PEAK_GBS})

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
                   "stack_images_per_sec": N / (dt / args.steps)},
        "roofline": roof,
        "stage_us": breakdown,
        "pack_unpack_gbs": {},
        "activation_bytes": {"stored": run.stored_bytes(), "exact_fp32": exact_bytes,
                             "ratio": run.stored_bytes() / exact_bytes},
    }
    bd0 = details[max(shapes, key=shapes.get)]
    result["pack_unpack_gbs"] = {"pack": bd0["pack"]["gbs"], "unpack": bd0["unpack"]["gbs"],
                                 "bn_relu_pack": bd0["bn_relu_pack"]["gbs"]}
    if args.kernel_reps > 0:
        result["pack_unpack_gbs_large"] = pack_unpack_large(G, B, K, max(2, min(args.kernel_reps, 20)))
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, K)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
