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


def time_events(fn, reps):
    """Average duration in ms of `fn` launched `reps` times back to back on the current stream."""
    import torch
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    fn()
    torch.cuda.synchronize()
    start.record()
    for _ in range(reps):
        fn()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / reps


def kernel_breakdown(G, B, s, K, reps, flags=0):
    """Per-stage timing of one layer shape with HIP events on the stream the kernels run on.
    Returns {stage: dict(ms, bytes, flops, launches)} with ALGORITHMIC bytes / flops per call."""
    import numpy as np
    import torch
    t = s.as_tuple()
    M, C, E = s.M, s.Cin, s.E
    Eo = s.N * s.Ho * s.Wo * s.Cout
    wbytes = 4 * s.R * s.S * s.Cin * s.Cout
    P = B.abl_packed_bytes(t, K)
    flops = 2.0 * s.N * s.Ho * s.Wo * s.Cin * s.Cout * s.R * s.S
    f32 = dict(dtype=torch.float32, device="cuda")
    x = torch.randn(E, **f32)
    dy = torch.randn(Eo, **f32)
    y = torch.empty(Eo, **f32)
    a3 = torch.empty(E, **f32)
    dx = torch.empty(E, **f32)
    w = torch.randn(s.R * s.S * s.Cin * s.Cout, **f32) * 0.1
    dw = torch.empty_like(w)
    gamma, beta = torch.ones(C, **f32), torch.zeros(C, **f32)
    dg, db = torch.empty(C, **f32), torch.empty(C, **f32)
    stats = G.zeros_bytes(B.abl_stats_bytes(t))
    packed = G.zeros_bytes(P)
    scratch = G.zeros_bytes(B.abl_scratch_bytes(t, K))
    B.abl_bn_stats(x, M, C, gamma, beta, K, scratch, stats)
    B.abl_bn_relu_pack(x, M, C, K, stats, a3, packed)
    stages = {
        "bn_stats": (lambda: B.abl_bn_stats(x, M, C, gamma, beta, K, scratch, stats), 4 * E, 0, 2),
        "bn_relu_pack": (lambda: B.abl_bn_relu_pack(x, M, C, K, stats, a3, packed), 8 * E + P, 0, 1),
        "conv_fwd": (lambda: B.abl_conv_fwd(t, a3, w, None, y, flags=flags), 4 * E + 4 * Eo + wbytes, flops, 1),
        "conv_dgrad": (lambda: B.abl_conv_dgrad(t, dy, w, a3, flags=flags), 4 * E + 4 * Eo + wbytes, flops, 1),
        "conv_wgrad_packed": (lambda: B.abl_conv_wgrad_packed(t, K, packed, stats, dy, scratch, dw, flags=flags),
                              P + 4 * Eo + wbytes, flops, 2),
        "bn_bwd": (lambda: B.abl_bn_bwd(packed, stats, a3, M, C, K, scratch, dx, dg, db), 2 * P + 12 * E, 0, 3),
        "pack": (lambda: B.abl_pack(x, M, C, K, stats, packed), 4 * E + P, 0, 1),
        "unpack": (lambda: B.abl_unpack(packed, M, C, K, stats, a3), 4 * E + P, 0, 1),
    }
    out = {}
    for name, (fn, nbytes, fl, launches) in stages.items():
        ms = time_events(fn, reps)
        out[name] = dict(ms=ms, bytes=nbytes, flops=fl, launches=launches,
                         gbs=nbytes / ms / 1e6, tflops=fl / ms / 1e9)
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
    from tests import gpu_util as G

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
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    N, L = wl.shapes[0].N, len(layers)
    value = N * L / (dt / args.steps)

    # per-kernel timing of the (most frequent) layer shape, for the roofline block
    shapes = {}
    for s in wl.shapes:
        shapes[s] = shapes.get(s, 0) + 1
    per_step = {}
    breakdown = {}
    for s, count in shapes.items():
        bd = kernel_breakdown(G, B, s, K, args.kernel_reps, flags)
        breakdown["x".join(map(str, s.as_tuple()))] = {k: round(v["ms"] * 1e3, 2) for k, v in bd.items()}
        for k, v in bd.items():
            if k in ("pack", "unpack"):
                continue
            key = (s, k)
            per_step[key] = (v["ms"] * count, v)
    (dom_shape, dom_name), (_, dom) = max(per_step.items(), key=lambda kv: kv[1][0])
    mfma_peak = MFMA_BF16_PEAK_TFLOPS if args.math == "bf16" else MFMA_FP32_PEAK_TFLOPS
    flops_bound_ms = dom["flops"] / (mfma_peak * 1e9)
    bytes_bound_ms = dom["bytes"] / (HBM_PEAK_GBS * 1e6)
    if dom["flops"] > 0 and flops_bound_ms >= bytes_bound_ms:
        roof = {"bound": "mfma", "achieved": dom["tflops"], "peak": mfma_peak, "unit": "TFLOP/s",
                "frac": dom["tflops"] / mfma_peak}
    else:
        roof = {"bound": "hbm", "achieved": dom["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": dom["gbs"] / HBM_PEAK_GBS}
    roof.update({"traffic": None, "kernel": dom_name, "shape": "x".join(map(str, dom_shape.as_tuple())),
                 "avg_us": dom["ms"] * 1e3, "launches_per_call": dom["launches"]})

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
                   "stack_images_per_sec": N / (dt / args.steps)},
        "roofline": roof,
        "stage_us": breakdown,
        "pack_unpack_gbs": {},
        "activation_bytes": {"stored": run.stored_bytes(), "exact_fp32": exact_bytes,
                             "ratio": run.stored_bytes() / exact_bytes},
    }
    s0 = max(shapes, key=shapes.get)
    bd0 = kernel_breakdown(G, B, s0, K, args.kernel_reps, flags)
    result["pack_unpack_gbs"] = {"pack": bd0["pack"]["gbs"], "unpack": bd0["unpack"]["gbs"],
                                 "bn_relu_pack": bd0["bn_relu_pack"]["gbs"]}
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, K)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
