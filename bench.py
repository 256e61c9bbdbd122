#!/usr/bin/env python3
"""Throughput of the SQuant solver on one MI355X.

A step is one pass of the whole path (absmax scale, SQuant-E, SQuant-K, candidate update,
SQuant-C, int8 emit) over the whole workload, as ONE batched library call, with the
weights already resident in HBM.  Prints one JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5|c1|c2|c3|c4] [--bits 4]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
WORKLOADS = {
    "c1": (1, "1 x [64,64,3,3] He-normal"),
    "c2": (2, "ResNet-18-shaped layer set (21 tensors), He-normal"),
    "c3": (3, "ResNet-50-shaped layer set (54 tensors), He-normal + 1% Laplace outliers"),
    "c4": (4, "MobileNetV2-shaped layer set (53 tensors), He-normal"),
    "c5": (5, "256 x [512,512,3,3] fp32, N(0,s) / Student-t(3) per tensor, one batched call"),
    "c6": (6, "InceptionV3-style layer set (95 tensors: 1x7, 7x1, 1x3, 3x1, 5x5, 3x3, 1x1), He-normal"),
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


K9_SOURCES = ("squant_k9.h", "squant_select.h", "squant_io.h", "squant_common.h", "squant_arith.h")


def kernel_source_digest() -> str:
    """SHA-256 over the code (comments and blank space dropped) the 3x3 kernel is compiled from."""
    import hashlib
    import re
    h = hashlib.sha256()
    for name in K9_SOURCES:
        with open(os.path.join(ROOT, "paper_2202_07471_amd", "csrc", name)) as f:
            text = re.sub(r"//[^\n]*", "", f.read())
        h.update(" ".join(text.split()).encode())
    return h.hexdigest()


def load_traffic():
    """HBM bytes per launch measured with rocprofv3 --pmc (see profiles/); None when the
    kernel's sources have changed since the counters were taken."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            t = json.load(f)
        if t.get("kernel_source_sha256") == kernel_source_digest():
            return float(t["bytes_per_launch"])
    except (OSError, ValueError, KeyError):
        pass
    return None


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50,
                    help="untimed steps first; the GPU needs a few tens of launches to settle its clocks")
    ap.add_argument("--workload", default="c5", choices=sorted(WORKLOADS))
    ap.add_argument("--bits", type=int, default=4)
    ap.add_argument("--mode", default="EKC", choices=["E", "EK", "EKC", "EC"],
                    help="stages to run; the headline metric is EKC")
    ap.add_argument("--tensors", type=int, default=None, help="truncate the tensor list (debug)")
    ap.add_argument("--shape", default=None,
                    help="cout,cin,kh,kw: replace the workload by --count He-normal tensors of this shape "
                         "(exploration only; not the headline configuration)")
    ap.add_argument("--count", type=int, default=1)
    ap.add_argument("--output", default="int8", choices=["int8", "int4", "f32", "bf16"],
                    help="what the solver writes per weight: int8 codes (headline), packed 4-bit "
                         "codes, or dequantised float32 / bfloat16")
    ap.add_argument("--wtype", default="f32", choices=["f32", "f16", "bf16"],
                    help="element type the weights are handed over in (headline: f32)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference point for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; every output channel is independent, so "
              "more GPUs would each take a slice of the tensors with no exchange. "
              "Run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2202_07471_amd as sq
    from paper_2202_07471_amd import synth

    sq.binding.lib()   # fails loudly when the HIP library has not been built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    config, desc = WORKLOADS[args.workload]
    specs = synth.config_specs(config, n_tensors=args.tensors)
    if args.shape:
        shp = tuple(int(v) for v in args.shape.split(","))
        desc = f"custom: {args.count} x {list(shp)} He-normal"
        specs = [synth.TensorSpec(9, i, shp, "normal", synth.he_sigma(shp)) for i in range(args.count)]
    n_params = sum(s.numel for s in specs)
    n_channels = sum(s.shape[0] for s in specs)
    log(f"[bench] workload {args.workload}: {len(specs)} tensors, {n_params} weights, "
        f"{n_channels} output channels")

    # ---- synthetic weights: generated once on the host, uploaded, a sample kept for the CPU leg
    # the CPU leg runs the reference over the whole workload (C5: about 1 s on 16 threads, some
    # 15 s of CPU work) and every GPU output of the timed configuration is compared with it
    cpu_sample_tensors = 64 if args.shape else len(specs)
    t0 = time.time()
    host_sample, dws = [], []
    for s in specs:
        w = synth.generate(s)
        dw = torch.from_numpy(w).to(dev)
        if args.wtype != "f32":        # the generator's weights rounded once to the 16-bit type
            dw = dw.to(torch.float16 if args.wtype == "f16" else torch.bfloat16)
        dws.append(dw)
        if s.index < cpu_sample_tensors:
            host_sample.append(w if args.wtype == "f32" else dw.float().cpu().numpy())
    torch.cuda.synchronize()
    log(f"[bench] generated + uploaded in {time.time() - t0:.1f} s "
        f"({sum(s.dist == 'student_t3' for s in specs)} Student-t tensors)")

    plan = sq.BatchPlan(dws, sq.OUTPUTS[args.output])
    mode = sq.MODES[args.mode]
    if args.calibrate_copy:
        a_ = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        b_ = torch.empty_like(a_)
        b_.copy_(a_)            # 1 GiB read + 1 GiB written by one elementwise copy kernel
        torch.cuda.synchronize()
        del a_, b_

    def step():
        plan.run(args.bits, mode)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    sq.squant_kernel_timer_enable(max(args.steps, 1))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kernel_ms = [sq.squant_kernel_timer_elapsed_ms(c) for c in range(args.steps)]
    sq.squant_kernel_timer_enable(0)

    ms_per_step = elapsed * 1e3 / max(args.steps, 1)
    value = n_params * args.steps / elapsed / 1e9
    k_avg_ms = float(np.mean(kernel_ms))
    # bytes read + written per weight (4 + 1 in the headline configuration), 4 B per scale
    in_bytes = {"f32": 4.0, "f16": 2.0, "bf16": 2.0}[args.wtype]
    out_bytes = {"int8": 1.0, "int4": 0.5, "f32": 4.0, "bf16": 2.0}[args.output]
    algo_bytes = (in_bytes + out_bytes) * n_params + 4.0 * n_channels
    achieved = algo_bytes / (k_avg_ms * 1e-3) / 1e9
    headline_io = args.output == "int8" and args.wtype == "f32"
    traffic = (load_traffic()
               if args.workload == "c5" and args.tensors is None and headline_io else None)
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "kernel": "squant solver kernel(s) of the batched call",
                "kernel_ms_avg": round(k_avg_ms, 4), "kernel_ms_median": round(float(np.median(kernel_ms)), 4),
                "kernel_ms_min": round(float(np.min(kernel_ms)), 4),
                "algorithmic_bytes_per_launch": algo_bytes}
    if os.environ.get("SQUANT_BENCH_TRACE"):
        log("[bench] kernel ms per step: " + " ".join(f"{v:.3f}" for v in kernel_ms))
    log(f"[bench] {ms_per_step:.4f} ms/step wall, kernel avg {k_avg_ms:.4f} ms -> "
        f"{value:.1f} Gparams/s, {achieved:.0f} GB/s algorithmic ({100 * achieved / HBM_PEAK_GBS:.1f}% of peak)")

    # ---- CPU baseline: the reference solver as it stands, on this machine's host cores ----
    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        cores = oracle.hardware_threads()
        env_threads = os.environ.get("OMP_NUM_THREADS")
        threads = min(cores, int(env_threads)) if env_threads and env_threads.isdigit() else cores
        sample_params = sum(w.size for w in host_sample)
        t0 = time.perf_counter()
        ref = [oracle.quantize(w, args.bits, mode, threads=threads) for w in host_sample]
        cpu_s = time.perf_counter() - t0
        t0 = time.perf_counter()
        n1 = max(1, min(4, len(host_sample)))
        for w in host_sample[:n1]:
            oracle.quantize(w, args.bits, mode, threads=1)
        cpu1_s = time.perf_counter() - t0
        p1 = sum(w.size for w in host_sample[:n1])
        # the GPU result of the timed configuration, checked against the same reference
        mism = 0
        for i, (rc, rs) in enumerate(ref):
            go = plan.codes[i]
            gc = (go.view(torch.int16) if go.dtype == torch.bfloat16 else go).cpu().numpy()
            gs = plan.scales[i].cpu().numpy()
            if args.output == "int4":
                rc = oracle.pack_int4(rc)
            elif args.output == "f32":
                rc, gc = oracle.dequantize(rc, rs).view(np.uint32), gc.view(np.uint32)
            elif args.output == "bf16":
                rc, gc = oracle.dequantize_bf16(rc, rs), gc.view(np.uint16)
            mism += int((gc != rc).sum()) + int((gs.view(np.uint32) != rs.view(np.uint32)).sum())
        cpu_baseline = {"value": round(sample_params / cpu_s / 1e9, 5), "unit": "Gparams/s",
                        "cores": threads, "kind": "oracle",
                        "sample": (f"all {len(host_sample)} tensors of the workload" if len(host_sample) == len(specs)
                                   else f"first {len(host_sample)} tensors of the workload") +
                                  f" ({sample_params} weights), {args.mode}, {threads} threads over output channels",
                        "single_thread_value": round(p1 / cpu1_s / 1e9, 5),
                        "cpu_model": cpu_model(),
                        "gpu_mismatches_on_sample": mism}
        log(f"[bench] CPU reference: {sample_params / cpu_s / 1e6:.1f} Mparams/s on {threads} threads, "
            f"{p1 / cpu1_s / 1e6:.1f} Mparams/s on 1; GPU mismatches on the sample: {mism}")
        if mism:
            log("[bench] ERROR: GPU output differs from the CPU reference")

    out = {
        "metric": "Gparams/s quantized (4-bit, SQuant-EKC) + achieved HBM GB/s vs peak",
        "value": round(value, 2), "unit": "Gparams/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32+int32",
        "data": "synthetic",
        "config": {"workload": desc if args.shape else f"{args.workload}: {desc}", "bits": args.bits, "mode": args.mode,
                   "weight_type": args.wtype, "output": args.output,
                   "tensors": len(specs), "weights": n_params, "output_channels": n_channels,
                   "seed": synth.DEFAULT_SEED},
        "roofline": roofline, "cpu_baseline": cpu_baseline,
    }
    print(json.dumps(out), flush=True)
    return 1 if (cpu_baseline and cpu_baseline["gpu_mismatches_on_sample"]) else 0


if __name__ == "__main__":
    sys.exit(main())
