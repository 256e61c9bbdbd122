#!/usr/bin/env python3
"""Throughput of the SQuant solver on one MI355X.

A step is one pass of the whole path (absmax scale, SQuant-E, SQuant-K, candidate update,
SQuant-C, int8 emit) over the whole workload, as ONE batched library call, with the
weights already resident in HBM.  Prints one JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5|c1|c2|c3|c4] [--bits 4]

Every step is bracketed by a pair of events on the stream the library launches on, so the
kernel time of each single step is known; `steps` and `warmup` are what the command line says.
The defaults (3 warm-up steps, 20 timed ones) are a cold protocol: the first tens of launches
after an idle period run while the GPU settles its clocks, which is what a one-shot
quantization of a network sees.  A long warm-up (--warmup 100) shows the settled rate.
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


def timed_steps(torch, step, warmup: int, steps: int):
    """`warmup` untimed steps, then `steps` timed ones: wall time per step (synchronised on both
    sides) and the elapsed time of every single step between two events recorded on the stream
    the library launches on (torch's current stream)."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for e0, e1 in ev:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    return elapsed * 1e3 / max(steps, 1), [e0.elapsed_time(e1) for e0, e1 in ev]


def algorithmic_bytes(n_params: int, n_channels: int, wtype: str, output: str) -> float:
    """Bytes read + written per weight (4 + 1 in the headline configuration), 4 B per scale."""
    in_bytes = {"f32": 4.0, "f16": 2.0, "bf16": 2.0}[wtype]
    out_bytes = {"int8": 1.0, "int4": 0.5, "f32": 4.0, "bf16": 2.0}[output]
    return (in_bytes + out_bytes) * n_params + 4.0 * n_channels


def spread(np, kernel_ms):
    k = np.asarray(kernel_ms, dtype=np.float64)
    return {"kernel_ms_avg": round(float(k.mean()), 4), "kernel_ms_median": round(float(np.median(k)), 4),
            "kernel_ms_min": round(float(k.min()), 4), "kernel_ms_p10": round(float(np.percentile(k, 10)), 4),
            "kernel_ms_p90": round(float(np.percentile(k, 90)), 4), "kernel_ms_max": round(float(k.max()), 4)}


def extra_line(torch, np, sq, name, dws, n_params, n_channels, wtype, output, bits, warmup, steps):
    """One secondary configuration: same protocol, its own algorithmic bytes and fraction."""
    plan = sq.BatchPlan(dws, sq.OUTPUTS[output])
    ms_per_step, kernel_ms = timed_steps(torch, lambda: plan.run(bits, sq.MODE_EKC), warmup, steps)
    algo = algorithmic_bytes(n_params, n_channels, wtype, output)
    k_avg = float(np.mean(kernel_ms))
    out = {"name": name, "weight_type": wtype, "output": output, "bits": bits, "mode": "EKC",
           "weights": n_params, "ms_per_step": round(ms_per_step, 4),
           "gparams_per_s": round(n_params / (ms_per_step * 1e-3) / 1e9, 2),
           "algorithmic_bytes_per_launch": algo,
           "achieved_gbs": round(algo / (k_avg * 1e-3) / 1e9, 1),
           "frac": round(algo / (k_avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    out.update(spread(np, kernel_ms))
    log(f"[bench] extra {name}: kernel avg {k_avg:.4f} ms, {out['achieved_gbs']:.0f} GB/s "
        f"({100 * out['frac']:.1f}% of peak)")
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3, help="untimed steps first")
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
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the secondary configurations reported under \"extra\"")
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

    ms_per_step, kernel_ms = timed_steps(torch, lambda: plan.run(args.bits, mode), args.warmup, args.steps)
    value = n_params / (ms_per_step * 1e-3) / 1e9
    k_avg_ms = float(np.mean(kernel_ms))
    algo_bytes = algorithmic_bytes(n_params, n_channels, args.wtype, args.output)
    achieved = algo_bytes / (k_avg_ms * 1e-3) / 1e9
    headline_io = args.output == "int8" and args.wtype == "f32"
    traffic = (load_traffic()
               if args.workload == "c5" and args.tensors is None and headline_io else None)
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "kernel": "squant solver kernel(s) of the batched call, event pair around every step",
                "algorithmic_bytes_per_launch": algo_bytes}
    roofline.update(spread(np, kernel_ms))
    roofline["kernel_ms_steps"] = [round(float(v), 4) for v in kernel_ms]
    log(f"[bench] {ms_per_step:.4f} ms/step wall, kernel avg {k_avg_ms:.4f} ms -> "
        f"{value:.1f} Gparams/s, {achieved:.0f} GB/s algorithmic ({100 * achieved / HBM_PEAK_GBS:.1f}% of peak)")
    log("[bench] kernel ms per step: " + " ".join(f"{v:.3f}" for v in kernel_ms))

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
                        "single_thread_sample": f"first {n1} tensors of the sample ({p1} weights), 1 thread",
                        "cpu_model": cpu_model(),
                        "gpu_mismatches_on_sample": mism}
        log(f"[bench] CPU reference: {sample_params / cpu_s / 1e6:.1f} Mparams/s on {threads} threads, "
            f"{p1 / cpu1_s / 1e6:.1f} Mparams/s on 1; GPU mismatches on the sample: {mism}")
        if mism:
            log("[bench] ERROR: GPU output differs from the CPU reference")

    # ---- secondary configurations (same protocol; headline fields above are unaffected) ----
    extra = []
    if not args.no_extra and args.workload == "c5" and not args.shape and args.tensors is None \
            and headline_io and args.mode == "EKC" and args.bits == 4:
        del plan
        extra.append(extra_line(torch, np, sq, "c5, float32 weights -> packed 4-bit codes", dws, n_params,
                                n_channels, "f32", "int4", 4, args.warmup, args.steps))
        d16 = [w.to(torch.float16) for w in dws]
        del dws
        extra.append(extra_line(torch, np, sq, "c5, binary16 weights -> int8 codes", d16, n_params,
                                n_channels, "f16", "int8", 4, args.warmup, args.steps))
        del d16
        torch.cuda.empty_cache()
        for wl, bits in (("c2", 4), ("c3", 4), ("c3", 8), ("c4", 4)):
            sp = synth.config_specs(WORKLOADS[wl][0])
            ws = [torch.from_numpy(synth.generate(s_)).to(dev) for s_ in sp]
            extra.append(extra_line(torch, np, sq, f"{wl} layer set ({len(sp)} tensors, cache resident), {bits} bit",
                                    ws, sum(s_.numel for s_ in sp), sum(s_.shape[0] for s_ in sp),
                                    "f32", "int8", bits, args.warmup, args.steps))

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
        "roofline": roofline, "cpu_baseline": cpu_baseline, "extra": extra,
    }
    print(json.dumps(out), flush=True)
    return 1 if (cpu_baseline and cpu_baseline["gpu_mismatches_on_sample"]) else 0


if __name__ == "__main__":
    sys.exit(main())
