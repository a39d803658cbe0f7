#!/usr/bin/env python3
"""Benchmark of the Adasum tree combiner on one MI355X.

One "step" = one whole ``adasum_reduce`` (every tree level: Gram pass, finish,
weights, combine pass) over K synthetic worker gradients already resident in
HBM.  Default workload: K = 64 workers, BERT-Large-shaped (391 tensors,
335 141 888 elements), gradients stored bf16, bf16 result -- the configuration
the headline metric is quoted on.

Prints ONE JSON line: whole-job input GB/s (K*N*2 bytes / step time), the
roofline of the dominant kernel (algorithmic bytes / HIP-event duration against
the 8 TB/s HBM peak) and the CPU oracle timed on a bounded sample.
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

HBM_PEAK_GBS = 8000.0

# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc runs
# (FETCH_SIZE and WRITE_SIZE, scaled by a copy kernel of known size); see the
# summaries under profiles/.  Keyed by (workload, kernel name).
MEASURED_TRAFFIC_BYTES = {
    ("config4", "combine<bf16,f32,R=16>"): 43.234e9 + 5.795e9,
    ("config4", "gram<bf16,R=16,diag>"): 42.898e9 + 0.024e9,
    ("config4", "combine<bf16,f32,R=2>"): 43.571e9 + 43.066e9,
    ("config3", "combine<f32,f32,R=16>"): 21.617e9 + 1.341e9,
    ("config3", "gram<f32,R=16,diag>"): 21.450e9 + 0.025e9,
    ("config2", "combine<f32,f32,R=8>"): 0.8243e9 + 0.1022e9,
    ("config2", "gram<f32,R=8,diag>"): 0.8180e9 + 0.0006e9,
    # counters taken at K = 128 on config 4's generator (config 5 adds 16 one-element tensors to it)
    ("config5", "combine<bf16,f32,R=16>"): 86.468e9 + 11.586e9,
    ("config5", "gram<bf16,R=16,diag>"): 85.796e9 + 0.048e9,
}


def parse_args():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=10)
    p.add_argument("--warmup", type=int, default=2)
    p.add_argument("--workload", default="config4",
                   choices=["config1", "config2", "config3", "config4", "config5", "config4_small", "copy"])
    p.add_argument("--workers", type=int, default=0, help="override the workload's number of workers K")
    p.add_argument("--order", default="tree", choices=["tree", "linear"])
    p.add_argument("--radix", type=int, default=0, help="0 = library default")
    p.add_argument("--out-dtype", default="same", choices=["same", "f32", "bf16"])
    p.add_argument("--storage", default="same", choices=["same", "f16", "f64"],
                   help="convert the generated gradients to this storage type before timing")
    p.add_argument("--graph", action="store_true", help="replay the level ladder as one hipGraph launch")
    p.add_argument("--delta", action="store_true",
                   help="time the Adasum-after-optimizer form: the K buffers are parameters after a local step, "
                        "a starting-parameter buffer is subtracted on the fly and added back at the root")
    p.add_argument("--single-layer", action="store_true",
                   help="treat the whole buffer as one layer (isolates the cost of the layer structure)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--no-profile", action="store_true",
                   help="do not bracket kernels with HIP events in the timed region")
    return p.parse_args()


def make_workload(name, device, workers=0):
    from paper_2006_02924_amd import workloads as W
    kw = {"K": workers} if workers else {}
    if name == "config1":
        return W.config1(device)
    if name == "config2":
        return W.config2(device, **kw)
    if name == "config3":
        return W.config3(device, **kw)
    if name == "config4":
        return W.config4(device, **kw)
    if name == "config5":
        return W.config5(device, **kw)
    if name == "copy":
        # a plain copy of known size through the K = 1 path (reads N*4 bytes, writes N*4):
        # the yardstick that scales the FETCH_SIZE / WRITE_SIZE counters
        import torch
        n = 1 << 28
        g = torch.randn(n, device=device)
        # ... and the same copy done by a PyTorch elementwise kernel (y = g * 1), three times,
        # as a second yardstick that has no tile table or kernel-argument traffic
        y = torch.empty_like(g)
        for _ in range(3):
            torch.mul(g, 1.0, out=y)
        torch.cuda.synchronize()
        return W.Workload("copy", 1, torch.float32, [0, n], [g])
    if name == "config4_small":
        return W.config4(device, K=8, sizes=W.scaled_down(W.bert_large_layer_sizes(), 16, floor=64))
    raise ValueError(name)


def cpu_baseline(w, budget_elems=13_500_000):
    """The fp64 NumPy oracle, as it stands, on a bounded sample: the first layers
    of the same workload (all K workers) up to about `budget_elems` elements per
    worker, skipping any single layer larger than the budget."""
    import numpy as np
    from oracle import adasum_oracle as O
    try:
        from threadpoolctl import threadpool_limits
    except Exception:  # pragma: no cover
        threadpool_limits = None
    offs = w.layer_offsets
    layers, total = [], 0
    for l in range(w.n_layers):
        n = offs[l + 1] - offs[l]
        if n == 0 or n > budget_elems:
            continue
        if total + n > budget_elems:
            break
        layers.append(l)
        total += n
    host = [[g[offs[l]:offs[l + 1]].cpu() for g in w.grads] for l in layers]

    def run():
        t0 = time.perf_counter()
        for per_layer in host:
            O.adasum_tree([t.double().numpy() for t in per_layer])
        return time.perf_counter() - t0

    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            dt = run()
        cores = 1
    else:
        dt = run()
        cores = os.cpu_count() or 1
    in_bytes = total * w.K * w.grads[0].element_size()
    return {"value": in_bytes / dt / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"layers {layers[0]}..{layers[-1]} of {w.name} ({total} elements x K={w.K} workers, "
                      f"{in_bytes / 1e9:.2f} GB of input) in {dt:.1f} s, fp64 NumPy, input widening included"}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the K worker gradients are simulated buffers in one "
              "GPU's HBM); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2006_02924_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    B.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    t0 = time.perf_counter()
    w = make_workload(args.workload, dev, args.workers)
    torch.cuda.synchronize()
    print(f"[bench] {w.name}: K={w.K} N={w.N} layers={w.n_layers} dtype={w.dtype} "
          f"input={w.input_bytes / 1e9:.2f} GB generated in {time.perf_counter() - t0:.1f} s",
          file=sys.stderr, flush=True)
    if args.single_layer:
        w.layer_offsets = [0, w.N]
    if args.storage != "same":
        to = {"f16": torch.float16, "f64": torch.float64}[args.storage]
        for i in range(w.K):
            w.grads[i] = w.grads[i].to(to)
        w.dtype = to
        torch.cuda.synchronize()
    out_dtype = {"same": w.dtype, "f32": torch.float32, "bf16": torch.bfloat16}[args.out_dtype]
    out = torch.empty(w.N, dtype=out_dtype, device=dev)

    start = None
    if args.delta:
        start = (torch.randn(w.N, device=dev, dtype=torch.float32) * 0.02).to(w.dtype)

    def step():
        B.adasum_reduce(w.grads, w.layer_offsets, out, out_dtype=out_dtype, radix=args.radix,
                        use_graph=args.graph, delta_start=start,
                        order=B.ORDER_LINEAR if args.order == "linear" else B.ORDER_TREE)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    B.profile_collect()
    B.profile_enable(not args.no_profile)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    B.profile_enable(False)
    prof = B.profile_collect()

    ms_per_step = dt / args.steps * 1e3
    value = w.input_bytes / (dt / args.steps) / 1e9
    eight = args.delta or w.dtype == torch.float64     # these default to radix 8
    levels = B.plan_levels(w.K, args.radix if (args.radix or not eight) else 8) if args.order == "tree" else None

    roofline = None
    if prof:
        for k in prof:
            print(f"[bench] {k['name']:32s} launches={k['launches']:5d} avg={k['total_ms'] / k['launches']:9.4f} ms "
                  f"alg={k['bytes'] / max(k['total_ms'], 1e-9) / 1e6:8.1f} GB/s", file=sys.stderr, flush=True)
        dom = max(prof, key=lambda k: k["total_ms"])
        per_launch_bytes = dom["bytes"] / dom["launches"]
        avg_ms = dom["total_ms"] / dom["launches"]
        achieved = per_launch_bytes / (avg_ms * 1e-3) / 1e9
        total_bytes = sum(k["bytes"] for k in prof) / args.steps
        total_ms = sum(k["total_ms"] for k in prof) / args.steps
        roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS,
                    "traffic": MEASURED_TRAFFIC_BYTES.get((args.workload, dom["name"])),
                    "kernel": dom["name"], "kernel_avg_ms": avg_ms, "kernel_bytes_per_launch": per_launch_bytes,
                    "kernel_share_of_step": dom["total_ms"] / args.steps / ms_per_step,
                    "all_kernels_algorithmic_GBps": total_bytes / (total_ms * 1e-3) / 1e9,
                    "all_kernels_bytes_per_step": total_bytes}

    line = {
        "metric": "Adasum tree-reduce throughput: input GB/s and % of MI355X HBM peak",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64" if w.dtype == torch.float64 else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: K={w.K} workers, {w.n_layers} tensors, N={w.N} elements, "
                               f"stored {str(w.dtype).replace('torch.', '')}, output "
                               f"{str(out_dtype).replace('torch.', '')}",
                   "passes": levels, "radix": args.radix, "graph": bool(args.graph), "delta_form": bool(args.delta),
                   "order": args.order,
                   "input_GB": w.input_bytes / 1e9},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
