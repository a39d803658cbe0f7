#!/usr/bin/env python3
"""Benchmark of the Adasum tree combiner on one MI355X.

One "step" = one whole ``adasum_reduce`` (every tree level: Gram pass, finish,
weights, combine pass) over K synthetic worker gradients already resident in
HBM.  Headline workload: K = 64 workers, BERT-Large-shaped (391 tensors,
335 141 888 elements), gradients stored bf16, bf16 result -- the configuration
the metric is quoted on.

Prints ONE JSON line: whole-job input GB/s (K*N*2 bytes / step time), the
roofline of the dominant kernel (algorithmic bytes / HIP-event duration against
the 8 TB/s HBM peak), the CPU oracle timed on a bounded sample (one thread and
all cores) and -- in the default run -- the same measurements for the other four
synthetic configurations and for the one-pair-per-level schedule (radix 2).
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_table.md")


def measured_traffic(workload: str, kernel: str):
    """HBM bytes per launch of `kernel` on `workload` from the tracked counter summary
    (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a copy kernel of known size).
    Rows of the table: | workload | kernel | read bytes | written bytes | dispatches | commit |."""
    try:
        text = open(TRAFFIC_TABLE).read()
    except OSError:
        return None
    for line in text.splitlines():
        cells = [c.strip().strip("`") for c in line.strip().strip("|").split("|")]
        if len(cells) >= 6 and cells[0] == workload and cells[1] == kernel:
            try:
                return {"bytes": float(cells[2]) + float(cells[3]), "read_bytes": float(cells[2]),
                        "written_bytes": float(cells[3]), "measured_at_commit": cells[5],
                        "source": "profiles/hbm_traffic_table.md"}
            except ValueError:
                return None
    return None


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
    p.add_argument("--fuse-siblings", action="store_true",
                   help="with --radix 2: the combine of a level also leaves the next level's dot products")
    p.add_argument("--separate-passes", action="store_true",
                   help="every pass makes a reduce pass of its own (no combine leaves the next pass's Gram matrix)")
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
    p.add_argument("--combine-norms-ab", action="store_true",
                   help="instead of a reduction: time the combine step alone (adasum_group_combine over the first 16 "
                        "workers of the workload, fp32 result) with and without the per-tile squared norms it can "
                        "leave, and print both")
    p.add_argument("--headline-only", action="store_true",
                   help="only the workload named by --workload: skip the other configurations "
                        "(they run by default when nothing but --steps / --warmup is given)")
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


def pair_per_level_bytes(K, N, in_bytes, out_bytes):
    """Bytes of the schedule that follows the paper's structure literally on one GPU: one pair per
    tree level, two passes over both operands per level (dot products and norms, then the
    scaled sum), fp32 tree nodes, the root stored in the output type.  K a power of two."""
    total, level, pairs = 0, 0, K // 2
    while pairs >= 1:
        s = in_bytes if level == 0 else 4
        so = out_bytes if pairs == 1 else 4
        total += pairs * N * (4 * s + so)
        pairs //= 2
        level += 1
    return float(total)


def cpu_baseline(w, budget_elems=40_000_000):
    """The fp64 NumPy oracle, as it stands, on a bounded sample: the first layers
    of the same workload (all K workers) up to about `budget_elems` elements per
    worker, skipping any single layer larger than a third of the budget.  Timed twice:
    on one thread, and as a plain parallel-for over the sample's layers on all host cores
    this process may use (NumPy's own threading pinned to one thread per worker)."""
    from concurrent.futures import ThreadPoolExecutor

    from oracle import adasum_oracle as O
    try:
        from threadpoolctl import threadpool_limits
    except Exception:  # pragma: no cover
        threadpool_limits = None
    offs = w.layer_offsets
    layers, total = [], 0
    for l in range(w.n_layers):
        n = offs[l + 1] - offs[l]
        if n == 0 or n > budget_elems // 3:
            continue
        if total + n > budget_elems:
            break
        layers.append(l)
        total += n
    host = [[g[offs[l]:offs[l + 1]].cpu() for g in w.grads] for l in layers]

    def one_layer(per_layer):
        return O.adasum_tree([t.double().numpy() for t in per_layer])

    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:  # pragma: no cover
        usable = os.cpu_count() or 1
    env_cap = os.environ.get("OMP_NUM_THREADS")
    threads = max(1, min(usable, int(env_cap)) if env_cap and env_cap.isdigit() else usable)
    in_bytes = total * w.K * w.grads[0].element_size()

    class _Unlimited:
        def __enter__(self):
            return self

        def __exit__(self, *a):
            return False

    limit1 = (lambda: threadpool_limits(limits=1)) if threadpool_limits is not None else _Unlimited
    with limit1():
        t0 = time.perf_counter()
        for per_layer in host:
            one_layer(per_layer)
        t1 = time.perf_counter() - t0
        order = sorted(range(len(host)), key=lambda i: -host[i][0].numel())
        t0 = time.perf_counter()
        with ThreadPoolExecutor(threads) as pool:
            list(pool.map(lambda i: one_layer(host[i]), order))
        tn = time.perf_counter() - t0
    sample = (f"layers {layers[0]}..{layers[-1]} of {w.name} except those over {budget_elems // 3} elements "
              f"({total} elements x K={w.K} workers, {in_bytes / 1e9:.2f} GB of input), fp64 NumPy, input widening "
              f"included: {t1:.1f} s on 1 thread, {tn:.1f} s on {threads} threads")
    return {"value": in_bytes / tn / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle", "sample": sample,
            "single_thread": {"value": in_bytes / t1 / 1e9, "unit": "GB/s", "cores": 1, "seconds": t1},
            "seconds": tn, "host_cpus": os.cpu_count()}


def timed_steps(B, w, out, *, out_dtype, radix, order, graph, start, steps, warmup, profile, fuse=False,
                separate=False):
    """`warmup` untimed steps, then exactly `steps` timed ones between device synchronisations.
    Returns (seconds for the timed steps, per-kernel HIP-event records or [])."""
    import torch

    def step():
        B.adasum_reduce(w.grads, w.layer_offsets, out, out_dtype=out_dtype, radix=radix,
                        use_graph=graph, delta_start=start, fuse_siblings=fuse, separate_passes=separate,
                        order=B.ORDER_LINEAR if order == "linear" else B.ORDER_TREE)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    B.profile_collect()
    B.profile_enable(profile)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    B.profile_enable(False)
    return dt, B.profile_collect()


def kernel_summary(prof, steps, ms_per_step, workload, verbose_tag=None):
    """Dominant kernel (most GPU time) against the HBM roofline, from HIP-event records."""
    if not prof:
        return None
    if verbose_tag is not None:
        for k in prof:
            print(f"[bench] {verbose_tag}{k['name']:32s} launches={k['launches']:5d} "
                  f"avg={k['total_ms'] / k['launches']:9.4f} ms "
                  f"alg={k['bytes'] / max(k['total_ms'], 1e-9) / 1e6:8.1f} GB/s", file=sys.stderr, flush=True)
    dom = max(prof, key=lambda k: k["total_ms"])
    per_launch_bytes = dom["bytes"] / dom["launches"]
    avg_ms = dom["total_ms"] / dom["launches"]
    achieved = per_launch_bytes / (avg_ms * 1e-3) / 1e9
    total_bytes = sum(k["bytes"] for k in prof) / steps
    total_ms = sum(k["total_ms"] for k in prof) / steps
    return {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS, "traffic": None,
            "kernel": dom["name"], "kernel_avg_ms": avg_ms, "kernel_bytes_per_launch": per_launch_bytes,
            "kernel_share_of_step": dom["total_ms"] / steps / ms_per_step,
            "all_kernels_algorithmic_GBps": total_bytes / (total_ms * 1e-3) / 1e9,
            "all_kernels_ms_per_step": total_ms,
            "schedule_bytes": total_bytes}


def run_other(B, name, *, radix=0, steps=10, warmup=2, w=None, fuse=False, separate=False, order="tree",
              delta=False):
    """One more configuration, default options: the step time from an event-free loop, the kernel
    breakdown from a second, event-bracketed loop of the same steps."""
    import torch
    dev = "cuda:0"
    own = w is None
    t0 = time.perf_counter()
    if own:
        w = make_workload(name, dev)
        torch.cuda.synchronize()
    gen_s = time.perf_counter() - t0
    out = torch.empty(w.N, dtype=w.dtype, device=dev)
    # the Adasum-after-optimizer form (Section 4.1): the buffers stand for parameters after a local step
    start = (torch.randn(w.N, device=dev, dtype=torch.float32) * 0.02).to(w.dtype) if delta else None
    kw = dict(out_dtype=w.dtype, radix=radix, order=order, graph=False, start=start, fuse=fuse, separate=separate)
    dt, _ = timed_steps(B, w, out, steps=steps, warmup=warmup, profile=False, **kw)
    ms = dt / steps * 1e3
    dtp, prof = timed_steps(B, w, out, steps=steps, warmup=0, profile=True, **kw)
    tag = f"{name}{' radix ' + str(radix) if radix else ''}{' sibling-fused' if fuse else ''}" \
          f"{' separate passes' if separate else ''}{' left-to-right order' if order == 'linear' else ''}" \
          f"{' after-optimizer form' if delta else ''}"
    roof = kernel_summary(prof, steps, dtp / steps * 1e3, name, verbose_tag=tag + ": ")
    es = w.grads[0].element_size()
    row = {"workload": f"{name}: K={w.K}, {w.n_layers} tensors, N={w.N}, stored and output "
                       f"{str(w.dtype).replace('torch.', '')}",
           "passes": B.plan_levels(w.K, radix if (radix or not delta) else 8) if order == "tree" else None,
           "steps": steps, "warmup": warmup,
           "ms_per_step": ms, "input_GBps": w.input_bytes / (ms * 1e-3) / 1e9, "input_GB": w.input_bytes / 1e9,
           "generated_in_s": gen_s}
    if roof is not None:
        row.update({"schedule_bytes": roof["schedule_bytes"],
                    "algorithmic_GBps": roof["schedule_bytes"] / (ms * 1e-3) / 1e9,
                    "step_frac_of_hbm_peak": roof["schedule_bytes"] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                    "dominant_kernel": roof["kernel"], "dominant_kernel_avg_ms": roof["kernel_avg_ms"],
                    "dominant_kernel_GBps": roof["achieved"], "dominant_kernel_frac": roof["frac"],
                    "ms_per_step_with_events": dtp / steps * 1e3})
        t = measured_traffic((name if not radix else f"{name}_radix{radix}") + ("_fused" if fuse else "")
                             + ("_separate" if separate else ""), roof["kernel"]) if (order == "tree" and not delta) else None
        row["dominant_kernel_traffic"] = t["bytes"] if t else None
    if w.K & (w.K - 1) == 0 and w.K > 1 and order == "tree" and not delta:
        row["pair_per_level_bytes"] = pair_per_level_bytes(w.K, w.N, es, es)
    del out, start
    if own:
        del w
    B.shutdown()
    gc.collect()
    torch.cuda.empty_cache()
    return row


def combine_norms_ab(B, w, steps, warmup):
    """The radix-16 combine step alone through the C-ABI, with and without the squared norms of the
    result per tile (the stores a later pass reads its diagonal from): what those stores cost."""
    import torch
    R = min(16, w.K)
    xs = w.grads[:R]
    weights = torch.full((w.n_layers, R), 1.0 / R, dtype=torch.float64, device=xs[0].device)
    out = torch.empty(w.N, dtype=torch.float32, device=xs[0].device)
    es = xs[0].element_size()
    res = {}
    for want in (True, False, True, False):
        for _ in range(warmup):
            B.adasum_group_combine(xs, w.layer_offsets, weights, out=out, out_dtype=torch.float32, want_sqnorm=want)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(steps):
            B.adasum_group_combine(xs, w.layer_offsets, weights, out=out, out_dtype=torch.float32, want_sqnorm=want)
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / steps
        res.setdefault(want, []).append(ms)
    nbytes = w.N * (R * es + 4)
    line = {"what": f"adasum_group_combine, R={R}, {w.name}, N={w.N}, {str(w.dtype).replace('torch.', '')} -> float32",
            "bytes_per_call": nbytes, "steps": steps,
            "with_norms_ms": res[True], "without_norms_ms": res[False],
            "with_norms_GBps": [nbytes / m / 1e6 for m in res[True]],
            "without_norms_GBps": [nbytes / m / 1e6 for m in res[False]],
            "note": "with norms the call also runs two small kernels that sum the per-tile norms per layer"}
    print(json.dumps(line), flush=True)


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
    plain = (args.workload == "config4" and not args.workers and args.order == "tree" and args.radix == 0
             and args.out_dtype == "same" and args.storage == "same" and not args.graph and not args.delta
             and not args.single_layer and not args.no_profile and not args.fuse_siblings
             and not args.separate_passes)
    with_others = plain and not args.headline_only
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
    if args.combine_norms_ab:
        combine_norms_ab(B, w, args.steps, args.warmup)
        return
    out = torch.empty(w.N, dtype=out_dtype, device=dev)

    start = None
    if args.delta:
        start = (torch.randn(w.N, device=dev, dtype=torch.float32) * 0.02).to(w.dtype)

    dt, prof = timed_steps(B, w, out, out_dtype=out_dtype, radix=args.radix, order=args.order, graph=args.graph,
                           start=start, steps=args.steps, warmup=args.warmup, profile=not args.no_profile,
                           fuse=args.fuse_siblings, separate=args.separate_passes)

    ms_per_step = dt / args.steps * 1e3
    value = w.input_bytes / (dt / args.steps) / 1e9
    eight = args.delta or w.dtype == torch.float64     # these default to radix 8
    levels = B.plan_levels(w.K, args.radix if (args.radix or not eight) else 8) if args.order == "tree" else None

    roofline = kernel_summary(prof, args.steps, ms_per_step, args.workload, verbose_tag="")
    if roofline is not None:
        key = (args.workload if not args.radix else f"{args.workload}_radix{args.radix}") + \
              ("_fused" if args.fuse_siblings else "") + ("_separate" if args.separate_passes else "")
        t = measured_traffic(key, roofline["kernel"]) if (args.order == "tree" and not args.delta) else None
        if t is not None:
            roofline["traffic"] = t["bytes"]
            roofline["traffic_detail"] = t
        # the whole step against the same peak, on the bytes this schedule moves ...
        roofline["step_algorithmic_GBps"] = roofline["schedule_bytes"] / (ms_per_step * 1e-3) / 1e9
        roofline["step_frac"] = roofline["step_algorithmic_GBps"] / HBM_PEAK_GBS
        # ... which are fewer than those of one pair per level and two passes per level
        if w.K > 1 and w.K & (w.K - 1) == 0 and args.order == "tree" and not args.delta:
            ppl = pair_per_level_bytes(w.K, w.N, w.grads[0].element_size(), out.element_size())
            roofline["pair_per_level_bytes"] = ppl
            roofline["schedule_over_pair_per_level"] = roofline["schedule_bytes"] / ppl

    line = {
        "metric": "Adasum tree-reduce throughput: input GB/s and % of MI355X HBM peak",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64" if w.dtype == torch.float64 else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: K={w.K} workers, {w.n_layers} tensors, N={w.N} elements, "
                               f"stored {str(w.dtype).replace('torch.', '')}, output "
                               f"{str(out_dtype).replace('torch.', '')}",
                   "passes": levels, "radix": args.radix, "graph": bool(args.graph), "delta_form": bool(args.delta),
                   "order": args.order, "fuse_siblings": bool(args.fuse_siblings),
                   "separate_passes": bool(args.separate_passes),
                   "input_GB": w.input_bytes / 1e9},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        t0 = time.perf_counter()
        line["cpu_baseline"] = cpu_baseline(w)
        print(f"[bench] cpu baseline in {time.perf_counter() - t0:.1f} s", file=sys.stderr, flush=True)

    if with_others:
        others = []
        del out
        B.shutdown()
        torch.cuda.empty_cache()
        # the one-pair-per-level schedule on the headline workload, then the other four configurations
        # (the headline workload is dropped before the first of them is generated)
        # (name, radix, steps, warm-up, fuse_siblings, separate_passes); the first five reuse the headline
        # buffers (radix 64 and 32: the opt-in wide first pass, whose Gram matrix comes from the matrix cores)
        # (the sixth and seventh: the left-to-right order of Section 3.4 and the after-optimizer form of
        # Section 4.1 on the headline buffers)
        todo = [("config4", 64, 20, 5, False, False), ("config4", 32, 20, 5, False, False),
                ("config4", 0, 20, 5, False, True), ("config4", 2, 10, 2, False, True), ("config4", 2, 10, 2, True, False),
                ("config4", 0, 10, 2, False, False, "linear"), ("config4", 0, 10, 2, False, False, "tree", True),
                ("config1", 0, 200, 20, False, False), ("config2", 0, 50, 5, False, False),
                ("config3", 0, 20, 3, False, False), ("config5", 0, 10, 2, False, False),
                ("config5", 64, 10, 2, False, False)]
        w5 = None
        for item in todo:
            name, radix, steps, warmup, fuse, separate = item[:6]
            order = item[6] if len(item) > 6 else "tree"
            delta = item[7] if len(item) > 7 else False
            reuse = w if name == "config4" else w5 if (name == "config5" and radix) else None
            if name != "config4" and w is not None:
                w = None
                gc.collect()
                torch.cuda.empty_cache()
            if name == "config5" and w5 is None:
                w5 = reuse = make_workload("config5", "cuda:0")
                torch.cuda.synchronize()
            try:
                t0 = time.perf_counter()
                row = run_other(B, name, radix=radix, steps=steps, warmup=warmup, w=reuse, fuse=fuse, separate=separate,
                                order=order, delta=delta)
                print(f"[bench] {name}{f' radix {radix}' if radix else ''}{' sibling-fused' if fuse else ''}"
                      f"{' separate passes' if separate else ''}{' left-to-right order' if order == 'linear' else ''}"
                      f"{' after-optimizer form' if delta else ''}: "
                      f"{row['ms_per_step']:.4f} ms/step, "
                      f"{row['input_GBps']:.0f} GB/s of input ({time.perf_counter() - t0:.1f} s in all)",
                      file=sys.stderr, flush=True)
            except Exception as exc:  # keep the headline line whatever happens here
                row = {"workload": name, "error": f"{type(exc).__name__}: {exc}"}
            del reuse
            if radix or separate or order != "tree" or delta:
                row["radix"] = radix
                row["fuse_siblings"] = fuse
                row["separate_passes"] = separate
                row["order"] = order
                row["delta_form"] = delta
            others.append(row)
        line["other_configs"] = others
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
