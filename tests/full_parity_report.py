#!/usr/bin/env python3
"""Every layer of one configuration against the CPU oracle, at full size, plus the
oracle's own time on this host: one row of the results table.

    python -m tests.full_parity_report --config 4 [--threads 16] [--out-dtype same|f32] [--radix 64]

The library reduces the workload once (default path, or the radix given: the launch
configuration bench.py times).  The oracle then reduces every layer from the stored bits copied
back from the device -- first on one thread, then as a plain parallel-for over
layers on `--threads` threads (NumPy's own threading pinned to 1) -- and each
layer's relative L2 error is taken.  Prints progress lines and ONE JSON line.
Not collected by pytest (it runs for minutes); needs a GPU.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, required=True, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--threads", type=int, default=16)
    ap.add_argument("--out-dtype", default="same", choices=["same", "f32"])
    ap.add_argument("--skip-single", action="store_true", help="only the parallel oracle pass")
    ap.add_argument("--radix", type=int, default=0, help="0 = library default")
    args = ap.parse_args()

    import torch
    from threadpoolctl import threadpool_limits

    from oracle import adasum_oracle as O
    from paper_2006_02924_amd import binding as B
    from paper_2006_02924_amd import workloads as W
    from tests import gpu_util as U

    dev = "cuda:0"
    w = getattr(W, f"config{args.config}")(dev)
    torch.cuda.synchronize()
    out_dtype = w.dtype if args.out_dtype == "same" else torch.float32
    print(f"[report] {w.name}: K={w.K} N={w.N} layers={w.n_layers} {w.dtype} -> {out_dtype}", flush=True)
    print(f"[report] radix {args.radix}: passes {B.plan_levels(w.K, args.radix)}", flush=True)
    out = B.adasum_reduce(w.grads, w.layer_offsets, out_dtype=out_dtype, radix=args.radix)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    reps = 5
    for _ in range(reps):
        B.adasum_reduce(w.grads, w.layer_offsets, out, out_dtype=out_dtype, radix=args.radix)
    torch.cuda.synchronize()
    gpu_ms = (time.perf_counter() - t0) / reps * 1e3
    got = U.to_f64(out)
    offs = list(w.layer_offsets)
    sizes = np.diff(np.asarray(offs))
    tol = U.tol_for(out_dtype)

    def layer_task(l):
        lo, hi = offs[l], offs[l + 1]
        if hi == lo:
            return l, 0.0, False
        parts = [g[lo:hi].cpu().double().numpy() for g in w.grads]
        ref = O.adasum_tree(parts)
        if hi - lo <= U.ILL_POSED_MAX_SIZE and U._node_is_ill_posed(parts, "tree"):
            return l, 0.0, True
        return l, float(O.rel_l2_per_layer(got[lo:hi], ref, [0, hi - lo])[0]), False

    def sweep(n_threads):
        t0 = time.perf_counter()
        with threadpool_limits(limits=1):
            if n_threads == 1:
                res = []
                for l in range(w.n_layers):
                    res.append(layer_task(l))
                    if l % 50 == 0:
                        print(f"[report]   layer {l} of {w.n_layers}, {time.perf_counter() - t0:.0f} s", flush=True)
            else:
                # largest layers first so the pool drains evenly
                order = sorted(range(w.n_layers), key=lambda l: -sizes[l])
                with ThreadPoolExecutor(n_threads) as pool:
                    res = list(pool.map(layer_task, order))
        return time.perf_counter() - t0, res

    t1 = None
    if not args.skip_single:
        t1, res = sweep(1)
        print(f"[report] oracle, 1 thread: {t1:.1f} s", flush=True)
    tn, res_n = sweep(args.threads)
    print(f"[report] oracle, {args.threads} threads: {tn:.1f} s", flush=True)
    if args.skip_single:
        res = res_n
    err = np.zeros(w.n_layers)
    skipped = []
    for l, e, ill in res:
        err[l] = e
        if ill:
            skipped.append(l)
    tols = np.full(w.n_layers, tol)
    if out_dtype in (torch.bfloat16, torch.float16):
        tiny = U.TOL_BF16_TINY if out_dtype == torch.bfloat16 else U.TOL_F16_TINY
        tols[sizes < U.TINY_LAYER] = max(tol, tiny)
    worst = int(np.argmax(err))
    big = sizes >= U.TINY_LAYER
    row = {
        "config": args.config, "K": w.K, "radix": args.radix, "passes": B.plan_levels(w.K, args.radix), "layers": w.n_layers, "layers_checked": int(w.n_layers - len(skipped)),
        "layers_without_reference": skipped, "out_dtype": str(out_dtype).replace("torch.", ""),
        "gpu_ms": gpu_ms, "input_GBps": w.input_bytes / gpu_ms / 1e6,
        "max_rel_l2": float(err.max()), "max_rel_l2_layer": worst, "max_rel_l2_layer_size": int(sizes[worst]),
        "max_rel_l2_layers_of_256_or_more": float(err[big].max()) if big.any() else None,
        "all_within_tolerance": bool(np.all(err <= tols)),
        "oracle_1_thread_s": t1, "oracle_n_thread_s": tn, "threads": args.threads,
        "host_cpus": os.cpu_count(),
    }
    print(json.dumps(row), flush=True)
    sys.exit(0 if row["all_within_tolerance"] else 1)


if __name__ == "__main__":
    main()
