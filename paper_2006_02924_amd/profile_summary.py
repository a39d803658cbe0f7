"""Turns rocprofv3 CSV output of a ``bench.py`` run into the short summaries kept under
``profiles/``.  Reads files only; nothing here touches a GPU.

    python -m paper_2006_02924_amd.profile_summary counters  <..._counter_collection.csv>
        per library kernel: dispatches and the mean of every counter in the file
    python -m paper_2006_02924_amd.profile_summary stats     <..._kernel_stats.csv>
        the library's kernels of a --kernel-trace --stats run as a markdown table
    python -m paper_2006_02924_amd.profile_summary traffic --workload config4 --commit <hash> \\
            --fetch <FETCH_SIZE csv> --write <WRITE_SIZE csv> --copy-fetch <csv> --copy-write <csv>
        rows of profiles/hbm_traffic_table.md: HBM bytes per dispatch of each streaming kernel
        (| workload | kernel | read bytes | written bytes | dispatches averaged | commit |).
        FETCH_SIZE / WRITE_SIZE count in units that a plain copy of known size calibrates: the
        --copy-* files come from ``bench.py --workload copy``, whose PyTorch kernel y = g * 1
        reads and writes exactly 2^30 bytes per dispatch.
"""
from __future__ import annotations

import argparse
import collections
import csv
import re
import sys

TYPES = {"adasum::(anonymous namespace)::bf16_t": "bf16", "adasum::(anonymous namespace)::f16_t": "f16",
         "bf16_t": "bf16", "f16_t": "f16", "float": "f32", "double": "f64"}
COPY_BYTES = float(1 << 30)


def library_name(kernel_name: str):
    """The name bench.py prints for a kernel ("combine<bf16,f32,R=16>"), from rocprofv3's
    demangled one; None for kernels that are not the library's."""
    if "adasum" not in kernel_name:
        return None
    m = re.search(r"(\w+)_kernel(?:<(.*?)>)?\(", kernel_name)
    if not m:
        return None
    kind, targs = m.group(1), m.group(2)
    args = [a.strip() for a in targs.split(",")] if targs else []
    args = [TYPES.get(a, a.replace("adasum::(anonymous namespace)::", "")) for a in args]
    if kind == "gram" and len(args) >= 4:
        head = "+f32 head" if len(args) >= 6 and args[5] == "true" else ""
        delta = " (delta)" if args[3] == "true" else ""
        return f"gram<{args[0]},R={args[1]},{'diag' if args[2] == 'true' else 'offdiag'}>{head}{delta}"
    if kind == "combine" and len(args) >= 3:
        head = "+f32 head" if len(args) >= 5 and args[4] == "true" else ""
        delta = " (delta)" if len(args) >= 4 and args[3] == "true" else ""
        return f"combine<{args[0]},{args[1]},R={args[2]}>{head}{delta}"
    if kind == "combine_siblings" and len(args) >= 2:
        return f"combine<{args[0]},{args[1]},R=2>+dot"
    if kind == "gram_wide" and len(args) >= 2:
        return f"gram<{args[0]},R={args[1]},diag>"
    if kind == "combine_wide" and len(args) >= 3:
        return f"combine<{args[0]},{args[1]},R={args[2]}>"
    if kind == "gram_finish_wide" and len(args) >= 1:
        return f"gram_finish<R={args[0]},diag>"
    if kind == "combine_feed" and len(args) >= 4:
        return f"combine<{args[0]},{args[1]},R={args[2]}>+gram{args[3]}"
    if kind == "gram_finish" and len(args) >= 2:
        return f"gram_finish<R={args[0]},{'diag' if args[1] == 'true' else 'offdiag'}>"
    if kind == "parts_coarsen":
        return "gram_from_combine"       # (the name bench.py times that launch under)
    return kind + (f"<{','.join(args)}>" if args else "")


def read_counters(path):
    """{(library kernel name, grid size): {counter: (dispatches, mean)}} in dispatch order, plus
    the PyTorch copy yardstick under the name 'torch_copy'."""
    acc = collections.OrderedDict()
    with open(path, newline="") as f:
        for row in csv.DictReader(f):
            name = library_name(row["Kernel_Name"])
            if name is None:
                k = row["Kernel_Name"]
                if "elementwise" in k and "Mul" in k and int(row["Grid_Size"]) >= (1 << 24):
                    name = "torch_copy"
                else:
                    continue
            a = acc.setdefault((name, int(row["Grid_Size"])), collections.OrderedDict())
            c = a.setdefault(row["Counter_Name"], [0, 0.0])
            c[0] += 1
            c[1] += float(row["Counter_Value"])
    return acc


def cmd_counters(args):
    for (name, grid), counters in read_counters(args.csv).items():
        for cname, (n, tot) in counters.items():
            print(f"{name:40s} grid={grid:>11d} {cname:24s} dispatches={n:4d} mean={tot / n:18.3f}")


def cmd_stats(args):
    print("| kernel | calls | avg ms | min ms | max ms |\n|---|---|---|---|---|")
    with open(args.csv, newline="") as f:
        for r in csv.DictReader(f):
            name = library_name(r["Name"] if "(" in r["Name"] else r["Name"] + "(")
            if name is None:
                continue
            print(f"| `{name}` | {int(r['Calls'])} | {float(r['AverageNs']) / 1e6:.4f} | "
                  f"{float(r['MinNs']) / 1e6:.4f} | {float(r['MaxNs']) / 1e6:.4f} |")


def _yardstick(path, counter):
    for (name, _grid), counters in read_counters(path).items():
        if name == "torch_copy" and counter in counters:
            n, tot = counters[counter]
            return COPY_BYTES / (tot / n)      # bytes per counter unit
    raise SystemExit(f"{path}: no PyTorch copy kernel with {counter}")


def cmd_traffic(args):
    fetch_unit = _yardstick(args.copy_fetch, "FETCH_SIZE")
    write_unit = _yardstick(args.copy_write, "WRITE_SIZE")
    print(f"<!-- yardstick: one FETCH_SIZE unit = {fetch_unit:.3f} bytes, one WRITE_SIZE unit = {write_unit:.3f} bytes "
          f"(PyTorch y = g * 1 over 2^28 fp32: 2^30 bytes each way) -->")
    # per kernel name: the mean over all its dispatches (a name launched at several sizes in one
    # step, as the pair passes of radix 2 are, gets the mean over those sizes, like bench.py's
    # per-launch averages)
    def by_name(path, counter):
        acc = collections.OrderedDict()
        for (name, _grid), counters in read_counters(path).items():
            if counter in counters and (name.startswith("gram<") or name.startswith("combine<")):
                a = acc.setdefault(name, [0, 0.0])
                a[0] += counters[counter][0]
                a[1] += counters[counter][1]
        return acc
    fetch = by_name(args.fetch, "FETCH_SIZE")
    write = by_name(args.write, "WRITE_SIZE")
    for name, (n, tot) in fetch.items():
        if name not in write:
            continue
        rd = tot / n * fetch_unit
        wr = write[name][1] / write[name][0] * write_unit
        print(f"| {args.workload} | `{name}` | {rd:.4e} | {wr:.4e} | {n} | {args.commit} |")


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    c = sub.add_parser("counters")
    c.add_argument("csv")
    c.set_defaults(fn=cmd_counters)
    s = sub.add_parser("stats")
    s.add_argument("csv")
    s.set_defaults(fn=cmd_stats)
    t = sub.add_parser("traffic")
    t.add_argument("--workload", required=True)
    t.add_argument("--commit", required=True)
    for name in ("fetch", "write", "copy-fetch", "copy-write"):
        t.add_argument(f"--{name}", required=True)
    t.set_defaults(fn=cmd_traffic)
    args = ap.parse_args(argv)
    args.fn(args)


if __name__ == "__main__":
    main()
    sys.exit(0)
