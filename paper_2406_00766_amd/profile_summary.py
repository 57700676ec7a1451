"""Turn rocprofv3 CSV output into the short text summaries kept under profiles/ (and read back by bench.py).

    python -m paper_2406_00766_amd.profile_summary stats    <*_kernel_stats.csv> <out.txt> --command "..." [--note "..."]
    python -m paper_2406_00766_amd.profile_summary counters <out.txt> --workload NAME --K K --command "..." \
           NAME=<*_counter_collection.csv> [NAME=<csv> ...]          # one CSV per --pmc run (one counter group each)

`counters` groups the dispatches by kernel class (the classes of pc_profile_read) and prints, per class and counter,
the value per launch; lines start with "class=" and are parsed by read_counters().  With FETCH_SIZE and WRITE_SIZE
(KiB per dispatch) it adds the HBM bytes per launch, each counter scaled by what it read for bench.py's plain
256 MiB copy kernel in the same run.
"""
import argparse
import collections
import csv
import re
import sys


def kernel_class(name: str) -> str:
    """Kernel class (as reported by pc_profile_read) of a demangled kernel name."""
    n = name.replace("void ", "").replace("pc::", "")
    m = re.match(r"k_sum_mfma<\s*\d+,\s*\d+,\s*\d+,\s*(true|false)", n)
    if m:
        return "sum_bwd_child" if m.group(1) == "true" else "sum_fwd"
    m = re.match(r"k_sum_bf16<\s*\d+,\s*\d+,\s*(true|false)", n)
    if m:
        return "sum_bwd_child" if m.group(1) == "true" else "sum_fwd"
    for prefix, cls in (("k_split_", "split"), ("k_sum_fwd", "sum_fwd"), ("k_sum_bwd_child", "sum_bwd_child"), ("k_sum_bwd_small", "sum_bwd_child"),
                        ("k_sum_bwd_param", "sum_bwd_param"), ("k_param_flow", "sum_bwd_param"), ("k_prod_fwd", "prod_fwd"),
                        ("k_prod_bwd", "prod_bwd"), ("k_input_fwd", "input_fwd"), ("k_input_bwd", "input_bwd"), ("k_em_", "em"),
                        ("k_measure_copy", "measure_copy"), ("k_measure_mfma", "measure_mfma")):
        if n.startswith(prefix):
            return cls
    return "misc"


def write_stats(src, dst, command, note):
    rows = list(csv.DictReader(open(src)))
    with open(dst, "w") as f:
        f.write("rocprofv3 kernel-trace statistics (summary of *_kernel_stats.csv)\n")
        f.write("command (run from /tmp with TMPDIR=/tmp on the MI355X box):\n  " + command + "\n")
        if note:
            f.write(note + "\n")
        f.write("\n%-90s %-14s %7s %12s %12s %7s\n" % ("kernel", "class", "calls", "total_ms", "avg_us", "pct"))
        for r in rows:
            if float(r["Percentage"]) < 0.01:
                continue
            name = r["Name"].split("(")[0].replace("void ", "")
            f.write("%-90s %-14s %7s %12.3f %12.2f %7.2f\n" % (name, kernel_class(name), r["Calls"], float(r["TotalDurationNs"]) / 1e6,
                                                              float(r["AverageNs"]) / 1e3, float(r["Percentage"])))


def read_counter_csv(path):
    """{(class, counter): [sum of values, dispatches]} and {class: set of kernel names} from one counter_collection CSV."""
    agg = collections.defaultdict(lambda: [0.0, 0])
    names = collections.defaultdict(set)
    seen = collections.defaultdict(set)
    for r in csv.DictReader(open(path)):
        kname = r["Kernel_Name"].split("(")[0].replace("void ", "")
        cls = kernel_class(kname)
        names[cls].add(kname.replace("pc::", ""))
        ctr = r["Counter_Name"]
        a = agg[(cls, ctr)]
        a[0] += float(r["Counter_Value"])
        key = (r.get("Dispatch_Id"), ctr)
        if key not in seen[cls]:                      # one row per dispatch and counter (per-XCC rows add up)
            seen[cls].add(key)
            a[1] += 1
    return agg, names


def write_counters(dst, workload, K, command, runs, note):
    per = collections.defaultdict(dict)               # class -> counter -> (per launch, launches)
    names = collections.defaultdict(set)
    for label, path in runs:
        agg, nm = read_counter_csv(path)
        for (cls, ctr), (tot, n) in agg.items():
            per[cls][ctr] = (tot / max(n, 1), n)
        for cls, s in nm.items():
            names[cls] |= s
    with open(dst, "w") as f:
        f.write(f"rocprofv3 --pmc counters per kernel class (summary of *_counter_collection.csv)\n")
        f.write(f"workload={workload} K={K}\n")
        f.write("commands (run from /tmp with TMPDIR=/tmp on the MI355X box), one counter group per run:\n")
        for line in command:
            f.write("  " + line + "\n")
        if note:
            f.write(note + "\n")
        scale = counter_scale(per)
        if "measure_copy" in per and "FETCH_SIZE" in per["measure_copy"]:
            f.write(f"scale factors from the calibration copy (256 MiB read, 256 MiB written per launch): "
                    f"FETCH_SIZE x {scale[0]:.3f}, WRITE_SIZE x {scale[1]:.3f}; hbm_bytes_per_launch applies them\n")
        f.write("\nper launch (value summed over the chip, divided by the dispatches of the class):\n")
        for cls in sorted(per, key=lambda c: -per[c].get("FETCH_SIZE", per[c].get("SQ_BUSY_CU_CYCLES", (0, 0)))[0]):
            if cls in ("misc",):
                continue
            vals = per[cls]
            launches = max(n for _, n in vals.values())
            f.write(f"class={cls} launches={launches}")
            for ctr in sorted(vals):
                f.write(f" {ctr}={vals[ctr][0]:.6g}")
            d = derived(vals, scale)
            for k, v in d.items():
                f.write(f" {k}={v:.4g}")
            f.write("\n    kernels: " + ", ".join(sorted(names[cls])) + "\n")


COPY_KIB = 256.0 * 1024          # bench.py's calibration kernel (class measure_copy) reads and writes 256 MiB per launch


def derived(vals, scale=(1.0, 1.0)):
    """HBM bytes per launch from FETCH_SIZE / WRITE_SIZE (KiB per dispatch), each scaled by what the same counter read
    for the plain copy kernel of known size in the same run."""
    out = {}
    if "FETCH_SIZE" in vals and "WRITE_SIZE" in vals:
        out["hbm_bytes_per_launch"] = (vals["FETCH_SIZE"][0] * scale[0] + vals["WRITE_SIZE"][0] * scale[1]) * 1024.0
    return out


def counter_scale(per):
    """(fetch factor, write factor) = known size of the calibration copy / what the counters read for it."""
    c = per.get("measure_copy", {})
    f = COPY_KIB / c["FETCH_SIZE"][0] if c.get("FETCH_SIZE", (0,))[0] else 1.0
    w = COPY_KIB / c["WRITE_SIZE"][0] if c.get("WRITE_SIZE", (0,))[0] else 1.0
    return f, w


def read_counters(path):
    """Parse a file written by write_counters: ({'workload':..., 'K':...}, {class: {name: float}})."""
    head, out = {}, {}
    for line in open(path):
        if line.startswith("workload="):
            for tok in line.split():
                k, _, v = tok.partition("=")
                head[k] = v
        elif line.startswith("class="):
            d = {}
            cls = None
            for tok in line.split():
                k, _, v = tok.partition("=")
                if k == "class":
                    cls = v
                else:
                    try:
                        d[k] = float(v)
                    except ValueError:
                        pass
            out[cls] = d
    return head, out


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    a = sub.add_parser("stats")
    a.add_argument("src"); a.add_argument("dst"); a.add_argument("--command", required=True); a.add_argument("--note", default="")
    b = sub.add_parser("counters")
    b.add_argument("dst"); b.add_argument("--workload", required=True); b.add_argument("--K", required=True)
    b.add_argument("--command", action="append", required=True); b.add_argument("--note", default="")
    b.add_argument("runs", nargs="+", help="LABEL=path/to/counter_collection.csv")
    args = ap.parse_args()
    if args.cmd == "stats":
        write_stats(args.src, args.dst, args.command, args.note)
    else:
        runs = [tuple(r.split("=", 1)) for r in args.runs]
        write_counters(args.dst, args.workload, args.K, args.command, runs, args.note)


if __name__ == "__main__":
    main()
