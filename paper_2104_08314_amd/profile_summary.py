"""Condense rocprofv3 CSV output into the short text summaries kept under profiles/.

Inputs are directories written by
    rocprofv3 --kernel-trace --stats --output-format csv -d <stats_dir> -- python3 bench.py ...
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <fetch_dir> -- python3 bench.py ... --calibrate-copy
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <write_dir> -- python3 bench.py ... --calibrate-copy
The counter runs hold a plain elementwise kernel of known size (bench.py --calibrate-copy); the
FETCH_SIZE / WRITE_SIZE readings of every other kernel are scaled by known bytes / reading of
that kernel.  Lines `traffic_bytes_per_launch[<kernel>]: <bytes>` are what bench.py reads back.
"""
import argparse
import csv
import glob
import os
import re
import sys
from collections import defaultdict

csv.field_size_limit(1 << 30)

OURS = ("encode_kernel", "encode_small_kernel", "encode_channel_kernel", "encode_channel64_kernel", "column_table_kernel", "conv_prologue_kernel", "conv_prologue_wave_kernel",
        "zero_fill_kernel", "spmv_conv_tile_kernel", "spmv_conv_strip_kernel", "spmv_conv_runs_kernel",
        "spmv_conv_lds_kernel", "reduce_transpose_kernel", "im2col_lower_kernel", "im2col_lower_direct_kernel",
        "gemm_f32_kernel", "gemm_bf16_kernel", "splitk_reduce_kernel", "prepare_weights_kernel", "prepare_weights_bf16_kernel")


def _find(directory, suffix):
    hits = sorted(glob.glob(os.path.join(directory, "**", "*" + suffix), recursive=True))
    if not hits:
        sys.exit(f"profile_summary: no *{suffix} under {directory}")
    return hits


def short_name(name):
    """Kernel name without template arguments, parameters, namespaces or _kernel suffix.  The three
    encoders keep their names (encode: column bands; encode_channel / encode_channel64: a workgroup
    per channel, the latter for maps up to 64 x 64 padded cells; encode_small: a wavefront per
    channel - the library's timing aid calls all of them encode), a
    publish-only instantiation gets _count appended; the lowering kernels are named for their
    output type, the direct one (small launches) with _direct appended."""
    name = name.replace("(anonymous namespace)::", "")
    base = re.split(r"[<(]", name, 1)[0].replace("void ", "").split("::")[-1].strip()
    short = base[:-len("_kernel")] if base.endswith("_kernel") else base
    if short in ("encode", "encode_channel", "encode_channel64", "encode_small"):
        m = re.search(r"_kernel<\(?(?:[\w:]+\))?\s*(\w+)", name)
        return short + "_count" if (m and m.group(1) == "1") else short
    if short in ("im2col_lower", "im2col_lower_direct"):
        m = re.search(r"_kernel<\s*(\w+)", name)
        kind = "bf16" if (m and m.group(1) in ("true", "1")) else "f32"
        return "im2col_lower_" + kind + ("_direct" if short.endswith("direct") else "")
    return short


def kernel_stats(directory):
    rows = []
    for path in _find(directory, "kernel_stats.csv"):
        with open(path, newline="") as f:
            for r in csv.DictReader(f):
                rows.append((short_name(r["Name"]), int(r["Calls"]), float(r["AverageNs"]), float(r["TotalDurationNs"]),
                             float(r["MinNs"]), float(r["MaxNs"]), r["Name"]))
    return rows


def counter_means(directory, counter):
    total, n, grids = defaultdict(float), defaultdict(int), {}
    for path in _find(directory, "counter_collection.csv"):
        with open(path, newline="") as f:
            for r in csv.DictReader(f):
                if r["Counter_Name"] != counter:
                    continue
                k = short_name(r["Kernel_Name"])
                if "elementwise" in r["Kernel_Name"]:
                    m = re.search(r"(\w+Functor)<\w+> *>", r["Kernel_Name"])
                    k = "elementwise[%s,grid=%s]" % (m.group(1) if m else "?", r["Grid_Size"])
                total[k] += float(r["Counter_Value"])
                n[k] += 1
    return {k: (total[k] / n[k], n[k]) for k in total}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--stats", help="directory of the --kernel-trace --stats run")
    ap.add_argument("--fetch", help="directory of the --pmc FETCH_SIZE run")
    ap.add_argument("--write", help="directory of the --pmc WRITE_SIZE run")
    ap.add_argument("--counters", action="append", default=[],
                    help="directory of a --pmc run with other counters (repeat): per kernel and grid size, the mean of every counter")
    ap.add_argument("--copy-bytes", type=float, help="bytes the calibration kernel reads (= bytes it writes)")
    ap.add_argument("--command", action="append", default=[], help="full command line of a run (repeat)")
    ap.add_argument("--key-suffix", default="", help="appended to the kernel names of the traffic_bytes_per_launch lines (e.g. @32images)")
    ap.add_argument("--title", default="rocprofv3 summary")
    ap.add_argument("--out", required=True)
    a = ap.parse_args()

    lines = [a.title, ""]
    for c in a.command:
        lines.append("command: " + c)
    lines.append("")
    if a.stats:
        rows = kernel_stats(a.stats)
        whole = sum(r[3] for r in rows)
        lines.append("kernel-trace statistics (durations in microseconds)")
        lines.append("%-34s %8s %10s %10s %10s %7s" % ("kernel", "calls", "avg_us", "min_us", "max_us", "share%"))
        shared = defaultdict(int)
        for r in rows:
            shared[r[0]] += 1
        for name, calls, avg, tot, mn, mx, full in sorted(rows, key=lambda r: -r[3]):
            if not any(o in full for o in OURS):
                continue
            if shared[name] > 1:   # several instantiations of one kernel template: tell them apart
                m = re.search(r"<([^>]*)>", full.replace("(anonymous namespace)::", ""))
                if m:
                    name += "<" + m.group(1).replace(" ", "") + ">"
            lines.append("%-34s %8d %10.2f %10.2f %10.2f %7.2f" % (name, calls, avg / 1e3, mn / 1e3, mx / 1e3, 100 * tot / whole))
        other = sum(r[3] for r in rows if not any(o in r[6] for o in OURS))
        lines.append("%-34s %8s %10s %10s %10s %7.2f" % ("(kernels of other libraries)", "", "", "", "", 100 * other / whole))
        lines.append("")
    if a.fetch or a.write:
        if not a.copy_bytes:
            sys.exit("profile_summary: --copy-bytes is required with --fetch / --write")
        fetch = counter_means(a.fetch, "FETCH_SIZE") if a.fetch else {}
        write = counter_means(a.write, "WRITE_SIZE") if a.write else {}

        def calibration(table, what):
            cand = {k: v for k, v in table.items() if k.startswith("elementwise[Mul")}
            if not cand:
                sys.exit(f"profile_summary: no calibration kernel in the {what} run")
            k = max(cand, key=lambda k: cand[k][0])
            return k, cand[k][0]

        lines.append("HBM traffic per launch (counter mean over launches, KiB, and bytes scaled by the calibration kernel)")
        scale_f = scale_w = None
        if fetch:
            k, v = calibration(fetch, "FETCH_SIZE")
            scale_f = a.copy_bytes / (v * 1024.0)
            lines.append("calibration FETCH_SIZE: %s reads %.0f bytes, counter %.1f KiB -> factor %.4f" % (k, a.copy_bytes, v, scale_f))
        if write:
            k, v = calibration(write, "WRITE_SIZE")
            scale_w = a.copy_bytes / (v * 1024.0)
            lines.append("calibration WRITE_SIZE: %s writes %.0f bytes, counter %.1f KiB -> factor %.4f" % (k, a.copy_bytes, v, scale_w))
        lines.append("%-34s %8s %14s %14s %14s" % ("kernel", "launches", "FETCH_KiB", "WRITE_KiB", "bytes"))
        names = [k for k in sorted(set(fetch) | set(write)) if not k.startswith("elementwise")]
        traffic = {}
        for k in names:
            fk, wk = fetch.get(k), write.get(k)
            b = (fk[0] * 1024 * scale_f if fk else 0.0) + (wk[0] * 1024 * scale_w if wk else 0.0)
            traffic[k] = b
            lines.append("%-34s %8d %14.1f %14.1f %14.0f" % (k, (fk or wk)[1], fk[0] if fk else float("nan"),
                                                             wk[0] if wk else float("nan"), b))
        lines.append("")
        for k, b in traffic.items():
            lines.append("traffic_bytes_per_launch[%s%s]: %.0f" % (k, a.key_suffix, b))
        lines.append("")
    if a.counters:
        table = defaultdict(lambda: defaultdict(lambda: [0.0, 0]))
        for directory in a.counters:
            for path in _find(directory, "counter_collection.csv"):
                with open(path, newline="") as f:
                    for r in csv.DictReader(f):
                        if not any(o in r["Kernel_Name"] for o in OURS):
                            continue
                        cell = table["%s grid=%s wg=%s" % (short_name(r["Kernel_Name"]), r["Grid_Size"], r["Workgroup_Size"])][r["Counter_Name"]]
                        cell[0] += float(r["Counter_Value"])
                        cell[1] += 1
        lines.append("hardware counters per launch (mean over launches; SQ_*_CYCLES and SQ_ACTIVE_* / SQ_WAIT_* count in units of 4 cycles)")
        for kernel in sorted(table):
            lines.append(kernel)
            for counter in sorted(table[kernel]):
                total, n = table[kernel][counter]
                lines.append("    %-28s %16.0f   (%d launches)" % (counter, total / n, n))
        lines.append("")
    os.makedirs(os.path.dirname(os.path.abspath(a.out)), exist_ok=True)
    with open(a.out, "w") as f:
        f.write("\n".join(lines))
    print("\n".join(lines))


if __name__ == "__main__":
    main()
