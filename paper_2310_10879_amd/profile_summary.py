"""Condense rocprofv3 CSV output of `bench.py` runs into the short summaries kept under profiles/.

    python -m paper_2310_10879_amd.profile_summary --workload 2 \
        --trace  $OUT/kt/kt_kernel_stats.csv \
        --fetch  $OUT/fetch/fetch_counter_collection.csv \
        --write  $OUT/write/write_counter_collection.csv \
        --bench  $OUT/kt.json

OUT is any scratch directory.  The three rocprofv3 runs that produce those files (each a run of its own, from the
repository root on the MI355X; `--calibrate-copy` adds a plain 1 GiB elementwise copy
whose known size scales the two HBM counters):

    rocprofv3 --kernel-trace --stats --output-format csv -d $OUT/kt -o kt -- \
        python3 bench.py --workload W --steps 10 --warmup 2 --only --no-cpu-baseline --calibrate-copy
    rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d $OUT/fetch -o fetch -- \
        python3 bench.py --workload W --steps 3 --warmup 1 --only --no-cpu-baseline --calibrate-copy
    rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d $OUT/write -o write -- \
        python3 bench.py --workload W --steps 3 --warmup 1 --only --no-cpu-baseline --calibrate-copy

Writes profiles/bload_workloadW_kernel_trace.md, profiles/bload_workloadW_hbm_counters.md
and profiles/bload_workloadW_hbm_traffic.json (read back by bench.py for the `traffic` fields).
"""
from __future__ import annotations

import argparse
import collections
import csv
import hashlib
import json
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CAL_KIB = 1048576.0          # the calibration copy reads 1 GiB and writes 1 GiB


def short(name: str) -> str:
    if "MulFunctor" in name:
        return "torch mul (1 GiB calibration copy)"
    if "at::native" in name:
        return "torch " + name.split("<")[0].split("::")[-1]
    return name.split("(")[0].replace("void ", "")


def counter_means(path):
    acc = collections.defaultdict(list)
    with open(path) as f:
        for r in csv.DictReader(f):
            acc[(short(r["Kernel_Name"]), r["Counter_Name"])].append(float(r["Counter_Value"]))
    return {k: (sum(v) / len(v), len(v)) for k, v in acc.items()}


def yardstick_summary(args) -> None:
    """Kernel trace of the yardstick kernels beside the rates bench.py computed from its own event timing."""
    with open(args.bench) as f:
        ys = json.loads([ln for ln in f if ln.startswith("{")][-1])["yardsticks"]
    lines = ["# rocprofv3 kernel trace of bench.py's yardstick kernels", "",
             "Command (on the MI355X, from the repository root; OUT = a scratch directory):", "",
             "    rocprofv3 --kernel-trace --stats --output-format csv -d $OUT/kt -o kt -- \\",
             "        python3 bench.py --yardsticks-only", "",
             "Summarised by `python -m paper_2310_10879_amd.profile_summary --yardsticks` from kt_kernel_stats.csv.",
             "Each kernel runs twice untimed and five times timed (torch's: three and ten).", "",
             "| kernel | calls | avg ns | min ns | max ns |", "|---|---|---|---|---|"]
    with open(args.trace) as f:
        for r in csv.DictReader(f):
            name = r["Name"].replace("(anonymous namespace)::", "").split("(")[0].replace("void ", "")
            if "ys_" in name or "at::native" in name:
                lines.append(f"| {name[:110]} | {r['Calls']} | {float(r['AverageNs']):.0f} | {r['MinNs']} | {r['MaxNs']} |")
    lines += ["", "bench.py's figures in the same run (bytes the pattern moves / mean event time, GB/s):", ""]
    lines += [f"* torch copy {ys['copy_GBps']:.0f}, torch fill {ys['fill_GBps']:.0f}"]
    for key, val in ys["patterns"].items():
        if key != "what":
            lines.append(f"* {key[:-5] if key.endswith('_GBps') else key}: {val:.0f}" if isinstance(val, float) else f"* {key}: {val}")
    lines += ["", ys["patterns"].get("what", "")]
    with open(os.path.join(ROOT, "profiles", "bload_yardsticks_kernel_trace.md"), "w") as f:
        f.write("\n".join(lines) + "\n")
    print(lines[-3])


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", type=int, default=0)
    ap.add_argument("--trace", required=True)
    ap.add_argument("--fetch", help="omit both counter files to summarise the kernel trace only")
    ap.add_argument("--write")
    ap.add_argument("--flags", default="", help="further bench.py flags the runs were made with, "
                                                "e.g. '--plan random-fit --scan'")
    ap.add_argument("--tag", default="", help="suffix of the summary's file name for such a run")
    ap.add_argument("--bench", required=True, help="the JSON line bench.py printed in the trace run")
    ap.add_argument("--yardsticks", action="store_true",
                    help="the trace is of `bench.py --yardsticks-only`: write profiles/bload_yardsticks_kernel_trace.md")
    args = ap.parse_args()
    if args.yardsticks:
        yardstick_summary(args)
        return
    w = args.workload
    flags = (" " + args.flags.strip()) if args.flags.strip() else ""
    tag = ("_" + args.tag) if args.tag else ""
    with open(args.bench) as f:
        bench = json.loads([ln for ln in f if ln.startswith("{")][-1])
    cfg = bench["config"]["workload"]

    # ---- kernel trace
    lines = [f"# rocprofv3 kernel trace of bench.py, workload {cfg}", "",
             "Command (on the MI355X, from the repository root; OUT = a scratch directory):", "",
             "    rocprofv3 --kernel-trace --stats --output-format csv -d $OUT/kt -o kt -- \\",
             f"        python3 bench.py --workload {w} --steps 10 --warmup 2 --only --no-cpu-baseline --calibrate-copy{flags}",
             "", "Summarised by `python -m paper_2310_10879_amd.profile_summary` from kt_kernel_stats.csv.", "",
             "| kernel | calls | avg ns | min ns | max ns | % of GPU time |", "|---|---|---|---|---|---|"]
    with open(args.trace) as f:
        for r in csv.DictReader(f):
            lines.append(f"| {short(r['Name'])} | {r['Calls']} | {float(r['AverageNs']):.0f} | {r['MinNs']} | "
                         f"{r['MaxNs']} | {float(r['Percentage']):.2f} |")
    ph = bench["phases_ms"]
    lines += ["", "bench.py's event timing in the same run (ms per call): "
              + ", ".join(f"{name} {ms:.4f}" for name, ms in ph.items()) + "."]
    for name in ("pack", "segment_reduce", "segment_scan"):
        if name in bench:
            r = bench[name]
            lines += [f"{name}: {r['algorithmic_bytes_per_launch'] / 1e9:.4f} GB of algorithmic bytes per call / "
                      f"{r['launch_ms']:.4f} ms = {r['achieved']:.0f} GB/s = {100 * r['frac']:.1f} % of "
                      f"{r['peak']:.0f} GB/s."]
    with open(os.path.join(ROOT, "profiles", f"bload_workload{w}{tag}_kernel_trace.md"), "w") as f:
        f.write("\n".join(lines) + "\n")
    if not args.fetch or not args.write:
        print(lines[-1])
        return

    # ---- HBM counters
    fetch, write = counter_means(args.fetch), counter_means(args.write)
    cal = "torch mul (1 GiB calibration copy)"
    f_scale = CAL_KIB / fetch[(cal, "FETCH_SIZE")][0]
    w_scale = CAL_KIB / write[(cal, "WRITE_SIZE")][0]
    rows = ["| kernel | dispatches | FETCH_SIZE KiB (raw) | read GB (scaled) | WRITE_SIZE KiB (raw) | written GB (scaled) |",
            "|---|---|---|---|---|---|"]
    # kernel families of one library call each: (bench key, kernel name prefix, prefixes of the kernel that
    # runs exactly once per call, source file)
    families = {"pack": ("pack", "bload::pack_", ("bload::pack_prepare",), "bload_pack.hip"),
                "reduce": ("segment_reduce", "bload::reduce_", ("bload::reduce_wide", "bload::reduce_narrow"),
                           "bload_reduce.hip"),
                "scan": ("segment_scan", "bload::scan_", ("bload::scan_apply",), "bload_scan.hip")}
    totals = {k: [0.0, 0.0, 0] for k in families}          # read bytes, written bytes, calls
    names = sorted({k[0] for k in fetch} | {k[0] for k in write})
    for name in names:
        if not (name.startswith("bload::") or name == cal):
            continue
        fr, n_f = fetch.get((name, "FETCH_SIZE"), (0.0, 0))
        wr, n_w = write.get((name, "WRITE_SIZE"), (0.0, 0))
        rd_b, wr_b = fr * f_scale * 1024, wr * w_scale * 1024
        for fam, (_, prefix, mains, _) in families.items():
            if name.startswith(prefix):
                totals[fam][0] += rd_b * n_f
                totals[fam][1] += wr_b * n_w
                if name.startswith(mains):
                    totals[fam][2] += n_f
        if rd_b + wr_b < 1e6:
            continue
        rows.append(f"| {name} | {n_f} | {fr:.1f} | {rd_b / 1e9:.4f} | {wr:.1f} | {wr_b / 1e9:.4f} |")
    out = [f"# rocprofv3 HBM counters of bench.py, workload {cfg}", "",
           "Two counter passes, each a run of its own (on the MI355X, from the repository root; OUT = a scratch directory):", "",
           "    rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d $OUT/fetch -o fetch -- \\",
           f"        python3 bench.py --workload {w} --only --steps 3 --warmup 1 --no-cpu-baseline --calibrate-copy",
           "    rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d $OUT/write -o write -- \\",
           f"        python3 bench.py --workload {w} --only --steps 3 --warmup 1 --no-cpu-baseline --calibrate-copy",
           "", "Mean per dispatch.  Scale factors from the calibration copy (known: 1048576 KiB read, 1048576 KiB",
           f"written): FETCH_SIZE x {f_scale:.5f}, WRITE_SIZE x {w_scale:.5f}.", ""] + rows + [""]
    record = {"workload": w, "fetch_scale": f_scale, "write_scale": w_scale, "families": {}}
    for fam, (key, _, _, source) in families.items():
        rd, wr, calls = totals[fam]
        if calls == 0 or key not in bench:
            continue
        rd, wr = rd / calls, wr / calls
        alg = bench[key]["algorithmic_bytes_per_launch"]
        out += [f"{key} (all its kernels, per call): {rd / 1e9:.4f} GB read + {wr / 1e9:.4f} GB written = "
                f"{(rd + wr) / 1e9:.4f} GB of HBM traffic against {alg / 1e9:.4f} GB of algorithmic bytes "
                f"({100 * ((rd + wr) / alg - 1):+.2f} %)."]
        with open(os.path.join(ROOT, "paper_2310_10879_amd", "csrc", source), "rb") as f:
            digest = hashlib.sha256(f.read()).hexdigest()
        record["families"][fam] = {"hbm_bytes_per_call": rd + wr, "read_bytes_per_call": rd,
                                   "written_bytes_per_call": wr, "algorithmic_bytes_per_call": alg,
                                   "source": source, "source_sha256": digest}
    with open(os.path.join(ROOT, "profiles", f"bload_workload{w}_hbm_traffic.json"), "w") as f:
        json.dump(record, f, indent=1)
        f.write("\n")
    with open(os.path.join(ROOT, "profiles", f"bload_workload{w}_hbm_counters.md"), "w") as f:
        f.write("\n".join(out) + "\n")
    print("\n".join(lines[-3:] + out[-3:]))


if __name__ == "__main__":
    main()
