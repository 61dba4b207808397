"""Short text summaries of rocprofv3 runs of bench.py, as kept under profiles/.

    python -m paper_2508_12851_amd.profile_summary kernel-stats <rocprofv3 -d dir> <workload> [--args "..."]
    python -m paper_2508_12851_amd.profile_summary traffic <dir with fetch/ write/ cal_fetch/ cal_write/> <workload>
    python -m paper_2508_12851_amd.profile_summary counters <rocprofv3 -d dir> <name> --title "..." --command "..."

Every summary starts with the commit it was measured at and a hash of the kernel sources;
bench.py reports a committed traffic figure only while that hash still matches the sources it
runs (kernel_source_hash below), so a figure cannot outlive the kernel it was measured on.
The raw rocprofv3 output stays where the run wrote it; only these few lines are committed.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import hashlib
import os
import re
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
PROFILES = os.path.join(ROOT, "profiles")
KIB_1GIB = 1048576           # the calibration copy moves 1 GiB each way


def kernel_source_hash() -> str:
    """sha256 over the HIP sources and headers the library is built from (names and contents)."""
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(PKG, "csrc", "*")) + glob.glob(os.path.join(ROOT, "include", "*.h")))
    for path in files:
        if path.endswith((".hip", ".h")):
            h.update(os.path.basename(path).encode())
            h.update(open(path, "rb").read())
    return h.hexdigest()


def provenance() -> list:
    try:
        commit = subprocess.run(["git", "-C", ROOT, "rev-parse", "HEAD"], capture_output=True, text=True,
                                check=True).stdout.strip()
        dirty = subprocess.run(["git", "-C", ROOT, "status", "--porcelain", "--", "paper_2508_12851_amd/csrc",
                                "include", "bench.py"], capture_output=True, text=True).stdout.strip()
        if dirty:
            commit += " + uncommitted changes to the sources (see kernel_source_sha256)"
    except Exception:
        commit = "unknown (no git checkout)"
    return [f"commit = {commit}", f"kernel_source_sha256 = {kernel_source_hash()}"]


def _one(pattern):
    found = glob.glob(pattern, recursive=True)
    if len(found) != 1:
        raise SystemExit(f"expected one file matching {pattern}, found {found}")
    return found[0]


def _write(name, lines):
    os.makedirs(PROFILES, exist_ok=True)
    path = os.path.join(PROFILES, name)
    open(path, "w").write("\n".join(lines) + "\n")
    print("\n".join(lines))
    print("->", os.path.relpath(path, ROOT))


def kernel_stats(run_dir, workload, bench_args):
    rows = list(csv.DictReader(open(_one(os.path.join(run_dir, "**", "*kernel_stats.csv")))))
    cmd = ("cd /tmp && export TMPDIR=/tmp && rocprofv3 --kernel-trace --stats -d <out> --output-format csv -- "
           f"python3 /root/repo/bench.py {bench_args}").rstrip()
    out = [f"rocprofv3 kernel statistics, workload {workload}, one MI355X", *provenance(),
           f"command: {cmd}",
           "(every layer kernel is launched warm-up + timed steps times, plus the per-step timing calls)", "",
           f"{'kernel':<100} {'calls':>6} {'avg_us':>10} {'min_us':>10} {'max_us':>10} {'pct':>7}"]
    for r in rows:
        if float(r["Percentage"]) < 0.05:
            continue
        out.append(f"{r['Name'][:100]:<100} {r['Calls']:>6} {float(r['AverageNs']) / 1e3:>10.1f} "
                   f"{float(r['MinNs']) / 1e3:>10.1f} {float(r['MaxNs']) / 1e3:>10.1f} {float(r['Percentage']):>7.2f}")
    _write(f"{workload}_kernel_stats.txt", out)


def _counter(run_dir, name, match):
    vals = []
    for path in glob.glob(os.path.join(run_dir, "**", "*counter_collection.csv"), recursive=True):
        for r in csv.DictReader(open(path)):
            if r["Counter_Name"] == name and match(r["Kernel_Name"]):
                vals.append(float(r["Counter_Value"]))
    return vals


def _is_gated(k):
    m = re.search(r"grouped_gemm_kernel<([^>]*)>", k)
    return bool(m) and m.group(1).split(",")[6].strip() == "true"


def _is_plain(k):
    """The down projection's main launch (not the launch for the slices of a cut last round)."""
    m = re.search(r"grouped_gemm_kernel<([^>]*)>", k)
    if not m:
        return False
    a = [t.strip() for t in m.group(1).split(",")]
    return a[6] == "false" and (len(a) < 11 or a[10] == "false")


def traffic(base, workload, bench_args):
    avg = lambda v: sum(v) / len(v)
    fd = _counter(os.path.join(base, "fetch"), "FETCH_SIZE", _is_gated)
    wd = _counter(os.path.join(base, "write"), "WRITE_SIZE", _is_gated)
    f2 = _counter(os.path.join(base, "fetch"), "FETCH_SIZE", _is_plain)
    w2 = _counter(os.path.join(base, "write"), "WRITE_SIZE", _is_plain)
    is_copy = lambda k: "elementwise" in k or "copy" in k.lower()
    cf = max(_counter(os.path.join(base, "cal_fetch"), "FETCH_SIZE", is_copy))
    cw = max(_counter(os.path.join(base, "cal_write"), "WRITE_SIZE", is_copy))
    sf, sw = KIB_1GIB / cf, KIB_1GIB / cw
    rd, wr = avg(fd) * sf * 1024, avg(wd) * sw * 1024
    pre = "cd /tmp && export TMPDIR=/tmp && rocprofv3 --pmc"
    post = f"-d <out> --output-format csv -- python3 /root/repo/bench.py {bench_args}".rstrip()
    out = [f"HBM-side traffic of the dominant kernel (gate/up grouped GEMM), workload {workload}, one MI355X",
           *provenance(),
           "two rocprofv3 --pmc passes, counters in KiB per dispatch, averaged over the dispatches of that kernel:",
           f"  {pre} FETCH_SIZE {post}", f"  {pre} WRITE_SIZE {post}",
           "calibration on a plain 1 GiB device copy (reads 1 GiB, writes 1 GiB):",
           "  cd /root/repo && rocprofv3 --pmc FETCH_SIZE -d <out> --output-format csv -- python3 -m paper_2508_12851_amd.copy_calibration",
           "  cd /root/repo && rocprofv3 --pmc WRITE_SIZE -d <out> --output-format csv -- python3 -m paper_2508_12851_amd.copy_calibration",
           f"  copy kernel FETCH_SIZE = {cf:.0f} for {KIB_1GIB} KiB read  -> scale {sf:.4f}",
           f"  copy kernel WRITE_SIZE = {cw:.0f} for {KIB_1GIB} KiB written -> scale {sw:.4f}", "",
           f"FETCH_SIZE raw avg = {avg(fd):.0f} ({len(fd)} dispatches) -> {rd / 1e9:.3f} GB read per launch",
           f"WRITE_SIZE raw avg = {avg(wd):.0f} ({len(wd)} dispatches) -> {wr / 1e9:.3f} GB written per launch",
           f"traffic_bytes_per_launch = {rd + wr:.0f}", "",
           f"down-projection kernel, same passes: FETCH_SIZE raw {avg(f2):.0f} -> {avg(f2) * sf * 1024 / 1e9:.3f} GB, "
           f"WRITE_SIZE raw {avg(w2):.0f} -> {avg(w2) * sw * 1024 / 1e9:.3f} GB"]
    _write(f"hbm_traffic_{workload}.txt", out)


def counters(run_dir, name, title, command):
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for path in glob.glob(os.path.join(run_dir, "**", "*counter_collection.csv"), recursive=True):
        for r in csv.DictReader(open(path)):
            k = r["Kernel_Name"]
            m = re.search(r"<(.*?)>", k)
            short = k.split("<")[0].split("::")[-1][:32] + (" <" + m.group(1)[:44] + ">" if m else "")
            agg[short][r["Counter_Name"]].append(float(r["Counter_Value"]))
            if "Start_Timestamp" in r:
                agg[short]["duration_us"].append((float(r["End_Timestamp"]) - float(r["Start_Timestamp"])) / 1e3)
    out = [title, *provenance(), f"command: {command}", "(averages per dispatch)", ""]
    for short, c in sorted(agg.items()):
        n = max(len(v) for v in c.values())
        out.append(f"{short:<80} n={n:<5} " + "  ".join(f"{k}={sum(v) / len(v):.5g}" for k, v in sorted(c.items())))
    _write(f"{name}.txt", out)


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="what", required=True)
    a = sub.add_parser("kernel-stats")
    a.add_argument("run_dir"); a.add_argument("workload"); a.add_argument("--args", default="")
    b = sub.add_parser("traffic")
    b.add_argument("base"); b.add_argument("workload"); b.add_argument("--args", default="")
    c = sub.add_parser("counters")
    c.add_argument("run_dir"); c.add_argument("name"); c.add_argument("--title", required=True)
    c.add_argument("--command", required=True)
    args = ap.parse_args()
    if args.what == "kernel-stats":
        kernel_stats(args.run_dir, args.workload, args.args)
    elif args.what == "traffic":
        traffic(args.base, args.workload, args.args)
    else:
        counters(args.run_dir, args.name, args.title, args.command)


if __name__ == "__main__":
    main()
