"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

Usage (after the rocprofv3 runs named in each summary's header):
    python -m paper_2512_23049_amd.profile_summary stats  <dir>/<prefix>_kernel_stats.csv  <label>  "<command>"
    python -m paper_2512_23049_amd.profile_summary pmc    <fetch.csv> <write.csv> <label> "<command>"
The pmc form scales FETCH_SIZE / WRITE_SIZE (KiB per dispatch) by what the same counters read
for a plain device copy of known size launched by `bench.py --copy-probe-mib N`.
"""
import collections
import csv
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def stats(path, label, command):
    rows = list(csv.DictReader(open(path)))
    out = [f"# rocprofv3 --kernel-trace --stats, {label}", f"# command: {command}",
           "name,calls,avg_ns,min_ns,max_ns,percent"]
    for r in rows:
        out.append(f"{r['Name'][:64]},{r['Calls']},{float(r['AverageNs']):.0f},{r['MinNs']},{r['MaxNs']},{r['Percentage']}")
    dst = os.path.join(ROOT, "profiles", f"{label}_kernel_stats.txt")
    open(dst, "w").write("\n".join(out) + "\n")
    print(dst)


def _per_kernel(path):
    agg = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        agg[(r["Kernel_Name"].split("(")[0][:48], r["Grid_Size"])].append(float(r["Counter_Value"]))
    return {k: sum(v) / len(v) for k, v in agg.items()}, {k: len(v) for k, v in agg.items()}


def pmc(fetch_csv, write_csv, label, command, copy_mib=1024):
    f, fn = _per_kernel(fetch_csv)
    w, wn = _per_kernel(write_csv)
    copy = [k for k in f if "copyBuffer" in k[0] and f[k] > 1e5]
    assert copy, "no copy probe found: run bench.py with --copy-probe-mib"
    k = max(copy, key=lambda x: f[x])
    f_scale = copy_mib * 1024.0 / f[k]
    w_scale = copy_mib * 1024.0 / w[k]
    out = [f"# rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE (KiB per dispatch), {label}",
           f"# command (run once per counter): {command}",
           f"# scale: a plain device copy of {copy_mib} MiB read {f[k]:.0f} KiB and wrote {w[k]:.0f} KiB by these counters",
           f"#        -> fetch x{f_scale:.3f}, write x{w_scale:.3f}",
           "kernel,grid,dispatches,fetch_MB_per_launch,write_MB_per_launch"]
    for key in sorted(f):
        if not key[0].startswith(("pc_prefill", "pc_decode", "void pc_merge")):
            continue
        out.append(f"{key[0]},{key[1]},{fn[key]},{f[key] * f_scale * 1024 / 1e6:.2f},{w.get(key, 0) * w_scale * 1024 / 1e6:.2f}")
    dst = os.path.join(ROOT, "profiles", f"{label}_hbm_traffic.txt")
    open(dst, "w").write("\n".join(out) + "\n")
    print(dst)


if __name__ == "__main__":
    if sys.argv[1] == "stats":
        stats(*sys.argv[2:5])
    else:
        pmc(*sys.argv[2:6])
