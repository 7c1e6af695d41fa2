"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

Usage (after the rocprofv3 runs named in each summary's header):
    python -m paper_2512_23049_amd.profile_summary stats  <dir>/<prefix>_kernel_stats.csv  <label>  "<command>"
    python -m paper_2512_23049_amd.profile_summary pmc    <fetch.csv> <write.csv> <label> "<command>" [kernel:grid=workload,...]
    python -m paper_2512_23049_amd.profile_summary counters <counter_collection.csv> <label> "<command>"
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


def pmc(fetch_csv, write_csv, label, command, names="", copy_mib=1024):
    """names: comma list kernel_prefix:grid=workload, naming the workload each (kernel, grid) row belongs to."""
    tag = {}
    for item in names.split(","):
        if item:
            kg, wl = item.split("=")
            tag[tuple(kg.split(":"))] = wl
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
           "kernel,grid,dispatches,fetch_MB_per_launch,write_MB_per_launch,workload"]
    for key in sorted(f):
        if not key[0].startswith(("pc_prefill", "pc_decode", "void pc_merge")):
            continue
        wl = next((v for (kp, g), v in tag.items() if key[0].startswith(kp) and g == key[1]), "")
        out.append(f"{key[0]},{key[1]},{fn[key]},{f[key] * f_scale * 1024 / 1e6:.2f},{w.get(key, 0) * w_scale * 1024 / 1e6:.2f},{wl}")
    dst = os.path.join(ROOT, "profiles", f"{label}_hbm_traffic.txt")
    open(dst, "w").write("\n".join(out) + "\n")
    print(dst)


def counters(path, label, command):
    """Average per dispatch of every collected counter, for the attention kernels."""
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(path)):
        agg[(r["Kernel_Name"].split("(")[0][:48], r["Grid_Size"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    out = [f"# rocprofv3 --pmc (SQ counters, average per dispatch), {label}", f"# command: {command}"]
    for key in sorted(agg):
        if not key[0].startswith(("pc_prefill", "pc_decode")):
            continue
        c = {k: sum(v) / len(v) for k, v in agg[key].items()}
        out.append(f"kernel {key[0]} grid {key[1]} dispatches {len(next(iter(agg[key].values())))}")
        for k in sorted(c):
            out.append(f"  {k} {c[k]:.4g}")
        if "SQ_VALU_MFMA_BUSY_CYCLES" in c and "SQ_BUSY_CYCLES" in c:
            # SQ_BUSY_CYCLES sums over the 32 shader engines, MFMA busy cycles over the 1024 SIMDs
            out.append(f"  derived: MFMA pipe busy {c['SQ_VALU_MFMA_BUSY_CYCLES'] / 1024 / (c['SQ_BUSY_CYCLES'] / 32):.3f} of kernel cycles")
        if "SQ_ACTIVE_INST_VALU" in c and "SQ_BUSY_CYCLES" in c:
            # counted in units of 4 cycles per wave; two waves share a SIMD
            out.append(f"  derived: VALU issue busy {c['SQ_ACTIVE_INST_VALU'] * 4 / 1024 / (c['SQ_BUSY_CYCLES'] / 32):.3f} of SIMD cycles")
        if "SQ_INSTS_VALU" in c and "SQ_INSTS_MFMA" in c:
            out.append(f"  derived: vector ALU instructions per MFMA {(c['SQ_INSTS_VALU'] - c['SQ_INSTS_MFMA']) / c['SQ_INSTS_MFMA']:.2f}")
    dst = os.path.join(ROOT, "profiles", f"{label}_sq_counters.txt")
    open(dst, "w").write("\n".join(out) + "\n")
    print(dst)


if __name__ == "__main__":
    if sys.argv[1] == "stats":
        stats(*sys.argv[2:5])
    elif sys.argv[1] == "counters":
        counters(*sys.argv[2:5])
    else:
        pmc(*sys.argv[2:7])
