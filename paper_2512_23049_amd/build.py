"""Builds libpc.so (the C-ABI library) and libpc_probe.so (the benchmark's achievable-peak probes) in-tree with
hipcc for gfx950."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpc.so")
PROBE_LIB = os.path.join(HERE, "libpc_probe.so")
PROBE_SOURCES = ["pc_probe.hip"]
SOURCES = ["pc_lib.hip", "pc_plan.hip", "pc_attend.hip", "pc_kernels_basic.hip", "pc_kernels_backward.hip", "pc_kernels_mfma.hip", "pc_kernels_prefill.hip",
           "pc_kernels_shared.hip"]
# the prefill kernel never produces NaNs in its max reductions: let the compiler drop the
# canonicalising v_max x, x in front of every fmax
FILE_FLAGS = {"pc_kernels_prefill.hip": ["-fno-honor-nans"]}
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-result"]


def build(verbose: bool = False, extra=()):
    """Compile every source and link the shared library; always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for s in SOURCES + PROBE_SOURCES:
        o = os.path.join(CSRC, s.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *FILE_FLAGS.get(s, []), *extra, "-c", os.path.join(CSRC, s), "-o", o]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(o)
    failed = None
    for cmd, p in procs:                                  # every compiler runs to its end before anything is reported
        out, _ = p.communicate()
        lines = [l for l in out.splitlines() if "packed-fp32-ops" not in l or "error" in l]
        if p.returncode != 0 and failed is None:
            failed = "hipcc failed: " + " ".join(cmd) + "\n" + out
        if verbose and lines:
            print("\n".join(lines))
    for f in os.listdir(CSRC):                            # what an interrupted or failed compile leaves behind
        if f.endswith(".o.tmp"):
            os.remove(os.path.join(CSRC, f))
    if failed:
        raise RuntimeError(failed)
    n = len(SOURCES)
    for out_lib, its in ((LIB, objs[:n]), (PROBE_LIB, objs[n:])):
        cmd = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", *its, "-o", out_lib]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stdout)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
