"""Builds libosc.so (the product) and libosc_probe.so (the benchmark's matrix-core yardstick) in-tree
with hipcc, for gfx950 only."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libosc.so")
PROBE_LIB = os.path.join(HERE, "libosc_probe.so")
SOURCES = ["api.hip", "tuning.hip", "quant.hip", "gemm.hip", "profile.hip", "fused.hip", "g16.hip"]
PROBE_SOURCES = ["probe.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for s in SOURCES + PROBE_SOURCES:
        o = os.path.join(CSRC, s.replace(".hip", ".o"))
        objs.append(o)
        cmd = [hipcc, *FLAGS, "-c", os.path.join(CSRC, s), "-o", o]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((s, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
    for s, p in procs:
        out = p.communicate()[0].decode()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {s}:\n{out}")
        if verbose and out.strip():
            print(out)
    n = len(SOURCES)
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs[:n], "-o", LIB])
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs[n:], "-o", PROBE_LIB])
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
