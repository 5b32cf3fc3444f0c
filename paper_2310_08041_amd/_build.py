"""Compile libqllm.so (HIP kernels for gfx950 + host helpers) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libqllm.so")
SOURCES = ["fused_nrq.hip", "fused_planned.hip", "int_gemm.hip", "match_pairs.hip", "probes.hip", "calib_ops.hip", "swiglu.hip", "host_offline.cpp"]

# -ffp-contract=off: the fused kernel's fp32 arithmetic is defined with one rounding per operation.
# packed-fp32 instructions are switched off for the device passes.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off", "-fPIC", "-pthread",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function",
         "-I", os.path.join(ROOT, "include")]


def build_lib(verbose: bool = False) -> str:
    objs = []
    procs = []
    for s in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(s)[0] + ".o")
        objs.append(obj)
        procs.append((s, subprocess.Popen(["hipcc", *FLAGS, "-c", os.path.join(CSRC, s), "-o", obj],
                                          stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for s, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {s}:\n{out}")
        if verbose and out.strip():
            print(out)
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread", *objs, "-o", LIB], check=True)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
