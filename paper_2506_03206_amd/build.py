"""Compiles the HIP library for gfx950 with hipcc, in-tree:  paper_2506_03206_amd/librdk_hip.so,
and the stand-alone rate microbenchmark  paper_2506_03206_amd/ceilings."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librdk_hip.so")
CEILINGS = os.path.join(HERE, "ceilings")    # stand-alone microbenchmark of HBM and matrix-instruction rates
SOURCES = ["rdk_api.hip", "rdk_build.hip", "rdk_linear.hip", "rdk_sparse.hip", "rdk_exact.hip", "rdk_verify.hip", "rdk_multi.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc", "-Wall", "-Wno-unused-function",
         # packed fp32 instructions are kept off for every device function
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose=False):
    """Compile every translation unit and link the shared library (always rebuilds)."""
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = ["hipcc", *FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    # the microbenchmark is a program of its own; nothing in the library depends on it
    cmd = ["hipcc", *[f for f in FLAGS if f != "-fPIC"], os.path.join(CSRC, "ceilings.hip"), "-o", CEILINGS]
    if verbose:
        print(" ".join(cmd), flush=True)
    procs.append(("ceilings.hip", subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l or "error" in l)
        if p.returncode != 0:
            failed = True
            sys.stderr.write("hipcc failed on %s:\n%s\n" % (src, out))
        elif verbose and out.strip():
            print(out)
    if failed:
        raise RuntimeError("HIP compilation failed")
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
