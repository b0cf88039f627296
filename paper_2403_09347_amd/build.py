"""Builds libburst.so (the C-ABI library) from csrc/ with hipcc for gfx950, in-tree."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libburst.so")
SOURCES = ["burst_api.hip", "burst_elementwise.hip", "burst_generic.hip",
           "burst_fwd_mfma.hip", "burst_bwd_dq_mfma.hip", "burst_bwd_dkv_mfma.hip",
           "burst_materialized.hip", "burst_d64_mfma.hip", "burst_d128_plain.hip", "burst_probe.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-ffast-math", "-fno-finite-math-only", "-fno-honor-nans",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-amdgpu-mfma-vgpr-form=1", "-Wno-unused-command-line-argument",
         "-Wno-inline-asm"]   # the DMA helper names M0 as clobbered, which the compiler reports as a reserved register


def build(verbose=True, jobs=8):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs, procs = [], []
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    for src in SOURCES:
        obj = os.path.join(HERE, "_build", src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if len(procs) >= jobs:
            _drain(procs, verbose)
    _drain(procs, verbose)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    build_example(verbose)
    return LIB


EXAMPLE_SRC = os.path.join(HERE, "examples", "ring_walk.cpp")
EXAMPLE_BIN = os.path.join(HERE, "_build", "ring_walk")


def build_example(verbose=True):
    """The plain host program that walks a ring share through the C ABI (no Python on its path),
    linked against the library just built; run by tests/test_gpu_c_example.py."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-O2", "-std=c++17", "--offload-arch=gfx950", "-I", os.path.join(os.path.dirname(HERE), "include"),
           EXAMPLE_SRC, "-L", HERE, "-lburst", "-Wl,-rpath,$ORIGIN/..", "-o", EXAMPLE_BIN]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return EXAMPLE_BIN


def _drain(procs, verbose):
    while procs:
        src, p = procs.pop(0)
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            sys.stderr.write(out + "\n")
            raise RuntimeError("hipcc failed on " + src)
        if verbose and out.strip():
            print(out)


if __name__ == "__main__":
    build()
