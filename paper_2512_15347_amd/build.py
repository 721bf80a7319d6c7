"""Builds the HIP library in-tree: paper_2512_15347_amd/libprogrpo.so (gfx950 only)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libprogrpo.so")
SOURCES = ["api.hip", "sampler_kernels.hip", "ovf_kernels.hip", "gemm.hip", "attention.hip", "dit_kernels.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-ffp-contract=off", "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes"]


def build(verbose=True, jobs=4):
    """Compiles every source to an object (in parallel) and links the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if out.strip() and verbose:
            print(out, flush=True)
        if p.returncode != 0:
            failed = True
            print(f"compile failed: {src}\n{out}", file=sys.stderr)
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.check_call(cmd)
    if verbose:
        print("built", LIB, flush=True)
    return LIB


def ensure_built():
    """Build only if no library is there (tests, the smoke run and the benchmark load what is built)."""
    if not os.path.exists(os.environ.get("PROGRPO_LIB", LIB)):
        build(verbose=False)


if __name__ == "__main__":
    build()
