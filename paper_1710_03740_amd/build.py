"""Compile the HIP sources into paper_1710_03740_amd/libmpt.so for gfx950.

Run as `python -m paper_1710_03740_amd.build`.  hipcc cross-compiles without a
GPU.  The library is built in-tree so that it travels with the source tree.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libmpt.so")
OBJDIR = os.path.join(HERE, "_build")

HIP_SOURCES = ["elementwise.hip", "gemm.hip", "norm.hip", "optim.hip", "lstm.hip", "probe.hip"]
CXX_SOURCES = ["host.cpp"]

# -ffp-contract=off: the update path is specified as separately rounded FP32 operations.
# packed-fp32 VALU forms are disabled for the whole library.
HIP_FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-ffp-contract=off",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wno-unused-command-line-argument", "-I", INCLUDE, "-I", CSRC]


def _run(cmd):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)
    if p.returncode != 0:
        raise RuntimeError("build failed: %s\n%s" % (" ".join(cmd), out))
    if out.strip():
        print(out)


def build(verbose=True):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJDIR, exist_ok=True)
    objs = []
    procs = []
    for src in HIP_SOURCES + CXX_SOURCES:
        path = os.path.join(CSRC, src)
        if not os.path.exists(path):
            raise RuntimeError("missing source " + path)
        obj = os.path.join(OBJDIR, src + ".o")
        objs.append(obj)
        lang = ["-x", "hip"] if src.endswith(".hip") else []
        cmd = [hipcc] + HIP_FLAGS + lang + ["-c", path, "-o", obj]
        if verbose:
            print("[mpt build]", src, flush=True)
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("build failed: %s\n%s" % (" ".join(cmd), out))
        if out.strip() and verbose:
            print(out)
    _run([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs)
    if verbose:
        print("[mpt build] wrote", LIB, flush=True)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
