"""Builds libssd_magc.so (HIP, gfx950 only) in-tree, next to this file."""
import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
SOURCES = ["api.hip", "generic_kernels.hip", "mfma_kernels.hip", "dual_kernel.hip", "grad_bc_kernels.hip", "stack.hip", "prof.hip", "decode.hip", "conv1d.hip", "gated_norm.hip", "linear.hip", "few_rows.hip", "block.hip", "magc_plan.cpp"]
LIB = os.path.join(_HERE, "libssd_magc.so")
# Per-file compiler options.  The head-walking backward kernels are long straight-line bodies at the register limit:
# LLVM's iterative ILP scheduler interleaves their matrix-core and vector instructions better than the default one
# (measured: 114 -> 96 us per launch of the three passes; the small kernels of the other files get slower with it).
EXTRA_FLAGS = {"grad_bc_kernels.hip": ["-mllvm", "-amdgpu-sched-strategy=iterative-ilp"]}


def build(verbose: bool = False, jobs: int = 8) -> str:
    csrc = os.path.join(_HERE, "csrc")
    objdir = os.path.join(_HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    common = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
              "-I", os.path.join(_ROOT, "include"), "-I", csrc,
              # keep the compiler from forming packed-fp32 instructions
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    procs, objs = [], []
    for src in SOURCES:
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        objs.append(obj)
        cmd = common + EXTRA_FLAGS.get(src, []) + (["-x", "hip"] if src.endswith(".hip") else []) + ["-c", os.path.join(csrc, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if len(procs) >= jobs:
            _drain(procs, verbose)
    _drain(procs, verbose)
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.check_call(link)
    return LIB


def _drain(procs, verbose):
    while procs:
        src, p = procs.pop(0)
        out, _ = p.communicate()
        keep = [ln for ln in out.splitlines() if "packed-fp32-ops" not in ln or "error" in ln]
        if p.returncode != 0:
            sys.stderr.write(out)
            raise RuntimeError(f"hipcc failed on {src}")
        if verbose and keep:
            print("\n".join(keep), flush=True)


if __name__ == "__main__":
    build(verbose=True)
    print(LIB)
