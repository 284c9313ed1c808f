"""Build libdfp4.so (HIP kernels + C ABI) and the mfma_peak measurement helper in-tree with hipcc for gfx950.

    python -m paper_2501_01144_amd.build

hipcc cross-compiles without a GPU.  The shared library is written next to
this file; the ctypes binding loads it from there.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdfp4.so")
PEAK = os.path.join(HERE, "mfma_peak")
SOURCES = ["api.hip", "quantize.hip", "dequantize.hip", "gemm.hip", "gemm_native.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-fconstexpr-steps=200000000",
    # keep hipcc from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
]


def build_library(verbose=True):
    # the hand-scheduled GEMM step is generated text (see csrc/gen_gemm_step.py)
    subprocess.run([sys.executable, os.path.join(CSRC, "gen_gemm_step.py")], check=True,
                   stdout=subprocess.DEVNULL)
    subprocess.run([sys.executable, os.path.join(CSRC, "gen_native_loop.py")], check=True,
                   stdout=subprocess.DEVNULL)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if out.strip() and verbose:
            print(out)
        if p.returncode != 0:
            failed = True
            print(f"hipcc failed on {src}", file=sys.stderr)
    if failed:
        raise RuntimeError("libdfp4 build failed")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    # measurement helper used by bench.py: register-only int8 MFMA loop
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", os.path.join(CSRC, "mfma_peak.hip"), "-o", PEAK]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build_library()
