"""Build libdfp4.so (HIP kernels + C ABI) in-tree with hipcc for gfx950, and the two
measurement helpers of bench.py (bench_helpers/ at the repository root).

    python -m paper_2501_01144_amd.build

hipcc cross-compiles without a GPU.  The shared library is written next to
this file; the ctypes binding loads it from there.
"""
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdfp4.so")
HELPERS = os.path.join(ROOT, "bench_helpers")
SOURCES = ["api.hip", "quantize.hip", "dequantize.hip", "gemm.hip", "gemm_native.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-fconstexpr-steps=200000000",
    # keep hipcc from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
]

_AGPR = re.compile(r"\ba(\d+|\[\d+:\d+\])(?![\w.])")


def check_accumulators_untouched(asm_text):
    """Guard for gemm_fast_kernel.  Its main loop is one inline-assembly statement that leaves
    the 256 int32 accumulators in a0..a255; the epilogue reads them back with further
    inline-assembly statements.  The compiler is told the loop clobbers those registers, so
    nothing in the language stops it from using an accumulation register for its own purposes
    (a spill, a copy) between the two.  This check makes that a build error instead of a silent
    wrong result: in every gemm_fast_kernel, no compiler-generated instruction that can execute
    after the main loop (followed through the kernel's branches) may name an accumulation
    register, and the kernel must not use scratch memory."""
    problems = []
    lines = asm_text.splitlines()
    i, n = 0, len(lines)
    while i < n:
        m = re.match(r"^(_ZN\S*gemm_fast_kernel\S*):", lines[i])
        if not m:
            i += 1
            continue
        name = m.group(1)
        j = i + 1
        while j < n and ".end_amdhsa_kernel" not in lines[j]:
            j += 1
        body = lines[i + 1:j]
        labels = {}
        in_asm, asm_region, first_end = False, [], None
        for k, ln in enumerate(body):
            if ";;#ASMSTART" in ln:
                in_asm = True
            elif ";;#ASMEND" in ln:
                in_asm = False
                if first_end is None:
                    first_end = k
            asm_region.append(in_asm)
            lm = re.match(r"^(\.LBB\w+):", ln)
            if lm and not in_asm:
                labels[lm.group(1)] = k
        if first_end is None:
            problems.append(f"{name}: main loop not found")
        else:
            seen, work = set(), [first_end + 1]
            while work:
                k = work.pop()
                while k < len(body) and k not in seen:
                    seen.add(k)
                    code = body[k].split(";")[0].strip()
                    if not asm_region[k] and code and not code.startswith("."):
                        if _AGPR.search(code):
                            problems.append(f"{name}: compiler-generated code touches an accumulation register "
                                            f"after the main loop: {code}")
                        op = code.split()[0]
                        tm = re.search(r"(\.LBB\w+)", code)
                        if op.startswith("s_cbranch") or op == "s_branch":
                            if tm and tm.group(1) in labels:
                                work.append(labels[tm.group(1)])
                            if op == "s_branch":
                                break
                        elif op in ("s_endpgm", "s_setpc_b64"):
                            break
                    k += 1
        # resource summary that follows the kernel descriptor
        k = j
        while k < n and k < j + 60:
            if "; ScratchSize:" in lines[k]:
                if lines[k].split(":")[1].strip() != "0":
                    problems.append(f"{name}: uses scratch memory ({lines[k].strip()})")
                break
            k += 1
        i = j
    return problems


def build_library(verbose=True):
    # the hand-scheduled GEMM loops are generated text (see csrc/gen_gemm_step.py, csrc/gen_native_loop.py)
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
    # device assembly of the GEMM, for the accumulator guard
    gemm_s = os.path.join(objdir, "gemm.s")
    cmd = [hipcc, *FLAGS, "-S", "--cuda-device-only", os.path.join(CSRC, "gemm.hip"), "-o", gemm_s]
    procs.append(("gemm.hip (assembly)", subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    # measurement helpers used by bench.py: register-only int8 MFMA loops, plain streaming kernels
    for name in ("mfma_peak", "stream_peak", "mfma_shadow"):
        cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Wno-inline-asm", os.path.join(HELPERS, name + ".hip"),
               "-o", os.path.join(HELPERS, name)]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((name, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
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
    problems = check_accumulators_untouched(open(gemm_s).read())
    if problems:
        raise RuntimeError("gemm_fast_kernel accumulator guard:\n" + "\n".join(problems))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build_library()
