#!/usr/bin/env python3
"""Benchmark of the DialectFP4 hot path on one MI355X.

A step is one pass of the whole path over the LLaMA-3-8B MLP prefill batch
(M = 2048 tokens): quantize x online -> gate GEMM, up GEMM (K = 4096,
N = 14336) -> quantize h online -> down GEMM (K = 14336, N = 4096).  Weights
are quantized once, before the timed region (the paper pre-quantizes weights).
All inputs are seeded synthetic tensors already resident in HBM.

Prints ONE JSON line.  `value` is the step's integer-op throughput
(2*M*N*K summed over the three GEMMs, divided by the whole step time including
both quantizer launches).  `roofline` is the GEMM kernel against the int8 MFMA
peak, `roofline_quantizer` the quantizer against HBM on the streaming tensors,
`cpu_baseline` the NumPy oracle on a sample of the same workload.
"""
import argparse
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
INT8_PEAK_TOPS = 5000.0
FP6_PEAK_TOPS = 10100.0


def _events(n, torch):
    return [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]


def measured_traffic(key):
    """Per-launch HBM-side bytes measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    (scaled by a plain copy of known size); the summary is kept under profiles/."""
    path = os.path.join(ROOT, "profiles", "bench_mlp_prefill_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith(key + " = "):
                return float(line.split("=")[1]) * 1e6
    except OSError:
        pass
    return None


def quant_bytes(rows, K, mx=False):
    """Algorithmic bytes of one quantizer launch: 2 B/element in, 0.5 B codes +
    one exponent byte (+ one dialect byte) per 32 out."""
    return rows * K * (2.0 + 0.5 + (1.0 if mx else 2.0) / 32.0)


def gemm_bytes(M, N, K, out_bytes=4):
    """Algorithmic bytes of one GEMM launch: both quantized operands once
    (4-bit codes + exponent and dialect bytes per 32) and the output once."""
    return (M + N) * K * (0.5 + 2.0 / 32.0) + M * N * out_bytes


def cpu_baseline(ops, target_seconds=25.0):
    """The oracle as it stands, timed on the host on a sample of the step: the first
    `tokens` rows of x and h against the first `cols` rows of each weight matrix.
    A short calibration run picks the sample so that the timed part takes roughly
    `target_seconds` on this machine."""
    import numpy as np
    from oracle import dfp4_oracle as O
    from paper_2501_01144_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = 1
    def prepare(tokens, cols):
        x, h = synth.to_f64(ops["x"][:tokens]), synth.to_f64(ops["h"][:tokens])
        wq = {k: O.dfp4_quantize(synth.to_f64(ops[k][:cols])) for k in ("w_gate", "w_up", "w_down")}
        return x, h, wq

    def run(x, h, wq):
        t0 = time.perf_counter()
        qx = O.dfp4_quantize(x)
        O.dfp4_gemm(qx, wq["w_gate"])
        O.dfp4_gemm(qx, wq["w_up"])
        qh = O.dfp4_quantize(h)
        O.dfp4_gemm(qh, wq["w_down"])
        return time.perf_counter() - t0

    run(*prepare(32, 32))                         # first-call costs stay out of the calibration
    tokens, cols = 128, 512
    dt = run(*prepare(tokens, cols))
    grow = max(1.0, target_seconds / dt)
    new_tokens = int(min(ops["x"].shape[0], tokens * grow))
    grow /= new_tokens / tokens
    tokens, cols = new_tokens, int(min(4096, cols * max(1.0, grow)))
    x, h, wq = prepare(tokens, cols)
    dt, reps = run(x, h, wq), 1
    while dt < 0.5 * target_seconds and reps < 8:     # fast hosts: repeat the (largest) sample
        dt += run(x, h, wq)
        reps += 1
    int_ops = 2.0 * reps * tokens * cols * (2 * x.shape[1] + h.shape[1])
    return {"value": int_ops / dt / 1e12, "unit": "TOP/s", "cores": int(cores), "kind": "oracle",
            "seconds": round(dt, 3),
            "sample": f"{reps} x ({tokens} tokens x {cols} output columns of each of the three GEMMs) "
                      f"(weights pre-quantized untimed, activations quantized inside the timed region), "
                      f"NumPy float64 oracle"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--out-dtype", choices=["f32", "bf16"], default="f32", help="GEMM output type")
    ap.add_argument("--no-mfma-peak", action="store_true", help="skip the register-only MFMA loop")
    ap.add_argument("--gemm", choices=["int8", "native"], default="int8",
                    help="which GEMM path the headline fields describe: the int8 matrix-core path "
                         "(dfp4_gemm) or the block-scaled FP6 one (dfp4_gemm_native_packed); both are "
                         "always measured and reported")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stream-quant", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (a known-size kernel to scale "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    # register-only int8 MFMA loop in a child process, before this process touches the GPU
    peak = None
    if not args.no_mfma_peak:
        exe = os.path.join(ROOT, "bench_helpers", "mfma_peak")
        if not os.path.exists(exe):
            print(f"bench.py: {exe} not found (build it with `python -m paper_2501_01144_amd.build`); "
                  "the register-only MFMA loop is left out of the report", file=sys.stderr)
        else:
            r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
            if r.returncode == 0 and r.stdout.strip():
                peak = json.loads(r.stdout.strip().splitlines()[-1])
            else:
                print("bench.py: mfma_peak failed: " + r.stderr, file=sys.stderr)

    import torch
    from paper_2501_01144_amd import dfp4, synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    dfp4.load()
    dev = torch.device("cuda:0")

    ops = synth.llama3_8b_mlp(seed=2)
    M, H = ops["x"].shape
    I = ops["h"].shape[1]
    x, h = ops["x"].to(dev), ops["h"].to(dev)
    wq = {k: dfp4.quantize(ops[k].to(dev)) for k in ("w_gate", "w_up", "w_down")}
    qx, qh = dfp4.empty_qtensor(M, H, dev), dfp4.empty_qtensor(M, I, dev)
    odt = torch.float32 if args.out_dtype == "f32" else torch.bfloat16
    gate = torch.empty((M, I), dtype=odt, device=dev)
    up = torch.empty((M, I), dtype=odt, device=dev)
    down = torch.empty((M, H), dtype=odt, device=dev)
    ws_bytes = max(dfp4.gemm_workspace_bytes(M, I, H), dfp4.gemm_workspace_bytes(M, H, I))
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    names = ["quantize_x", "gemm_gate", "gemm_up", "quantize_h", "gemm_down"]

    def step(ev=None):
        calls = [
            lambda: dfp4.quantize(x, out=qx),
            lambda: dfp4.gemm(qx, wq["w_gate"], out=gate, workspace=ws),
            lambda: dfp4.gemm(qx, wq["w_up"], out=up, workspace=ws),
            lambda: dfp4.quantize(h, out=qh),
            lambda: dfp4.gemm(qh, wq["w_down"], out=down, workspace=ws),
        ]
        for i, c in enumerate(calls):
            if ev is not None:
                ev[i][0].record()
            c()
            if ev is not None:
                ev[i][1].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # HIP events around every call of every EVERY-th step of the timed region (events between all kernels of
    # all steps would add their own gaps to the step time)
    EVERY = 8
    evs = [_events(len(names), torch) if s % EVERY == 0 else None for s in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(evs[s])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    evs = [e for e in evs if e is not None]
    kern_ms = {n: sum(e[i][0].elapsed_time(e[i][1]) for e in evs) / len(evs) for i, n in enumerate(names)}
    gemm_ops = {"gemm_gate": 2.0 * M * I * H, "gemm_up": 2.0 * M * I * H, "gemm_down": 2.0 * M * H * I}
    total_ops = sum(gemm_ops.values())
    gemm_ms = sum(kern_ms[n] for n in gemm_ops)
    gemm_tops = total_ops / (gemm_ms * 1e-3) / 1e12
    value = total_ops / (ms_per_step * 1e-3) / 1e12
    q_bytes = quant_bytes(M, H) + quant_bytes(M, I)
    q_ms = kern_ms["quantize_x"] + kern_ms["quantize_h"]

    out = {
        "metric": "DialectFP4 quant GB/s + quantized GEMM TOPS (% int8 MFMA peak), LLaMA-3-8B shapes",
        "value": round(value, 3), "unit": "TOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "LLaMA-3-8B MLP prefill, M=2048: quantize x[2048x4096] -> gate/up GEMM "
                               "(K=4096,N=14336) -> quantize h[2048x14336] -> down GEMM (K=14336,N=4096); "
                               "activations N(0,1) + 0.5% outlier channels x50, weights N(0,0.02), "
                               "weights pre-quantized", "M": M, "hidden": H, "intermediate": I,
                   "out_dtype": args.out_dtype},
        "kernel_ms": {k: round(v, 4) for k, v in kern_ms.items()},
        "pct_int8_peak_step": round(100.0 * value / INT8_PEAK_TOPS, 2),
        "quantize_in_step_GBps": round(q_bytes / (q_ms * 1e-3) / 1e9, 1),
        "roofline": {"bound": "mfma",
                     "kernel": "dfp4_gemm call = gemm_prep_kernel + gemm_fast_kernel + gemm_block_kernel "
                               "(3 calls per step, HIP events around each call on the launch stream)",
                     "achieved": round(gemm_tops, 3), "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                     "frac": round(gemm_tops / INT8_PEAK_TOPS, 4),
                     "traffic": measured_traffic("gemm_fast_kernel_avg_MB_per_launch"),
                     "algorithmic_bytes_per_launch": round(
                         (2 * gemm_bytes(M, I, H, 4 if args.out_dtype == "f32" else 2)
                          + gemm_bytes(M, H, I, 4 if args.out_dtype == "f32" else 2)) / 3)},
    }
    if peak is not None:
        # the same matrix cores with nothing but MFMAs: the sustained clock, and with it the
        # attainable rate, depends on how many operand bits toggle
        out["roofline"]["measured_mfma_loop"] = peak
        out["roofline"]["frac_of_measured_random_int8_loop"] = round(
            gemm_tops / peak["random_int8_operands"]["TOPs"], 4)

    # the MXFP4 comparison path on the same inputs and launch configuration
    wqm = {k: dfp4.mxfp4_quantize(ops[k].to(dev)) for k in ("w_gate", "w_up", "w_down")}
    qxm, qhm = dfp4.empty_qtensor(M, H, dev, True), dfp4.empty_qtensor(M, I, dev, True)

    def step_mx():
        dfp4.mxfp4_quantize(x, out=qxm)
        dfp4.mxfp4_gemm(qxm, wqm["w_gate"], out=gate, workspace=ws)
        dfp4.mxfp4_gemm(qxm, wqm["w_up"], out=up, workspace=ws)
        dfp4.mxfp4_quantize(h, out=qhm)
        dfp4.mxfp4_gemm(qhm, wqm["w_down"], out=down, workspace=ws)

    nmx = max(10, args.steps // 4)
    for _ in range(max(3, args.warmup // 4)):
        step_mx()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(nmx):
        step_mx()
    torch.cuda.synchronize()
    ms_mx = (time.perf_counter() - t0) / nmx * 1e3
    out["mxfp4_step"] = {"ms_per_step": round(ms_mx, 4), "TOPs": round(total_ops / (ms_mx * 1e-3) / 1e12, 1),
                         "steps": nmx}
    del wqm

    # the same step on the block-scaled matrix instruction: DialectFP4 operands repacked (exactly) to
    # FP6 E2M3, weights packed once beforehand like they are quantized once beforehand
    wpk = {k: dfp4.native_pack(wq[k]) for k in ("w_gate", "w_up", "w_down")}
    lib = dfp4.load()
    xbuf = torch.empty(max(int(lib.dfp4_native_packed_bytes(M, H)), 256), dtype=torch.uint8, device=dev)
    hbuf = torch.empty(max(int(lib.dfp4_native_packed_bytes(M, I)), 256), dtype=torch.uint8, device=dev)
    ws_n = torch.empty(max(int(lib.dfp4_gemm_native_splitk_bytes(M, H, I)),
                           int(lib.dfp4_gemm_native_splitk_bytes(M, I, H)), 256), dtype=torch.uint8, device=dev)
    nnames = ["quantize_native_x", "gemm_gate", "gemm_up", "quantize_native_h", "gemm_down"]
    packed = {}

    def step_native(ev=None):
        calls = [
            # online quantization straight into the matrix instruction's operand order, once for gate and up
            lambda: packed.__setitem__("x", dfp4.quantize_native(x, buf=xbuf)),
            lambda: dfp4.gemm_native_packed(packed["x"], wpk["w_gate"], out=gate, workspace=ws_n),
            lambda: dfp4.gemm_native_packed(packed["x"], wpk["w_up"], out=up, workspace=ws_n),
            lambda: packed.__setitem__("h", dfp4.quantize_native(h, buf=hbuf)),
            lambda: dfp4.gemm_native_packed(packed["h"], wpk["w_down"], out=down, workspace=ws_n),
        ]
        for i, c in enumerate(calls):
            if ev is not None:
                ev[i][0].record()
            c()
            if ev is not None:
                ev[i][1].record()

    nn = max(10, args.steps // 2)
    for _ in range(max(3, args.warmup // 2)):
        step_native()
    torch.cuda.synchronize()
    nev = [_events(len(nnames), torch) if s % EVERY == 0 else None for s in range(nn)]
    t0 = time.perf_counter()
    for s in range(nn):
        step_native(nev[s])
    torch.cuda.synchronize()
    ms_n = (time.perf_counter() - t0) / nn * 1e3
    nev = [e for e in nev if e is not None]
    nk = {n: sum(e[i][0].elapsed_time(e[i][1]) for e in nev) / len(nev) for i, n in enumerate(nnames)}
    n_gemm_ms = sum(nk[n] for n in gemm_ops)
    n_tops = total_ops / (n_gemm_ms * 1e-3) / 1e12
    out["native_fp6_step"] = {
        "what": "same step with dfp4_quantize_native + dfp4_gemm_native_packed (v_mfma_scale_f32_32x32x64_f8f6f4, "
                "FP6 E2M3 operands, fp32 accumulation in the matrix core); weights packed beforehand, each "
                "activation quantized online straight into the packed form",
        "ms_per_step": round(ms_n, 4), "TOPs": round(total_ops / (ms_n * 1e-3) / 1e12, 1), "steps": nn,
        "kernel_ms": {k: round(v, 4) for k, v in nk.items()},
        "roofline": {"bound": "mfma", "kernel": "dfp4_gemm_native_packed call = gemm_native_kernel "
                                                 "(+ native_reduce_kernel where K is split)", "achieved": round(n_tops, 1),
                     "peak": FP6_PEAK_TOPS, "unit": "TOP/s", "frac": round(n_tops / FP6_PEAK_TOPS, 4),
                     "traffic": None}}
    del wpk

    # and the MXFP4 comparison on the same instruction (FP4 E2M1 operands are the codes themselves)
    wqm = {k: dfp4.mxfp4_quantize(ops[k].to(dev)) for k in ("w_gate", "w_up", "w_down")}
    wpm = {k: dfp4.native_pack(wqm[k], mx=True) for k in wqm}
    del wqm

    def step_native_mx():
        dfp4.mxfp4_quantize(x, out=qxm)
        px = dfp4.native_pack(qxm, mx=True, buf=xbuf)
        dfp4.gemm_native_packed(px, wpm["w_gate"], out=gate, workspace=ws_n)
        dfp4.gemm_native_packed(px, wpm["w_up"], out=up, workspace=ws_n)
        dfp4.mxfp4_quantize(h, out=qhm)
        ph = dfp4.native_pack(qhm, mx=True, buf=hbuf)
        dfp4.gemm_native_packed(ph, wpm["w_down"], out=down, workspace=ws_n)

    for _ in range(max(3, args.warmup // 4)):
        step_native_mx()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(nmx):
        step_native_mx()
    torch.cuda.synchronize()
    ms_nmx = (time.perf_counter() - t0) / nmx * 1e3
    out["native_fp4_mxfp4_step"] = {
        "what": "MXFP4 step on the same instruction: mxfp4_quantize + mxfp4_native_pack + mxfp4_gemm_native_packed",
        "ms_per_step": round(ms_nmx, 4), "TOPs": round(total_ops / (ms_nmx * 1e-3) / 1e12, 1), "steps": nmx}
    del wpm

    # the small single-linear case (few rows: bound by the weight stream, reported in GB/s)
    a1, w1 = synth.single_linear(seed=0)
    qa1, qw1 = dfp4.quantize(a1.to(dev)), dfp4.quantize(w1.to(dev))
    o1 = torch.empty((a1.shape[0], w1.shape[0]), dtype=torch.float32, device=dev)
    ws1 = torch.empty(max(dfp4.gemm_workspace_bytes(a1.shape[0], w1.shape[0], a1.shape[1]), 256), dtype=torch.uint8,
                      device=dev)
    for _ in range(5):
        dfp4.gemm(qa1, qw1, out=o1, workspace=ws1)
    ev1 = _events(30, torch)
    for i in range(30):
        ev1[i][0].record()
        dfp4.gemm(qa1, qw1, out=o1, workspace=ws1)
        ev1[i][1].record()
    torch.cuda.synchronize()
    ms1 = sorted(e[0].elapsed_time(e[1]) for e in ev1)[15]
    b1 = gemm_bytes(a1.shape[0], w1.shape[0], a1.shape[1])
    out["single_linear_32x4096x4096"] = {"ms": round(ms1, 4), "GBps": round(b1 / (ms1 * 1e-3) / 1e9, 1),
                                         "algorithmic_bytes": int(b1), "kernel": "gemm_small_kernel"}
    # the same on the block-scaled instruction (weights packed beforehand: 7 bits per element instead of 4.5)
    wp1, ap1 = dfp4.native_pack(qw1), dfp4.quantize_native(a1.to(dev))
    for _ in range(5):
        dfp4.gemm_native_packed(ap1, wp1, out=o1)
    for i in range(30):
        ev1[i][0].record()
        dfp4.gemm_native_packed(ap1, wp1, out=o1)
        ev1[i][1].record()
    torch.cuda.synchronize()
    ms1n = sorted(e[0].elapsed_time(e[1]) for e in ev1)[15]
    b1n = (a1.shape[0] + w1.shape[0]) * a1.shape[1] * (1792 + 64) / 2048 + 4 * a1.shape[0] * w1.shape[0]
    out["single_linear_32x4096x4096_native"] = {"ms": round(ms1n, 4), "GBps": round(b1n / (ms1n * 1e-3) / 1e9, 1),
                                                "packed_bytes": int(b1n), "kernel": "gemm_native_small_kernel"}
    del wp1, ap1

    if not args.no_stream_quant:
        # quantizer-only streaming tensors (Student-t, df=3): DialectFP4 and MXFP4,
        # warm (same buffer, fits the memory-side cache) and cold (rotating buffers)
        streams = synth.quantizer_streams(seed=3)
        res = {}
        for name, t in streams.items():
            rows, K = t.shape
            nrot = 6
            bufs = [t.to(dev) if i == 0 else t.to(dev).clone() for i in range(nrot)]
            for mx in (False, True):
                fn = dfp4.mxfp4_quantize if mx else dfp4.quantize
                q = dfp4.empty_qtensor(rows, K, dev, mx)
                nbytes = quant_bytes(rows, K, mx)
                for mode in ("warm", "cold"):
                    for i in range(3):
                        fn(bufs[i % nrot if mode == "cold" else 0], out=q)
                    n = 24
                    ev = _events(n, torch)
                    for i in range(n):
                        src = bufs[i % nrot] if mode == "cold" else bufs[0]
                        ev[i][0].record()
                        fn(src, out=q)
                        ev[i][1].record()
                    torch.cuda.synchronize()
                    ms = sorted(e[0].elapsed_time(e[1]) for e in ev)[n // 2]
                    res[f"{'mxfp4' if mx else 'dfp4'}_{name}_{mode}"] = {
                        "ms": round(ms, 4), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1)}
            del bufs
        out["quantizer_stream"] = res
        # both streaming tensors together, DialectFP4, rotating buffers: total bytes / total time
        cold = [(n, t) for n, t in streams.items()]
        tot_bytes = sum(quant_bytes(t.shape[0], t.shape[1]) for _, t in cold)
        tot_ms = sum(res[f"dfp4_{n}_cold"]["ms"] for n, _ in cold)
        ach = tot_bytes / (tot_ms * 1e-3) / 1e9
        out["roofline_quantizer"] = {"bound": "hbm",
                                     "kernel": "dfp4_quantize on " + " + ".join(n for n, _ in cold) +
                                               " (Student-t, rotating buffers), total bytes / total time",
                                     "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                     "frac": round(ach / HBM_PEAK_GBPS, 4),
                                     "traffic": measured_traffic("quantize_x_2048x4096_MB_per_launch"),
                                     "traffic_note": "measured on the 2048x4096 launch of the step "
                                                     "(algorithmic %d bytes)" % quant_bytes(M, H)}

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(ops)
    if args.gemm == "native":
        n = out["native_fp6_step"]
        out["int8_step"] = {"ms_per_step": out["ms_per_step"], "TOPs": out["value"], "kernel_ms": out["kernel_ms"],
                            "roofline": out["roofline"]}
        out.update({"value": n["TOPs"], "ms_per_step": n["ms_per_step"], "kernel_ms": n["kernel_ms"], "dtype": "fp6",
                    "roofline": n["roofline"], "steps": n["steps"],
                    "pct_int8_peak_step": round(100.0 * n["TOPs"] / INT8_PEAK_TOPS, 2)})
        out["config"]["gemm"] = "native (v_mfma_scale_f32_32x32x64_f8f6f4, FP6 E2M3 operands)"
    else:
        out["config"]["gemm"] = "int8 (v_mfma_i32_32x32x32_i8, exact int32 accumulation)"
    print(json.dumps(out))


if __name__ == "__main__":
    main()
