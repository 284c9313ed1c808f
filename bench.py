#!/usr/bin/env python3
"""Benchmark of the DialectFP4 hot path on one MI355X.

A step is one pass of the whole path over the LLaMA-3-8B MLP prefill batch
(M = 2048 tokens): quantize x online -> prepare it once for both products ->
gate GEMM, up GEMM (K = 4096, N = 14336) -> quantize h online -> prepare ->
down GEMM (K = 14336, N = 4096).  Weights are quantized and prepared once, before
the timed region (the paper pre-quantizes weights).  All inputs are seeded
synthetic tensors already resident in HBM.

Prints ONE JSON line.  `value` is the step's integer-op throughput (2*M*N*K summed
over the three GEMMs, divided by the whole step time including both quantizer and
both prepare launches).  `roofline` is the GEMM call against the int8 MFMA peak,
`roofline_quantizer` the quantizer against HBM on the two streaming tensors,
`cpu_baseline` the NumPy oracle on a sample of the same workload.  Further keys
hold the other configurations: the MXFP4 and block-scaled-instruction steps, the
few-rows shapes, the LLaMA-2-7B linears, the attention products, dequantization.

    python bench.py [--steps K] [--warmup W] [--sections step,mx,native,few_rows,stream,llama2,attention,dequant,cpu]
"""
import argparse
import json
import os
import subprocess
import sys
import tempfile
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
INT8_PEAK_TOPS = 5000.0
FP6_PEAK_TOPS = 10100.0
ALL_SECTIONS = ["step", "mx", "native", "few_rows", "stream", "llama2", "attention", "dequant", "cpu"]
TRAFFIC_FILE = os.path.join("profiles", "bench_hbm_traffic.txt")


def _events(n, torch):
    return [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]


SIDE_RAMP_MS = [0.0]     # set from --ramp-ms: untimed load before every side measurement


def settle(fns, torch):
    """The GPU's clock follows the load with a delay of some hundred milliseconds, and between the sections of
    this file the GPU idles while the host prepares inputs: run the calls untimed until the clock has settled."""
    if SIDE_RAMP_MS[0] <= 0:
        return
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < SIDE_RAMP_MS[0]:
        for _ in range(4):
            for fn in fns:
                fn()
        torch.cuda.synchronize()


def median_ms(fn, torch, n=20, warm=5):
    """Median duration of fn() from HIP events on the launch stream."""
    settle([fn], torch)
    for _ in range(warm):
        fn()
    ev = _events(n, torch)
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return sorted(a.elapsed_time(b) for a, b in ev)[n // 2]


def stream_ms(fns, torch, reps=4, batches=5):
    """Per-call duration of the calls in `fns` issued back to back (reps rounds over the list between
    one pair of HIP events; median over batches).  With a list whose operands together exceed the
    memory-side cache every call finds its operands in HBM, as a decode loop over many layers does."""
    settle(fns, torch)
    for fn in fns:
        fn()
    ts = []
    for _ in range(batches):
        a, b = _events(1, torch)[0]
        a.record()
        for _ in range(reps):
            for fn in fns:
                fn()
        b.record()
        torch.cuda.synchronize()
        ts.append(a.elapsed_time(b) / (reps * len(fns)))
    return sorted(ts)[len(ts) // 2]


def measured_traffic(key):
    """Per-launch HBM-side bytes measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    (scaled by a plain copy of known size); read from the summary kept under profiles/."""
    try:
        for line in open(os.path.join(ROOT, TRAFFIC_FILE)):
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


def run_helper(name, args=(), timeout=120):
    exe = os.path.join(ROOT, "bench_helpers", name)
    if not os.path.exists(exe):
        print(f"bench.py: {exe} not found (build it with `python -m paper_2501_01144_amd.build`); "
              "its figures are left out of the report", file=sys.stderr)
        return None
    r = subprocess.run([exe, *args], capture_output=True, text=True, timeout=timeout)
    if r.returncode == 0 and r.stdout.strip():
        return json.loads(r.stdout.strip().splitlines()[-1])
    print(f"bench.py: {name} failed: {r.stderr}", file=sys.stderr)
    return None


def sampled_operand_bytes(qx, qw, torch, dfp4):
    """32 KiB of the int8 operands the GEMM's matrix instructions really see, for the register-only
    MFMA loop: signed dialect magnitudes u shifted left by the block's exponent offset modulo 4
    (A blocks of a higher class appear as zeros in the class-0 pass, as in the kernel).  Built from
    the library's own dequantizer output: value = 0.5 u 2^e, so u << d = value * 2^(1 - e + d)."""
    def operand(q, rows, blocks):
        deq = dfp4.dequantize(q)[:rows, :blocks * 32].double().view(rows, blocks, 32)
        e = q.exponent[:rows].int() - 127
        ref = e.min(dim=1, keepdim=True).values
        delta = (e - ref)[:, :blocks]
        u = torch.ldexp(deq, (1 - e[:, :blocks] + (delta & 3))[:, :, None])
        u = torch.where((delta >> 2)[:, :, None] == 0, u, torch.zeros_like(u))
        return u.to(torch.int8).contiguous().view(-1)[:16384]
    a8 = operand(qx, 32, 16)
    w8 = operand(qw, 32, 16)
    return bytes(a8.cpu().numpy().tobytes()) + bytes(w8.cpu().numpy().tobytes())


def cpu_baseline(ops, target_seconds=12.0):
    """The oracle as it stands, timed on the host on a sample of the step: the first
    `tokens` rows of x and h against the first `cols` rows of each weight matrix, once with
    the numeric libraries held to one thread and once with all the threads they take.
    A short calibration run picks the sample so that each timed part takes roughly
    `target_seconds` on this machine."""
    from oracle import dfp4_oracle as O
    from paper_2501_01144_amd import synth
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threadpool_limits, cores = None, 1

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

    def sized_run(limit):
        ctx = threadpool_limits(limits=limit) if (threadpool_limits and limit) else None
        try:
            if ctx:
                ctx.__enter__()
            run(*prepare(32, 32))                     # first-call costs stay out of the calibration
            tokens, cols = 128, 256
            dt = run(*prepare(tokens, cols))
            grow = max(1.0, target_seconds / dt)
            new_tokens = int(min(ops["x"].shape[0], tokens * grow))
            grow /= new_tokens / tokens
            tokens, cols = new_tokens, int(min(4096, cols * max(1.0, grow)))
            x, h, wq = prepare(tokens, cols)
            dt = run(x, h, wq)
            if dt < 0.5 * target_seconds and cols < 4096:      # the small calibration run over-estimated the cost
                cols = int(min(4096, cols * target_seconds / dt))
                x, h, wq = prepare(tokens, cols)
                dt = run(x, h, wq)
            int_ops = 2.0 * tokens * cols * (2 * x.shape[1] + h.shape[1])
            return int_ops / dt / 1e12, dt, tokens, cols
        finally:
            if ctx:
                ctx.__exit__(None, None, None)

    v1, dt1, t1, c1 = sized_run(1)
    vn, dtn, tn, cn = sized_run(None)
    return {"value": vn, "unit": "TOP/s", "cores": int(cores), "kind": "oracle", "seconds": round(dtn, 3),
            "sample": f"{tn} tokens x {cn} output columns of each of the three GEMMs (weights pre-quantized "
                      f"untimed, activations quantized inside the timed region), NumPy float64 oracle, all threads",
            "single_thread": {"value": v1, "unit": "TOP/s", "cores": 1, "seconds": round(dt1, 3),
                              "sample": f"{t1} tokens x {c1} output columns, numeric libraries limited to one thread"}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--ramp-ms", type=float, default=400.0,
                    help="run the step untimed for this long before the warm-up steps: the GPU's power management "
                         "takes some hundred milliseconds of load to reach the clock it then sustains, and a "
                         "measurement taken earlier (the first ~100 steps) reads 12-15 %% slower than every later one")
    ap.add_argument("--out-dtype", choices=["f32", "bf16"], default="f32", help="GEMM output type")
    ap.add_argument("--gemm", choices=["int8", "native"], default="int8",
                    help="which GEMM path the headline fields describe: the int8 matrix-core path "
                         "(dfp4_gemm_prepared) or the block-scaled FP6 one (dfp4_gemm_native_packed); both are "
                         "measured and reported")
    ap.add_argument("--sections", default="all",
                    help="comma-separated subset of " + ",".join(ALL_SECTIONS) + " (profiling runs pick one or two)")
    ap.add_argument("--no-helpers", action="store_true", help="skip the child processes (MFMA loop, streaming probe)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (a known-size kernel to scale "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    sections = ALL_SECTIONS if args.sections == "all" else [s for s in args.sections.split(",") if s]
    for s in sections:
        if s not in ALL_SECTIONS:
            print(f"bench.py: unknown section {s}", file=sys.stderr)
            sys.exit(2)

    SIDE_RAMP_MS[0] = min(args.ramp_ms, 120.0)
    # register-only int8 MFMA loop in a child process, before this process touches the GPU
    peak = None if args.no_helpers else run_helper("mfma_peak")
    # and what fits in an MFMA's shadow for the lone wave per SIMD the GEMM's main loop runs (ns per MFMA)
    shadow = None if args.no_helpers else run_helper("mfma_shadow")

    import torch
    from paper_2501_01144_amd import dfp4, synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    lib = dfp4.load()
    dev = torch.device("cuda:0")
    odt = torch.float32 if args.out_dtype == "f32" else torch.bfloat16
    osz = 4 if args.out_dtype == "f32" else 2

    ops = synth.llama3_8b_mlp(seed=2)
    M, H = ops["x"].shape
    I = ops["h"].shape[1]
    x, h = ops["x"].to(dev), ops["h"].to(dev)
    wq = {k: dfp4.quantize(ops[k].to(dev)) for k in ("w_gate", "w_up", "w_down")}
    wp = {k: dfp4.gemm_prepare(wq[k], weight=True) for k in wq}
    qx, qh = dfp4.empty_qtensor(M, H, dev), dfp4.empty_qtensor(M, I, dev)
    xbuf = torch.empty(max(int(lib.dfp4_gemm_prepared_bytes(M, H, 0)), 256), dtype=torch.uint8, device=dev)
    hbuf = torch.empty(max(int(lib.dfp4_gemm_prepared_bytes(M, I, 0)), 256), dtype=torch.uint8, device=dev)
    gate = torch.empty((M, I), dtype=odt, device=dev)
    up = torch.empty((M, I), dtype=odt, device=dev)
    down = torch.empty((M, H), dtype=odt, device=dev)
    ws_bytes = max(int(lib.dfp4_gemm_prepared_workspace_bytes(M, I, H)), int(lib.dfp4_gemm_prepared_workspace_bytes(M, H, I)),
                   dfp4.gemm_workspace_bytes(M, I, H), dfp4.gemm_workspace_bytes(M, H, I))
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    gemm_ops = {"gemm_gate": 2.0 * M * I * H, "gemm_up": 2.0 * M * I * H, "gemm_down": 2.0 * M * H * I}
    total_ops = sum(gemm_ops.values())
    out = {
        "metric": "DialectFP4 quant GB/s + quantized GEMM TOPS (% int8 MFMA peak), LLaMA-3-8B shapes",
        "value": None, "unit": "TOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": None, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "LLaMA-3-8B MLP prefill, M=2048: quantize x[2048x4096] -> prepare -> gate/up GEMM "
                               "(K=4096,N=14336) -> quantize h[2048x14336] -> prepare -> down GEMM (K=14336,N=4096); "
                               "activations N(0,1) + 0.5% outlier channels x50, weights N(0,0.02), "
                               "weights pre-quantized and prepared", "M": M, "hidden": H, "intermediate": I,
                   "out_dtype": args.out_dtype, "sections": sections},
    }
    EVERY = 4        # HIP events around every call of every EVERY-th timed step

    if "step" in sections:
        names = ["quantize_x", "prepare_x", "gemm_gate", "gemm_up", "quantize_h", "prepare_h", "gemm_down"]
        prepared = {}

        def step(ev=None):
            calls = [
                lambda: dfp4.quantize(x, out=qx),
                lambda: prepared.__setitem__("x", dfp4.gemm_prepare(qx, weight=False, buf=xbuf)),
                lambda: dfp4.gemm_prepared(prepared["x"], wp["w_gate"], out=gate, workspace=ws),
                lambda: dfp4.gemm_prepared(prepared["x"], wp["w_up"], out=up, workspace=ws),
                lambda: dfp4.quantize(h, out=qh),
                lambda: prepared.__setitem__("h", dfp4.gemm_prepare(qh, weight=False, buf=hbuf)),
                lambda: dfp4.gemm_prepared(prepared["h"], wp["w_down"], out=down, workspace=ws),
            ]
            for i, c in enumerate(calls):
                if ev is not None:
                    ev[i][0].record()
                c()
                if ev is not None:
                    ev[i][1].record()

        # clock ramp (untimed, reported as config.ramp_ms), then the W warm-up steps, then exactly K timed steps
        t_ramp, ramp_steps = time.perf_counter(), 0
        while (time.perf_counter() - t_ramp) * 1e3 < args.ramp_ms:
            for _ in range(16):
                step()
            ramp_steps += 16
            torch.cuda.synchronize()
        out["config"]["ramp_ms"] = args.ramp_ms
        out["config"]["ramp_steps"] = ramp_steps
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
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
        gemm_ms = sum(kern_ms[n] for n in gemm_ops)
        gemm_tops = total_ops / (gemm_ms * 1e-3) / 1e12
        value = total_ops / (ms_per_step * 1e-3) / 1e12
        q_bytes = quant_bytes(M, H) + quant_bytes(M, I)
        q_ms = kern_ms["quantize_x"] + kern_ms["quantize_h"]
        declined = dfp4.gemm_declined_tiles(prepared["x"]) + dfp4.gemm_declined_tiles(prepared["h"])
        out.update({
            "value": round(value, 3), "ms_per_step": round(ms_per_step, 4),
            "kernel_ms": {k: round(v, 4) for k, v in kern_ms.items()},
            "pct_int8_peak_step": round(100.0 * value / INT8_PEAK_TOPS, 2),
            "quantize_in_step_GBps": round(q_bytes / (q_ms * 1e-3) / 1e9, 1),
            "roofline": {"bound": "mfma",
                         "kernel": "dfp4_gemm_prepared call = gemm_fast_kernel (3 calls per step, HIP events around each "
                                   "call on the launch stream)",
                         "achieved": round(gemm_tops, 3), "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                         "frac": round(gemm_tops / INT8_PEAK_TOPS, 4),
                         "traffic": measured_traffic("gemm_fast_kernel_avg_MB_per_launch"),
                         "traffic_source": "not measured by this run: the rocprofv3 --pmc figure kept in " + TRAFFIC_FILE,
                         "algorithmic_bytes_per_launch": round((2 * gemm_bytes(M, I, H, osz) + gemm_bytes(M, H, I, osz)) / 3),
                         "declined_tiles_last_step": declined},
        })
        # the same three products through dfp4_gemm, which prepares both operands inside every call
        plain = {"gemm_gate": median_ms(lambda: dfp4.gemm(qx, wq["w_gate"], out=gate, workspace=ws), torch, 12, 3),
                 "gemm_down": median_ms(lambda: dfp4.gemm(qh, wq["w_down"], out=down, workspace=ws), torch, 12, 3)}
        plain_ms = 2 * plain["gemm_gate"] + plain["gemm_down"]
        out["gemm_unprepared"] = {"what": "dfp4_gemm (prepares A and W inside every call): gemm_prep_kernel + gemm_fast_kernel",
                                  "ms": {k: round(v, 4) for k, v in plain.items()},
                                  "TOPs": round(total_ops / (plain_ms * 1e-3) / 1e12, 1),
                                  "frac": round(total_ops / (plain_ms * 1e-3) / 1e12 / INT8_PEAK_TOPS, 4)}
        if peak is not None:
            # the same matrix cores with nothing but MFMAs: the sustained clock, and with it the
            # attainable rate, depends on how many operand bits toggle
            with tempfile.NamedTemporaryFile(suffix=".bin", delete=False) as f:
                f.write(sampled_operand_bytes(qx, wq["w_gate"], torch, dfp4))
                path = f.name
            torch.cuda.synchronize()
            more = run_helper("mfma_peak", ["25000", path])
            os.unlink(path)
            if more is not None and "sampled_gemm_operands" in more:
                peak["sampled_gemm_operands"] = more["sampled_gemm_operands"]
            out["roofline"]["measured_mfma_loop"] = peak
            if shadow is not None:
                out["roofline"]["measured_mfma_shadow"] = shadow
            out["roofline"]["frac_of_measured_random_int8_loop"] = round(
                gemm_tops / peak["random_int8_operands"]["TOPs"], 4)
            if "sampled_gemm_operands" in peak:
                out["roofline"]["frac_of_measured_sampled_operand_loop"] = round(
                    gemm_tops / peak["sampled_gemm_operands"]["TOPs"], 4)

    nside = max(10, args.steps // 2)
    if "mx" in sections:
        # the MXFP4 comparison path on the same inputs and launch configuration
        wqm = {k: dfp4.mxfp4_quantize(ops[k].to(dev)) for k in ("w_gate", "w_up", "w_down")}
        wpm = {k: dfp4.gemm_prepare(wqm[k], weight=True, mx=True) for k in wqm}
        qxm, qhm = dfp4.empty_qtensor(M, H, dev, True), dfp4.empty_qtensor(M, I, dev, True)

        def step_mx():
            dfp4.mxfp4_quantize(x, out=qxm)
            px = dfp4.gemm_prepare(qxm, weight=False, mx=True, buf=xbuf)
            dfp4.gemm_prepared(px, wpm["w_gate"], out=gate, workspace=ws)
            dfp4.gemm_prepared(px, wpm["w_up"], out=up, workspace=ws)
            dfp4.mxfp4_quantize(h, out=qhm)
            ph = dfp4.gemm_prepare(qhm, weight=False, mx=True, buf=hbuf)
            dfp4.gemm_prepared(ph, wpm["w_down"], out=down, workspace=ws)

        for _ in range(60):          # untimed: the clock has to settle after the previous section
            step_mx()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(nside):
            step_mx()
        torch.cuda.synchronize()
        ms_mx = (time.perf_counter() - t0) / nside * 1e3
        out["mxfp4_step"] = {"ms_per_step": round(ms_mx, 4), "TOPs": round(total_ops / (ms_mx * 1e-3) / 1e12, 1),
                             "steps": nside}
        del wqm, wpm

    if "native" in sections:
        # the same step on the block-scaled matrix instruction: DialectFP4 operands repacked (exactly) to
        # FP6 E2M3, weights packed once beforehand like they are quantized once beforehand
        wpk = {k: dfp4.native_pack(wq[k]) for k in ("w_gate", "w_up", "w_down")}
        nxbuf = torch.empty(max(int(lib.dfp4_native_packed_bytes(M, H)), 256), dtype=torch.uint8, device=dev)
        nhbuf = torch.empty(max(int(lib.dfp4_native_packed_bytes(M, I)), 256), dtype=torch.uint8, device=dev)
        ws_n = torch.empty(max(int(lib.dfp4_gemm_native_splitk_bytes(M, H, I)),
                               int(lib.dfp4_gemm_native_splitk_bytes(M, I, H)), 256), dtype=torch.uint8, device=dev)
        nnames = ["quantize_native_x", "gemm_gate", "gemm_up", "quantize_native_h", "gemm_down"]
        packed = {}

        def step_native(ev=None):
            calls = [
                # online quantization straight into the matrix instruction's operand order, once for gate and up
                lambda: packed.__setitem__("x", dfp4.quantize_native(x, buf=nxbuf)),
                lambda: dfp4.gemm_native_packed(packed["x"], wpk["w_gate"], out=gate, workspace=ws_n),
                lambda: dfp4.gemm_native_packed(packed["x"], wpk["w_up"], out=up, workspace=ws_n),
                lambda: packed.__setitem__("h", dfp4.quantize_native(h, buf=nhbuf)),
                lambda: dfp4.gemm_native_packed(packed["h"], wpk["w_down"], out=down, workspace=ws_n),
            ]
            for i, c in enumerate(calls):
                if ev is not None:
                    ev[i][0].record()
                c()
                if ev is not None:
                    ev[i][1].record()

        for _ in range(60):          # untimed: the clock has to settle after the previous section
            step_native()
        torch.cuda.synchronize()
        nev = [_events(len(nnames), torch) if s % EVERY == 0 else None for s in range(nside)]
        t0 = time.perf_counter()
        for s in range(nside):
            step_native(nev[s])
        torch.cuda.synchronize()
        ms_n = (time.perf_counter() - t0) / nside * 1e3
        nev = [e for e in nev if e is not None]
        nk = {n: sum(e[i][0].elapsed_time(e[i][1]) for e in nev) / len(nev) for i, n in enumerate(nnames)}
        n_gemm_ms = sum(nk[n] for n in gemm_ops)
        n_tops = total_ops / (n_gemm_ms * 1e-3) / 1e12
        out["native_fp6_step"] = {
            "what": "same step with dfp4_quantize_native + dfp4_gemm_native_packed (v_mfma_scale_f32_32x32x64_f8f6f4, "
                    "FP6 E2M3 operands, fp32 accumulation in the matrix core); weights packed beforehand, each "
                    "activation quantized online straight into the packed form",
            "ms_per_step": round(ms_n, 4), "TOPs": round(total_ops / (ms_n * 1e-3) / 1e12, 1), "steps": nside,
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
        qxm, qhm = dfp4.empty_qtensor(M, H, dev, True), dfp4.empty_qtensor(M, I, dev, True)

        def step_native_mx():
            dfp4.mxfp4_quantize(x, out=qxm)
            px = dfp4.native_pack(qxm, mx=True, buf=nxbuf)
            dfp4.gemm_native_packed(px, wpm["w_gate"], out=gate, workspace=ws_n)
            dfp4.gemm_native_packed(px, wpm["w_up"], out=up, workspace=ws_n)
            dfp4.mxfp4_quantize(h, out=qhm)
            ph = dfp4.native_pack(qhm, mx=True, buf=nhbuf)
            dfp4.gemm_native_packed(ph, wpm["w_down"], out=down, workspace=ws_n)

        for _ in range(60):          # untimed: the clock has to settle after the previous section
            step_native_mx()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(nside):
            step_native_mx()
        torch.cuda.synchronize()
        ms_nmx = (time.perf_counter() - t0) / nside * 1e3
        out["native_fp4_mxfp4_step"] = {
            "what": "MXFP4 step on the same instruction: mxfp4_quantize + mxfp4_native_pack + mxfp4_gemm_native_packed",
            "ms_per_step": round(ms_nmx, 4), "TOPs": round(total_ops / (ms_nmx * 1e-3) / 1e12, 1), "steps": nside}
        del wpm

    if "few_rows" in sections:
        # few rows of A (decode shapes): bound by the weight stream, reported in GB/s of the 4-bit operands.
        # "ms" brackets single calls with events (launch latency included: the time one isolated call
        # takes); "stream" issues calls back to back over enough copies of the weights (> 320 MB together,
        # more than the memory-side cache holds) that every call streams its weights from HBM.
        res = {}
        for (m1, n1, k1) in ((32, 4096, 4096), (16, 14336, 4096), (1, 4096, 4096)):
            a1 = synth.gaussian_outlier_channels(m1, k1, 8, 30.0, 1.0, seed=0)
            w1 = synth.gaussian(n1, k1, 0.02, seed=1000)
            qa1, qw1 = dfp4.quantize(a1.to(dev)), dfp4.quantize(w1.to(dev))
            o1 = torch.empty((m1, n1), dtype=torch.float32, device=dev)
            b1 = gemm_bytes(m1, n1, k1)
            ncopy = int(320e6 // b1) + 1
            qws = [qw1] + [dfp4.QTensor(qw1.codes.clone(), qw1.dialect.clone(), qw1.exponent.clone(), qw1.rows, qw1.K)
                           for _ in range(ncopy - 1)]
            ms1 = median_ms(lambda: dfp4.gemm(qa1, qw1, out=o1), torch, 30, 5)
            ms1s = stream_ms([(lambda q=q: dfp4.gemm(qa1, q, out=o1)) for q in qws], torch)
            entry = {"ms": round(ms1, 4), "stream_ms": round(ms1s, 4), "weight_copies": ncopy,
                     "GBps": round(b1 / (ms1s * 1e-3) / 1e9, 1), "algorithmic_bytes": int(b1),
                     "frac_hbm": round(b1 / (ms1s * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                     "kernel": "gemm_small_kernel (dfp4_gemm: per-block fp32 flush, nothing prepared)"}
            # weights prepared offline, the activation prepared once: exact sums, no per-block floating point
            pa1 = dfp4.gemm_prepare(qa1, weight=False)
            pws = [dfp4.gemm_prepare(q, weight=True) for q in qws]
            ms1p = median_ms(lambda: dfp4.gemm_prepared(pa1, pws[0], out=o1), torch, 30, 5)
            ms1ps = stream_ms([(lambda w=w: dfp4.gemm_prepared(pa1, w, out=o1)) for w in pws], torch)
            ms1a = median_ms(lambda: dfp4.gemm_prepare(qa1, weight=False, buf=pa1.buf), torch, 30, 5)
            b1p = b1 + n1 * (k1 // 32) * 4          # + one table dword per block of W
            entry["prepared"] = {"ms": round(ms1p, 4), "stream_ms": round(ms1ps, 4),
                                 "GBps": round(b1p / (ms1ps * 1e-3) / 1e9, 1),
                                 "frac_hbm": round(b1p / (ms1ps * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                                 "bytes": int(b1p), "prepare_a_ms": round(ms1a, 4),
                                 "kernel": "gemm_rows_kernel (dfp4_gemm_prepared)"}
            del pa1, pws
            # the same on the block-scaled instruction (weights packed beforehand: 7 bits per element instead of 4.5)
            wps, ap1 = [dfp4.native_pack(q) for q in qws], dfp4.quantize_native(a1.to(dev))
            ms1n = median_ms(lambda: dfp4.gemm_native_packed(ap1, wps[0], out=o1), torch, 30, 5)
            ms1ns = stream_ms([(lambda w=w: dfp4.gemm_native_packed(ap1, w, out=o1)) for w in wps], torch)
            b1n = (m1 + n1) * k1 * (1792 + 64) / 2048 + 4 * m1 * n1
            entry["native"] = {"ms": round(ms1n, 4), "stream_ms": round(ms1ns, 4),
                               "GBps": round(b1n / (ms1ns * 1e-3) / 1e9, 1),
                               "frac_hbm": round(b1n / (ms1ns * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                               "packed_bytes": int(b1n), "kernel": "gemm_native_small_kernel"}
            res[f"{m1}x{n1}x{k1}"] = entry
            del wps, ap1, qa1, qw1, qws
        out["few_rows"] = res
        out["single_linear_32x4096x4096"] = res["32x4096x4096"]

    if "stream" in sections:
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
                    settle([(lambda b=b: fn(b, out=q)) for b in (bufs if mode == "cold" else bufs[:1])], torch)
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
                                     "per_tensor_frac": {n: round(res[f"dfp4_{n}_cold"]["GBps"] / HBM_PEAK_GBPS, 4)
                                                         for n, _ in cold},
                                     "traffic": measured_traffic("quantize_8192x4096_MB_per_launch"),
                                     "traffic_source": "not measured by this run: the rocprofv3 --pmc figure kept in "
                                                       + TRAFFIC_FILE + " for the 8192x4096 launch (algorithmic %d bytes)"
                                                       % quant_bytes(8192, 4096)}
        if not args.no_helpers:
            torch.cuda.synchronize()
            sp = run_helper("stream_peak")
            if sp is not None:
                # plain streaming kernels with the quantizer's access structure and no arithmetic
                out["roofline_quantizer"]["measured_stream"] = sp
                for n, t in cold:
                    key = f"{t.shape[0]}x{t.shape[1]}"
                    if key in sp:
                        out["roofline_quantizer"].setdefault("frac_of_measured_stream", {})[n] = round(
                            res[f"dfp4_{n}_cold"]["GBps"] / sp[key]["read_write_GBps"], 4)

    if "llama2" in sections:
        # LLaMA-2-7B decoder linears at M = 4096 tokens, operands prepared ahead as in the step
        g = synth.llama2_7b_linears(seed=4)
        M4 = g["x"].shape[0]
        qx4, qh4 = dfp4.quantize(g["x"].to(dev)), dfp4.quantize(g["h"].to(dev))
        px4, ph4 = dfp4.gemm_prepare(qx4, weight=False), dfp4.gemm_prepare(qh4, weight=False)
        res = {}
        tot_ops4, tot_ms4 = 0.0, 0.0
        for name, act in (("w_qkv", px4), ("w_o", px4), ("w_gate", px4), ("w_up", px4), ("w_down", ph4)):
            w = g[name]
            N4, K4 = w.shape
            pw4 = dfp4.gemm_prepare(dfp4.quantize(w.to(dev)), weight=True)
            o4 = torch.empty((M4, N4), dtype=odt, device=dev)
            ws4 = torch.empty(max(int(lib.dfp4_gemm_prepared_workspace_bytes(M4, N4, K4)), 256), dtype=torch.uint8, device=dev)
            ms4 = median_ms(lambda: dfp4.gemm_prepared(act, pw4, out=o4, workspace=ws4), torch, 12, 4)
            ops4 = 2.0 * M4 * N4 * K4
            tot_ops4 += ops4
            tot_ms4 += ms4
            res[name] = {"M": M4, "N": N4, "K": K4, "ms": round(ms4, 4), "TOPs": round(ops4 / (ms4 * 1e-3) / 1e12, 1),
                         "frac": round(ops4 / (ms4 * 1e-3) / 1e12 / INT8_PEAK_TOPS, 4)}
            del pw4, o4, ws4
        res["declined_tiles"] = dfp4.gemm_declined_tiles(px4) + dfp4.gemm_declined_tiles(ph4)
        res["all_five"] = {"TOPs": round(tot_ops4 / (tot_ms4 * 1e-3) / 1e12, 1),
                           "frac": round(tot_ops4 / (tot_ms4 * 1e-3) / 1e12 / INT8_PEAK_TOPS, 4)}
        out["llama2_7b_linears_M4096"] = res
        del g, qx4, qh4, px4, ph4

    if "attention" in sections:
        # attention products of all 4 x 32 heads at sequence length 2048, head size 128 (Appendix C):
        # Q K^T is bound by the write of the scores (reported in GB/s), P V by the matrix cores
        B5, H5, S5, D5 = 4, 32, 2048, 128
        bh = B5 * H5
        ao = synth.attention_operands(seed=5, B=B5, H=H5, S=S5, D=D5)
        qq = dfp4.quantize(ao["q"].reshape(bh * S5, D5).to(dev))
        qk = dfp4.quantize(ao["k"].reshape(bh * S5, D5).to(dev))
        qvt = dfp4.quantize(ao["vt"].reshape(bh * D5, S5).to(dev))
        del ao
        res = {}
        ws5 = torch.empty(max(dfp4.gemm_workspace_bytes(S5, S5, D5), dfp4.gemm_workspace_bytes(S5, D5, S5), 256) * bh,
                          dtype=torch.uint8, device=dev)
        for dt5, nm in ((torch.float32, "f32"), (torch.bfloat16, "bf16")):
            sc = torch.empty((bh, S5, S5), dtype=dt5, device=dev)
            ms5 = median_ms(lambda: dfp4.gemm_batched(qq, qk, bh, S5, S5, out=sc, workspace=ws5), torch, 8, 2)
            nbytes = bh * gemm_bytes(S5, S5, D5, 4 if nm == "f32" else 2)
            res["qk_scores_" + nm] = {"ms": round(ms5, 4), "GBps": round(nbytes / (ms5 * 1e-3) / 1e9, 1),
                                      "frac_hbm": round(nbytes / (ms5 * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                                      "TOPs": round(2.0 * bh * S5 * S5 * D5 / (ms5 * 1e-3) / 1e12, 1),
                                      "algorithmic_bytes": int(nbytes)}
            del sc
        # P: softmax of seeded random logits, generated on the device (1 GiB of bf16)
        gen = torch.Generator(device=dev)
        gen.manual_seed(55)
        qp = dfp4.empty_qtensor(bh * S5, S5, dev)
        for b0 in range(0, bh, 16):
            logits = torch.randn((16 * S5, S5), generator=gen, device=dev, dtype=torch.float32)
            part = dfp4.quantize(torch.softmax(logits, dim=-1).to(torch.bfloat16))
            qp.codes[b0 * S5:(b0 + 16) * S5] = part.codes
            qp.dialect[b0 * S5:(b0 + 16) * S5] = part.dialect
            qp.exponent[b0 * S5:(b0 + 16) * S5] = part.exponent
            del logits, part
        ctx = torch.empty((bh, S5, D5), dtype=odt, device=dev)
        ms5 = median_ms(lambda: dfp4.gemm_batched(qp, qvt, bh, S5, D5, out=ctx, workspace=ws5), torch, 8, 2)
        ops5 = 2.0 * bh * S5 * D5 * S5
        res["pv_context"] = {"ms": round(ms5, 4), "TOPs": round(ops5 / (ms5 * 1e-3) / 1e12, 1),
                             "frac": round(ops5 / (ms5 * 1e-3) / 1e12 / INT8_PEAK_TOPS, 4),
                             "GBps": round(bh * gemm_bytes(S5, D5, S5, osz) / (ms5 * 1e-3) / 1e9, 1),
                             "workspace_bytes": int(ws5.numel())}
        res["shape"] = {"batch": bh, "seq": S5, "head_dim": D5}
        out["attention_products"] = res
        del qq, qk, qvt, qp, ctx, ws5

    if "dequant" in sections:
        # dequantization of the first streaming tensor: reads 0.5625 B/element, writes 2 or 4
        t = synth.quantizer_streams(seed=3)["act_8192x4096"]
        q = dfp4.quantize(t.to(dev))
        res = {}
        for dt6, nm, ob in ((torch.bfloat16, "bf16", 2), (torch.float32, "f32", 4)):
            y = torch.empty(t.shape, dtype=dt6, device=dev)
            ms6 = median_ms(lambda: dfp4.dequantize(q, out=y), torch, 24, 4)
            nbytes = t.numel() * (0.5 + 2.0 / 32.0 + ob)
            res[nm] = {"ms": round(ms6, 4), "GBps": round(nbytes / (ms6 * 1e-3) / 1e9, 1),
                       "frac_hbm": round(nbytes / (ms6 * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
            del y
        out["dequantize_8192x4096"] = res

    if "cpu" in sections:
        out["cpu_baseline"] = cpu_baseline(ops)
    if args.gemm == "native" and "native_fp6_step" in out:
        n = out["native_fp6_step"]
        out["int8_step"] = {"ms_per_step": out["ms_per_step"], "TOPs": out["value"], "kernel_ms": out.get("kernel_ms"),
                            "roofline": out.get("roofline")}
        out.update({"value": n["TOPs"], "ms_per_step": n["ms_per_step"], "kernel_ms": n["kernel_ms"], "dtype": "fp6",
                    "roofline": n["roofline"], "steps": n["steps"],
                    "pct_int8_peak_step": round(100.0 * n["TOPs"] / INT8_PEAK_TOPS, 2)})
        out["config"]["gemm"] = "native (v_mfma_scale_f32_32x32x64_f8f6f4, FP6 E2M3 operands)"
    else:
        out["config"]["gemm"] = "int8 (v_mfma_i32_32x32x32_i8, exact int32 accumulation)"
    print(json.dumps(out))


if __name__ == "__main__":
    main()
