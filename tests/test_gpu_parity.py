"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Quantizer outputs (codes, dialect ids, exponent
bytes) must match bit for bit; dequantization is exact; the GEMM must satisfy
|out - ref| <= 1e-5 * sum_k |A^[m,k]| |W^[n,k]| with ref the float64 product of
the oracle's dequantized operands."""
import numpy as np
import pytest
import torch

from oracle import dfp4_oracle as O
from oracle import mxfp4_oracle as MX
from paper_2501_01144_amd import dfp4, synth

pytestmark = pytest.mark.gpu
GEMM_RTOL = 1e-5


@pytest.fixture(scope="module", autouse=True)
def _library():
    assert torch.cuda.is_available(), "GPU tests need a device"
    dfp4.load()


def _dev(x):
    return x.cuda()


def _np(t):
    return t.cpu().numpy()


def _assert_quant_equal(q, ref, what):
    codes, dialect, expo = ref
    got_e, got_d, got_c = _np(q.exponent), _np(q.dialect), _np(q.codes)
    assert np.array_equal(got_e, expo), f"{what}: exponent bytes differ at {np.argwhere(got_e != expo)[:4]}"
    assert np.array_equal(got_d, dialect), f"{what}: dialect ids differ at {np.argwhere(got_d != dialect)[:4]}"
    assert np.array_equal(got_c, codes), f"{what}: codes differ at {np.argwhere(got_c != codes)[:4]}"


def _check_quantize(x_bf16, what):
    print(f"quantize parity: {what} shape={tuple(x_bf16.shape)}", flush=True)
    q = dfp4.quantize(_dev(x_bf16))
    torch.cuda.synchronize()
    _assert_quant_equal(q, O.dfp4_quantize(synth.to_f64(x_bf16)), what)
    qm = dfp4.mxfp4_quantize(_dev(x_bf16))
    torch.cuda.synchronize()
    codes, expo = MX.mxfp4_quantize(synth.to_f64(x_bf16))
    assert np.array_equal(_np(qm.exponent), expo), f"{what}: mx exponent"
    assert np.array_equal(_np(qm.codes), codes), f"{what}: mx codes at {np.argwhere(_np(qm.codes) != codes)[:4]}"
    return q, qm


# --------------------------------------------------------------------------
# quantizer
# --------------------------------------------------------------------------
def test_quantize_single_linear_activation():
    a, _ = synth.single_linear(seed=0)
    _check_quantize(a, "config1 A")


@pytest.mark.parametrize("rows,K", [(1, 32), (3, 96), (5, 2048), (65, 64), (127, 4096), (1000, 1056)])
def test_quantize_ragged_shapes(rows, K):
    # sizes that end inside a wavefront's 64-block group and inside a 16-block load
    _check_quantize(synth.student_t(rows, K, 3.0, seed=rows + K), f"t3 {rows}x{K}")


def test_quantize_every_bf16_value():
    x = synth.all_bf16_bit_patterns()                       # [2040, 32]: one block per row
    _check_quantize(x, "all finite bf16 patterns")
    # each value also as a lone element next to a larger block maximum
    g = torch.Generator().manual_seed(1)
    y = x[torch.randperm(x.shape[0], generator=g)].reshape(-1, 64)
    _check_quantize(y, "all finite bf16 patterns, shuffled pairs of rows")


def test_quantize_degenerate_blocks():
    x = torch.zeros(8, 128, dtype=torch.bfloat16)
    x[1, 5] = -0.0
    x[2, 40] = 1.0                                          # single nonzero
    x[3, :32] = 7.875                                       # rounded maximum 8.0
    x[3, 32:64] = 7.75
    x[4, 64:96] = torch.tensor(2.0 ** -133).to(torch.bfloat16)   # smallest subnormal
    x[5, :] = torch.tensor(3.3895e38).to(torch.bfloat16)    # largest finite
    x[6, ::3] = -1.5
    x[7, 96:] = torch.linspace(-8, 8, 32).to(torch.bfloat16)
    _check_quantize(x, "degenerate blocks")


def test_quantize_wide_dynamic_range_and_ties():
    g = torch.Generator().manual_seed(4)
    x = torch.randn(256, 512, generator=g) * torch.exp2(torch.randint(-120, 120, (256, 16), generator=g)
                                                        .repeat_interleave(32, dim=1).float())
    _check_quantize(x.to(torch.bfloat16), "wide range")
    ties = (torch.randint(-64, 64, (256, 512), generator=g).float() / 8).to(torch.bfloat16)
    _check_quantize(ties, "multiples of 1/8 (every rounding tie)")


def test_quantize_strided_rows():
    base = synth.student_t(64, 1024, 3.0, seed=9)
    view = base[:, 128:128 + 512]                           # ld = 1024, K = 512
    q = dfp4.quantize(_dev(base)[:, 128:128 + 512])
    torch.cuda.synchronize()
    _assert_quant_equal(q, O.dfp4_quantize(synth.to_f64(view.contiguous())), "strided")


def test_quantize_streaming_tensor_sampled_rows():
    # full-size streaming tensor in the benchmark's launch configuration;
    # the oracle checks a seeded sample of rows
    x = synth.student_t(8192, 4096, 3.0, seed=3)
    q = dfp4.quantize(_dev(x))
    qm = dfp4.mxfp4_quantize(_dev(x))
    torch.cuda.synchronize()
    rows = np.sort(np.random.default_rng(0).choice(8192, 96, replace=False))
    rows = np.concatenate([rows, [0, 8191]])
    ref = O.dfp4_quantize(synth.to_f64(x[rows]))
    assert np.array_equal(_np(q.codes)[rows], ref[0])
    assert np.array_equal(_np(q.dialect)[rows], ref[1])
    assert np.array_equal(_np(q.exponent)[rows], ref[2])
    refm = MX.mxfp4_quantize(synth.to_f64(x[rows]))
    assert np.array_equal(_np(qm.codes)[rows], refm[0])
    assert np.array_equal(_np(qm.exponent)[rows], refm[1])
    # properties that hold at any size: ids in range, exponent = max exponent field - 2
    assert int(q.dialect.max()) <= 15
    amax = x.abs().view(8192, -1, 32).amax(dim=2).float()
    _, ex = torch.frexp(amax)                               # amax = m * 2^ex, m in [0.5, 1)
    want = torch.where(amax == 0, torch.zeros_like(ex), torch.clamp(ex - 1 - 2 + 127, min=0)).to(torch.uint8)
    assert torch.equal(q.exponent.cpu(), want)


def test_quantize_second_streaming_tensor_sampled_rows():
    # 4096 x 14336 Student-t tensor (448 blocks per row) in the benchmark's launch configuration
    x = synth.student_t(4096, 14336, 3.0, seed=4)
    print("quantize parity: 4096x14336 sampled rows", flush=True)
    q = dfp4.quantize(_dev(x))
    qm = dfp4.mxfp4_quantize(_dev(x))
    torch.cuda.synchronize()
    rows = np.sort(np.random.default_rng(1).choice(4096, 48, replace=False))
    rows = np.concatenate([rows, [0, 4095]])
    ref = O.dfp4_quantize(synth.to_f64(x[rows]))
    assert np.array_equal(_np(q.codes)[rows], ref[0])
    assert np.array_equal(_np(q.dialect)[rows], ref[1])
    assert np.array_equal(_np(q.exponent)[rows], ref[2])
    refm = MX.mxfp4_quantize(synth.to_f64(x[rows]))
    assert np.array_equal(_np(qm.codes)[rows], refm[0])
    assert np.array_equal(_np(qm.exponent)[rows], refm[1])
    assert int(q.dialect.max()) <= 15
    amax = x.abs().view(4096, -1, 32).amax(dim=2).float()
    _, ex = torch.frexp(amax)
    want = torch.where(amax == 0, torch.zeros_like(ex), torch.clamp(ex - 1 - 2 + 127, min=0)).to(torch.uint8)
    assert torch.equal(q.exponent.cpu(), want)


# --------------------------------------------------------------------------
# dequantizer
# --------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_dequantize_exact(dtype):
    x = torch.cat([synth.student_t(37, 1088, 3.0, seed=12),
                   synth.all_bf16_bit_patterns().reshape(-1, 1088)])
    xf = synth.to_f64(x)
    q = dfp4.quantize(_dev(x))
    y = dfp4.dequantize(q, dtype)
    torch.cuda.synchronize()
    ref = O.dfp4_dequantize(*O.dfp4_quantize(xf))
    got = y.cpu().to(torch.float64).numpy()
    assert np.array_equal(got, ref)
    assert np.array_equal(np.signbit(got), np.signbit(ref))
    qm = dfp4.mxfp4_quantize(_dev(x))
    ym = dfp4.mxfp4_dequantize(qm, dtype)
    torch.cuda.synchronize()
    assert np.array_equal(ym.cpu().to(torch.float64).numpy(), MX.mxfp4_dequantize(*MX.mxfp4_quantize(xf)))


def test_dequantize_strided_output():
    x = synth.gaussian(16, 256, 1.0, seed=5)
    q = dfp4.quantize(_dev(x))
    buf = torch.full((16, 512), 99.0, dtype=torch.float32, device="cuda")
    dfp4.dequantize(q, out=buf[:, 64:64 + 256])
    torch.cuda.synchronize()
    ref = O.dfp4_dequantize(*O.dfp4_quantize(synth.to_f64(x)))
    assert np.array_equal(buf[:, 64:320].cpu().double().numpy(), ref)
    assert (buf[:, :64] == 99).all() and (buf[:, 320:] == 99).all()


# --------------------------------------------------------------------------
# GEMM
# --------------------------------------------------------------------------
def _gemm_ref(a_f64, w_f64, mx=False):
    if mx:
        ad = MX.mxfp4_dequantize(*MX.mxfp4_quantize(a_f64))
        wd = MX.mxfp4_dequantize(*MX.mxfp4_quantize(w_f64))
    else:
        ad = O.dfp4_dequantize(*O.dfp4_quantize(a_f64))
        wd = O.dfp4_dequantize(*O.dfp4_quantize(w_f64))
    return ad @ wd.T, np.abs(ad) @ np.abs(wd).T


def _assert_gemm_close(got, ref, absdot, what, bf16=False):
    got = got.cpu().to(torch.float64).numpy()
    if bf16:
        want = torch.from_numpy(ref).to(torch.bfloat16).to(torch.float64).numpy()
        ulp = np.exp2(np.floor(np.log2(np.maximum(np.abs(want), 1e-300))) - 7)
        assert (np.abs(got - want) <= ulp + GEMM_RTOL * absdot).all(), what
        return
    err = np.abs(got - ref)
    bad = err > GEMM_RTOL * absdot
    assert not bad.any(), f"{what}: {bad.sum()} outputs off, worst {np.max(err / np.maximum(absdot, 1e-300)):.3e}"


def test_gemm_single_linear_full():
    a, w = synth.single_linear(seed=0)
    print("gemm parity: config1 32x4096x4096", flush=True)
    out = dfp4.gemm(dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w)))
    torch.cuda.synchronize()
    ref, absdot = _gemm_ref(synth.to_f64(a), synth.to_f64(w))
    _assert_gemm_close(out, ref, absdot, "config1")
    outm = dfp4.mxfp4_gemm(dfp4.mxfp4_quantize(_dev(a)), dfp4.mxfp4_quantize(_dev(w)))
    torch.cuda.synchronize()
    refm, absm = _gemm_ref(synth.to_f64(a), synth.to_f64(w), mx=True)
    _assert_gemm_close(outm, refm, absm, "config1 mxfp4")


@pytest.mark.parametrize("M,N,K", [(1, 1, 32), (70, 200, 160), (129, 257, 96), (300, 130, 1024)])
def test_gemm_ragged_shapes(M, N, K):
    print(f"gemm parity: ragged {M}x{N}x{K}", flush=True)
    a = synth.gaussian_outlier_channels(M, K, max(1, K // 100), 50.0, 1.0, seed=M)
    w = synth.student_t(N, K, 3.0, seed=N)
    qa, qw = dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w))
    ref, absdot = _gemm_ref(synth.to_f64(a), synth.to_f64(w))
    out = dfp4.gemm(qa, qw)
    torch.cuda.synchronize()
    _assert_gemm_close(out, ref, absdot, "f32")
    outb = dfp4.gemm(qa, qw, dtype=torch.bfloat16)
    torch.cuda.synchronize()
    _assert_gemm_close(outb, ref, absdot, "bf16", bf16=True)
    # leading dimension larger than N, surroundings untouched
    buf = torch.full((M, N + 24), -7.0, dtype=torch.float32, device="cuda")
    dfp4.gemm(qa, qw, out=buf[:, 8:8 + N])
    torch.cuda.synchronize()
    _assert_gemm_close(buf[:, 8:8 + N], ref, absdot, "ldc")
    assert (buf[:, :8] == -7).all() and (buf[:, 8 + N:] == -7).all()


def test_gemm_wide_exponent_spread():
    # blocks whose exponents differ by tens of binades along K
    g = torch.Generator().manual_seed(6)
    scale = torch.exp2(torch.randint(-30, 30, (96, 8), generator=g).repeat_interleave(32, dim=1).float())
    a = (torch.randn(96, 256, generator=g) * scale).to(torch.bfloat16)
    w = (torch.randn(160, 256, generator=g) * scale[:1]).to(torch.bfloat16)
    out = dfp4.gemm(dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w)))
    torch.cuda.synchronize()
    ref, absdot = _gemm_ref(synth.to_f64(a), synth.to_f64(w))
    _assert_gemm_close(out, ref, absdot, "wide spread")


def test_gemm_batched():
    B, M, N, K = 3, 80, 144, 128
    a = synth.gaussian_outlier_channels(B * M, K, 2, 30.0, 1.0, seed=31)
    w = synth.gaussian_outlier_channels(B * N, K, 2, 30.0, 1.0, seed=32)
    out = dfp4.gemm_batched(dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w)), B, M, N)
    torch.cuda.synchronize()
    for b in range(B):
        ref, absdot = _gemm_ref(synth.to_f64(a[b * M:(b + 1) * M]), synth.to_f64(w[b * N:(b + 1) * N]))
        _assert_gemm_close(out[b], ref, absdot, f"batch {b}")


def test_gemm_mlp_prefill_sampled_outputs():
    # LLaMA-3-8B gate projection at full size, in the benchmark's launch
    # configuration; the oracle computes a seeded sample of rows x columns
    ops = synth.llama3_8b_mlp(seed=2)
    x, w = ops["x"], ops["w_gate"]
    print("gemm parity: 2048x14336x4096 sampled", flush=True)
    out = dfp4.gemm(dfp4.quantize(_dev(x)), dfp4.quantize(_dev(w)))
    torch.cuda.synchronize()
    rng = np.random.default_rng(1)
    rows = np.sort(rng.choice(x.shape[0], 24, replace=False))
    cols = np.sort(rng.choice(w.shape[0], 192, replace=False))
    ref, absdot = _gemm_ref(synth.to_f64(x[rows]), synth.to_f64(w[cols]))
    _assert_gemm_close(out[rows][:, cols], ref, absdot, "mlp gate sampled")
    # down projection, K = 14336
    h, wd = ops["h"], ops["w_down"]
    out = dfp4.gemm(dfp4.quantize(_dev(h)), dfp4.quantize(_dev(wd)))
    torch.cuda.synchronize()
    cols = np.sort(rng.choice(wd.shape[0], 64, replace=False))
    ref, absdot = _gemm_ref(synth.to_f64(h[rows]), synth.to_f64(wd[cols]))
    _assert_gemm_close(out[rows][:, cols], ref, absdot, "mlp down sampled")


def test_gemm_mlp_prefill_bf16_sampled_outputs():
    # bf16 output of a full-size GEMM (full tiles store two adjacent columns per lane)
    ops = synth.llama3_8b_mlp(seed=2)
    x, w = ops["x"], ops["w_up"]
    print("gemm parity: 2048x14336x4096 bf16 sampled", flush=True)
    out = dfp4.gemm(dfp4.quantize(_dev(x)), dfp4.quantize(_dev(w)), dtype=torch.bfloat16)
    torch.cuda.synchronize()
    rng = np.random.default_rng(2)
    rows = np.sort(rng.choice(x.shape[0], 24, replace=False))
    cols = np.sort(rng.choice(w.shape[0], 192, replace=False))
    ref, absdot = _gemm_ref(synth.to_f64(x[rows]), synth.to_f64(w[cols]))
    _assert_gemm_close(out[rows][:, cols], ref, absdot, "mlp up bf16 sampled", bf16=True)


def test_gemm_some_tiles_declined():
    # rows 520..539 carry block exponents spread over tens of binades, so the second 512-row
    # tile goes to the per-block-flush fallback while the first one takes the fast path
    g = torch.Generator().manual_seed(9)
    M, N, K = 600, 300, 512
    a = torch.randn(M, K, generator=g)
    scale = torch.exp2(torch.randint(-25, 25, (20, K // 32), generator=g).repeat_interleave(32, dim=1).float())
    a[520:540] *= scale
    a = a.to(torch.bfloat16)
    w = (torch.randn(N, K, generator=g) * 0.02).to(torch.bfloat16)
    print("gemm parity: 600x300x512 with declined tiles", flush=True)
    out = dfp4.gemm(dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w)))
    torch.cuda.synchronize()
    ref, absdot = _gemm_ref(synth.to_f64(a), synth.to_f64(w))
    _assert_gemm_close(out, ref, absdot, "mixed fast and declined tiles")


def test_gemm_llama2_down_projection_sampled_outputs():
    # LLaMA-2-7B down projection at M = 4096: K = 11008 is 344 blocks (not a multiple of 16)
    g = synth.llama2_7b_linears(seed=4)
    h, w = g["h"], g["w_down"]
    print("gemm parity: 4096x4096x11008 sampled", flush=True)
    out = dfp4.gemm(dfp4.quantize(_dev(h)), dfp4.quantize(_dev(w)))
    torch.cuda.synchronize()
    rng = np.random.default_rng(4)
    rows = np.sort(rng.choice(h.shape[0], 16, replace=False))
    cols = np.sort(rng.choice(w.shape[0], 96, replace=False))
    ref, absdot = _gemm_ref(synth.to_f64(h[rows]), synth.to_f64(w[cols]))
    _assert_gemm_close(out[rows][:, cols], ref, absdot, "llama2 down sampled")


@pytest.mark.parametrize("name,N", [("w_qkv", 12288), ("w_o", 4096), ("w_gate", 11008)])
def test_gemm_llama2_linears_sampled_outputs(name, N):
    # the other LLaMA-2-7B linears at M = 4096, K = 4096, full size, sampled outputs
    g = synth.llama2_7b_linears(seed=4)
    x, w = g["x"], g[name]
    assert w.shape[0] == N
    print(f"gemm parity: 4096x{N}x4096 ({name}) sampled", flush=True)
    out = dfp4.gemm(dfp4.quantize(_dev(x)), dfp4.quantize(_dev(w)))
    torch.cuda.synchronize()
    rng = np.random.default_rng(40 + N)
    rows = np.sort(np.concatenate([rng.choice(x.shape[0], 14, replace=False), [0, x.shape[0] - 1]]))
    cols = np.sort(np.concatenate([rng.choice(N, 94, replace=False), [0, N - 1]]))
    ref, absdot = _gemm_ref(synth.to_f64(x[rows]), synth.to_f64(w[cols]))
    _assert_gemm_close(out[rows][:, cols], ref, absdot, f"llama2 {name} sampled")


def test_gemm_attention_full_batch_first_and_last_head():
    # both attention products at the full batch of 4 x 32 = 128 heads; the oracle checks
    # sampled outputs of the first and the last head (the largest batch offsets)
    B, H, S, D = 4, 32, 2048, 128
    bh = B * H
    ops = synth.attention_operands(seed=5, B=B, H=H, S=S, D=D)
    q, k, vt = ops["q"], ops["k"], ops["vt"]
    print("gemm parity: attention 128 heads Q K^T", flush=True)
    out = dfp4.gemm_batched(dfp4.quantize(_dev(q.reshape(bh * S, D))), dfp4.quantize(_dev(k.reshape(bh * S, D))), bh, S, S)
    torch.cuda.synchronize()
    rng = np.random.default_rng(50)
    rows = np.sort(np.concatenate([rng.choice(S, 14, replace=False), [0, S - 1]]))
    cols = np.sort(np.concatenate([rng.choice(S, 126, replace=False), [0, S - 1]]))
    for hd in (0, 77, bh - 1):
        ref, absdot = _gemm_ref(synth.to_f64(q[hd][rows]), synth.to_f64(k[hd][cols]))
        _assert_gemm_close(out[hd][rows][:, cols], ref, absdot, f"QK^T head {hd}")
    del out
    print("gemm parity: attention 128 heads P V", flush=True)
    # P: softmax rows, generated per head to bound host memory; only the checked heads are kept
    qp = dfp4.empty_qtensor(bh * S, S, torch.device("cuda:0"))
    keep = {}
    for hd in range(bh):
        p = synth.softmax_rows(S, S, seed=5000 + hd)
        part = dfp4.quantize(_dev(p))
        qp.codes[hd * S:(hd + 1) * S] = part.codes
        qp.dialect[hd * S:(hd + 1) * S] = part.dialect
        qp.exponent[hd * S:(hd + 1) * S] = part.exponent
        if hd in (0, bh - 1):
            keep[hd] = p
    out = dfp4.gemm_batched(qp, dfp4.quantize(_dev(vt.reshape(bh * D, S))), bh, S, D)
    torch.cuda.synchronize()
    for hd in (0, bh - 1):
        ref, absdot = _gemm_ref(synth.to_f64(keep[hd][rows]), synth.to_f64(vt[hd]))
        _assert_gemm_close(out[hd][rows], ref, absdot, f"PV head {hd}")


def test_gemm_attention_shapes_batched_sampled():
    # attention matmuls at the real sequence length and head size, 4 of the 128 heads:
    # Q K^T (K = 128, blocks along the head dimension) and P V (K = 2048, blocks along the sequence)
    B, H, S, D = 1, 4, 2048, 128
    ops = synth.attention_operands(seed=5, B=B, H=H, S=S, D=D)
    q, k, vt = ops["q"], ops["k"], ops["vt"]
    print("gemm parity: attention 4 heads Q K^T", flush=True)
    out = dfp4.gemm_batched(dfp4.quantize(_dev(q.reshape(H * S, D))), dfp4.quantize(_dev(k.reshape(H * S, D))), H, S, S)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    rows = np.sort(rng.choice(S, 16, replace=False))
    cols = np.sort(rng.choice(S, 128, replace=False))
    for hd in (0, 3):
        ref, absdot = _gemm_ref(synth.to_f64(q[hd][rows]), synth.to_f64(k[hd][cols]))
        _assert_gemm_close(out[hd][rows][:, cols], ref, absdot, f"QK^T head {hd}")
    print("gemm parity: attention 4 heads P V", flush=True)
    p = synth.softmax_rows(H * S, S, seed=55)
    out = dfp4.gemm_batched(dfp4.quantize(_dev(p)), dfp4.quantize(_dev(vt.reshape(H * D, S))), H, S, D)
    torch.cuda.synchronize()
    for hd in (1, 2):
        ref, absdot = _gemm_ref(synth.to_f64(p[hd * S:(hd + 1) * S][rows]), synth.to_f64(vt[hd]))
        _assert_gemm_close(out[hd][rows], ref, absdot, f"PV head {hd}")


@pytest.mark.parametrize("M,N,K", [(5, 40, 64), (33, 100, 4096), (64, 96, 256), (16, 4096, 14336)])
def test_gemm_few_rows(M, N, K):
    # decode shapes (M <= 64) take the W-streaming kernel: per-block exponent pairs in fp32
    print(f"gemm parity: few rows {M}x{N}x{K}", flush=True)
    a = synth.gaussian_outlier_channels(M, K, max(1, K // 200), 50.0, 1.0, seed=100 + M)
    w = synth.gaussian(N, K, 0.02, seed=200 + N)
    ref, absdot = _gemm_ref(synth.to_f64(a), synth.to_f64(w))
    out = dfp4.gemm(dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w)))
    torch.cuda.synchronize()
    _assert_gemm_close(out, ref, absdot, "few rows f32")
    outb = dfp4.gemm(dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w)), dtype=torch.bfloat16)
    torch.cuda.synchronize()
    _assert_gemm_close(outb, ref, absdot, "few rows bf16", bf16=True)
    refm, absm = _gemm_ref(synth.to_f64(a), synth.to_f64(w), mx=True)
    outm = dfp4.mxfp4_gemm(dfp4.mxfp4_quantize(_dev(a)), dfp4.mxfp4_quantize(_dev(w)))
    torch.cuda.synchronize()
    _assert_gemm_close(outm, refm, absm, "few rows mxfp4")


@pytest.mark.parametrize("scale,K,exact", [(30.0, 4096, True), (2.0 ** 13, 512, False)])
def test_gemm_few_rows_both_forms_of_the_tile(scale, K, exact):
    # Nothing prepared, at most 64 rows: a tile whose exponents allow it is summed exactly in int32 (one
    # rounding of the exact sum, checked here to half an ulp); a tile with outliers 13 binades above the
    # rest cannot be and takes one fp32 term per block (held to the usual tolerance).
    M, N = 32, 96
    print(f"gemm parity: few rows {M}x{N}x{K}, outliers x{scale}, exact={exact}", flush=True)
    a = synth.gaussian_outlier_channels(M, K, 4, scale, 1.0, seed=901)
    w = synth.gaussian(N, K, 0.02, seed=902)
    ref, absdot = _gemm_ref(synth.to_f64(a), synth.to_f64(w))
    out = dfp4.gemm(dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w)))
    torch.cuda.synchronize()
    _assert_gemm_close(out, ref, absdot, "few rows, both forms")
    if exact:
        err = np.abs(out.cpu().double().numpy() - ref)
        assert (err <= np.abs(ref) * 2.0 ** -24 + 1e-300).all(), "more than one rounding of the exact sum"


def test_gemm_very_long_k_takes_block_flush_kernel():
    # K beyond the single-accumulator kernel's range (more than 512 blocks): every tile is
    # computed block by block with fp32 accumulation
    M, N, K = 70, 64, 32 * 520
    print(f"gemm parity: long K {M}x{N}x{K}", flush=True)
    a = synth.gaussian(M, K, 1.0, seed=71)
    w = synth.gaussian(N, K, 0.02, seed=72)
    out = dfp4.gemm(dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w)))
    torch.cuda.synchronize()
    ref, absdot = _gemm_ref(synth.to_f64(a), synth.to_f64(w))
    _assert_gemm_close(out, ref, absdot, "long K")


def test_gemm_batched_with_split_k():
    # few tiles per problem and a long K: the K ranges of every batch entry are summed separately
    B, M, N, K = 2, 100, 200, 2048
    print(f"gemm parity: batched split K {B}x{M}x{N}x{K}", flush=True)
    a = synth.gaussian_outlier_channels(B * M, K, 8, 50.0, 1.0, seed=81)
    w = synth.gaussian(B * N, K, 0.02, seed=82)
    out = dfp4.gemm_batched(dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w)), B, M, N)
    torch.cuda.synchronize()
    for b in range(B):
        ref, absdot = _gemm_ref(synth.to_f64(a[b * M:(b + 1) * M]), synth.to_f64(w[b * N:(b + 1) * N]))
        _assert_gemm_close(out[b], ref, absdot, f"batch {b}")


# --------------------------------------------------------------------------
# offline quantizer with MSE-based dialect selection
# --------------------------------------------------------------------------
def _check_quantize_mse(x_bf16, what):
    print(f"quantize_mse parity: {what} shape={tuple(x_bf16.shape)}", flush=True)
    q = dfp4.quantize_mse(_dev(x_bf16))
    torch.cuda.synchronize()
    _assert_quant_equal(q, O.dfp4_quantize_mse(synth.to_f64(x_bf16)), what)
    return q


@pytest.mark.parametrize("rows,K", [(1, 32), (7, 96), (33, 4096), (257, 1056)])
def test_quantize_mse_shapes(rows, K):
    _check_quantize_mse(synth.student_t(rows, K, 3.0, seed=rows + K), "student-t")
    _check_quantize_mse(synth.gaussian(rows, K, 0.02, seed=rows), "weights")


def test_quantize_mse_every_bf16_value_and_ties():
    _check_quantize_mse(synth.all_bf16_bit_patterns(), "all finite bf16 values")
    g = torch.Generator().manual_seed(12)
    grid = (torch.randint(-64, 64, (64, 256), generator=g).float() / 8.0).to(torch.bfloat16)   # many equal errors
    _check_quantize_mse(grid, "multiples of 1/8")
    scale = torch.exp2(torch.randint(-120, 120, (64, 8), generator=g).repeat_interleave(32, dim=1).float())
    _check_quantize_mse((torch.randn(64, 256, generator=g) * scale).to(torch.bfloat16), "wide range")
    _check_quantize_mse(torch.zeros(4, 64, dtype=torch.bfloat16), "zeros")


def test_gemm_with_mse_quantized_weights():
    M, N, K = 96, 160, 512
    a = synth.gaussian_outlier_channels(M, K, 4, 50.0, 1.0, seed=91)
    w = synth.gaussian(N, K, 0.02, seed=92)
    out = dfp4.gemm(dfp4.quantize(_dev(a)), dfp4.quantize_mse(_dev(w)))
    torch.cuda.synchronize()
    ad = O.dfp4_dequantize(*O.dfp4_quantize(synth.to_f64(a)))
    wd = O.dfp4_dequantize(*O.dfp4_quantize_mse(synth.to_f64(w)))
    _assert_gemm_close(out, ad @ wd.T, np.abs(ad) @ np.abs(wd).T, "mse weights")


# --------------------------------------------------------------------------
# transposing quantizer (blocks along the rows of the input)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("rows,cols", [(32, 8), (96, 72), (2048, 128), (160, 264), (4096, 64)])
def test_quantize_transposed(rows, cols):
    print(f"quantize_t parity: {rows}x{cols}", flush=True)
    x = synth.gaussian_outlier_channels(rows, cols, max(1, cols // 64), 30.0, 1.0, seed=rows + cols)
    xt = synth.to_f64(x).T.copy()
    q = dfp4.quantize_t(_dev(x))
    torch.cuda.synchronize()
    assert (q.rows, q.K) == (cols, rows)
    _assert_quant_equal(q, O.dfp4_quantize(xt), "transposed")
    qm = dfp4.mxfp4_quantize_t(_dev(x))
    torch.cuda.synchronize()
    codes, expo = MX.mxfp4_quantize(xt)
    assert np.array_equal(_np(qm.exponent), expo) and np.array_equal(_np(qm.codes), codes)


def test_quantize_transposed_strided_input_and_pv_product():
    # V stored [S, D] inside a wider buffer; P V with V quantized along the sequence by the
    # transposing quantizer equals the product with an explicitly transposed V
    S, D = 256, 64
    buf = synth.gaussian(S, D + 16, 1.0, seed=77).cuda()
    v = buf[:, 8:8 + D]
    qv = dfp4.quantize_t(v)
    torch.cuda.synchronize()
    vt = synth.to_f64(v.cpu()).T.copy()
    _assert_quant_equal(qv, O.dfp4_quantize(vt), "strided transposed")
    p = synth.softmax_rows(96, S, seed=78)
    out = dfp4.gemm(dfp4.quantize(_dev(p)), qv)
    torch.cuda.synchronize()
    ref, absdot = _gemm_ref(synth.to_f64(p), vt)
    _assert_gemm_close(out, ref, absdot, "P V")


# --------------------------------------------------------------------------
# GEMM on operands prepared ahead (dfp4_gemm_prepare / dfp4_gemm_prepared)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("M,N,K,why", [(600, 352, 512, "whole tiles"), (100, 256, 4096, "split K"),
                                       (2048, 1024, 2048, "many tiles"), (33, 100, 4096, "few rows"),
                                       (70, 200, 160, "ragged")])
def test_gemm_prepared_matches_oracle_and_gemm(M, N, K, why):
    print(f"gemm_prepared parity: {why} {M}x{N}x{K}", flush=True)
    a = synth.gaussian_outlier_channels(M, K, max(1, K // 200), 50.0, 1.0, seed=500 + M)
    w = synth.gaussian(N, K, 0.02, seed=600 + N)
    qa, qw = dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w))
    pa, pw = dfp4.gemm_prepare(qa, weight=False), dfp4.gemm_prepare(qw, weight=True)
    ref, absdot = _gemm_ref(synth.to_f64(a), synth.to_f64(w))
    want = dfp4.gemm(qa, qw)
    # the same prepared A serves several products in a row (its arrival counters return to zero)
    for rep in range(3):
        out = dfp4.gemm_prepared(pa, pw)
        torch.cuda.synchronize()
        _assert_gemm_close(out, ref, absdot, f"prepared {why} rep {rep}")
        if M > 64:
            assert torch.equal(out.view(torch.int32), want.view(torch.int32)), "prepared and plain GEMM differ"
        else:
            # few rows: the prepared form takes the exact scheme (one rounding of the exact sum),
            # the plain call adds one fp32 term per block
            assert (np.abs(out.cpu().double().numpy() - ref) <= np.abs(ref) * 2.0 ** -23 + 1e-300).all()
    outb = dfp4.gemm_prepared(pa, pw, dtype=torch.bfloat16)
    torch.cuda.synchronize()
    _assert_gemm_close(outb, ref, absdot, f"prepared {why} bf16", bf16=True)
    assert dfp4.gemm_declined_tiles(pa) == 0
    # MXFP4
    qam, qwm = dfp4.mxfp4_quantize(_dev(a)), dfp4.mxfp4_quantize(_dev(w))
    outm = dfp4.gemm_prepared(dfp4.gemm_prepare(qam, weight=False, mx=True), dfp4.gemm_prepare(qwm, weight=True, mx=True))
    torch.cuda.synchronize()
    refm, absm = _gemm_ref(synth.to_f64(a), synth.to_f64(w), mx=True)
    _assert_gemm_close(outm, refm, absm, f"prepared mxfp4 {why}")


@pytest.mark.parametrize("M,N,K", [(1, 1, 32), (5, 40, 64), (33, 100, 4096), (64, 96, 256), (32, 4096, 4096),
                                   (16, 14336, 4096), (16, 4096, 14336)])
def test_gemm_prepared_few_rows(M, N, K):
    # decode shapes on prepared operands: the few-rows kernel with exact int32 sums
    print(f"gemm_prepared parity: few rows {M}x{N}x{K}", flush=True)
    a = synth.gaussian_outlier_channels(M, K, max(1, K // 200), 50.0, 1.0, seed=700 + M)
    w = synth.gaussian(N, K, 0.02, seed=800 + N)
    qa, qw = dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w))
    pa, pw = dfp4.gemm_prepare(qa, weight=False), dfp4.gemm_prepare(qw, weight=True)
    ref, absdot = _gemm_ref(synth.to_f64(a), synth.to_f64(w))
    for dtype in (torch.float32, torch.bfloat16):
        out = dfp4.gemm_prepared(pa, pw, dtype=dtype)
        torch.cuda.synchronize()
        _assert_gemm_close(out, ref, absdot, f"few rows prepared {dtype}", bf16=dtype == torch.bfloat16)
        if dtype == torch.float32:
            assert (np.abs(out.cpu().double().numpy() - ref) <= np.abs(ref) * 2.0 ** -23 + 1e-300).all()
    assert dfp4.gemm_declined_tiles(pa) == 0
    qam, qwm = dfp4.mxfp4_quantize(_dev(a)), dfp4.mxfp4_quantize(_dev(w))
    outm = dfp4.gemm_prepared(dfp4.gemm_prepare(qam, weight=False, mx=True), dfp4.gemm_prepare(qwm, weight=True, mx=True))
    torch.cuda.synchronize()
    refm, absm = _gemm_ref(synth.to_f64(a), synth.to_f64(w), mx=True)
    _assert_gemm_close(outm, refm, absm, "few rows prepared mxfp4")


def test_gemm_prepared_few_rows_wide_exponents():
    # classes on both operands, absent class sums, and spreads the exact scheme declines
    # (spreads are those of the drawn powers of two; block maxima of Gaussian data add about one binade)
    for case, (sa, sw) in enumerate([(5, 2), (9, 0), (0, 9), (30, 30)]):
        g = torch.Generator().manual_seed(900 + case)
        M, N, K = 40, 200, 512           # 16 blocks: class sum 2 in every block stays within the int32 bound
        def operand(rows, spread, std):
            x = torch.randn(rows, K, generator=g) * std
            sh = torch.randint(0, spread + 1, (rows, K // 32, 1), generator=g)
            if case == 1 or case == 2:
                sh = torch.where(sh >= 4, torch.full_like(sh, 9), torch.zeros_like(sh))    # classes 0 and 2 only
            return (x.view(rows, K // 32, 32) * torch.exp2(sh.float())).view(rows, K).to(torch.bfloat16)
        a, w = operand(M, sa, 1.0), operand(N, sw, 0.02)
        qa, qw = dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w))
        pa, pw = dfp4.gemm_prepare(qa, weight=False), dfp4.gemm_prepare(qw, weight=True)
        out = dfp4.gemm_prepared(pa, pw)
        torch.cuda.synchronize()
        ref, absdot = _gemm_ref(synth.to_f64(a), synth.to_f64(w))
        _assert_gemm_close(out, ref, absdot, f"few rows prepared, spreads {sa}/{sw}")
        assert (dfp4.gemm_declined_tiles(pa) > 0) == (case == 3)


def test_gemm_prepared_declined_tiles_are_counted():
    # second 512-row tile: block exponents spread over tens of binades -> per-block fp32 path,
    # computed by the workgroup that finds it; the first tile takes the exact path
    g = torch.Generator().manual_seed(19)
    M, N, K = 700, 300, 512
    a = torch.randn(M, K, generator=g)
    scale = torch.exp2(torch.randint(-25, 25, (20, K // 32), generator=g).repeat_interleave(32, dim=1).float())
    a[520:540] *= scale
    a = a.to(torch.bfloat16)
    w = (torch.randn(N, K, generator=g) * 0.02).to(torch.bfloat16)
    qa, qw = dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w))
    pa, pw = dfp4.gemm_prepare(qa, weight=False), dfp4.gemm_prepare(qw, weight=True)
    out = dfp4.gemm_prepared(pa, pw)
    torch.cuda.synchronize()
    ref, absdot = _gemm_ref(synth.to_f64(a), synth.to_f64(w))
    _assert_gemm_close(out, ref, absdot, "prepared, mixed exact and declined tiles")
    assert dfp4.gemm_declined_tiles(pa) == 3              # the three column tiles of the second row tile


@pytest.mark.parametrize("spread_a,spread_w,K,expect_declined", [
    (0, 7, 1024, False), (7, 0, 1024, False), (3, 7, 1024, False),
    (4, 4, 512, False),      # class 1 on both sides: visits of class sum 2, 16 blocks stay within the int32 bound
    (4, 4, 1024, True),      # the same over 32 blocks could overflow int32 in the worst case
    (7, 7, 1024, True), (0, 13, 1024, True)])
def test_gemm_prepared_classes_on_both_operands(spread_a, spread_w, K, expect_declined):
    # block exponents spread over `spread` binades along K on either operand: the exact path takes
    # every pair (class of A, class of W) whose sum stays within the classes kept; beyond that the
    # tile is computed block by block in fp32.  Either way the result meets the oracle.
    M, N = 520, 260
    g = torch.Generator().manual_seed(100 + 16 * spread_a + spread_w)
    def operand(rows, spread, std):
        x = torch.randn(rows, K, generator=g) * std
        # every block max lands in the same binade, then a per-block power of two spreads them
        x = x.view(rows, K // 32, 32)
        x[:, :, 0] = 3.0 * std * torch.sign(x[:, :, 0] + 1e-9)
        x = torch.clamp(x, -3.0 * std, 3.0 * std)
        sh = torch.randint(0, spread + 1, (rows, K // 32, 1), generator=g)
        sh[:, 0] = 0
        sh[:, 1] = spread
        return (x * torch.exp2(sh.float())).view(rows, K).to(torch.bfloat16)
    a, w = operand(M, spread_a, 1.0), operand(N, spread_w, 0.02)
    qa, qw = dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w))
    ea, ew = qa.exponent.int(), qw.exponent.int()
    assert int((ea.max(dim=1).values - ea.min(dim=1).values).max()) == spread_a
    assert int((ew.max(dim=1).values - ew.min(dim=1).values).max()) == spread_w
    pa, pw = dfp4.gemm_prepare(qa, weight=False), dfp4.gemm_prepare(qw, weight=True)
    out = dfp4.gemm_prepared(pa, pw)
    torch.cuda.synchronize()
    ref, absdot = _gemm_ref(synth.to_f64(a), synth.to_f64(w))
    _assert_gemm_close(out, ref, absdot, f"spread A {spread_a} W {spread_w}")
    assert (dfp4.gemm_declined_tiles(pa) > 0) == expect_declined
    if not expect_declined:
        # exact path: one rounding of the exact sum
        got = out.cpu().double().numpy()
        assert (np.abs(got - ref) <= np.abs(ref) * 2.0 ** -23 + 1e-300).all()


def test_gemm_prepared_shared_activation_full_size():
    # LLaMA-3-8B gate and up projections on one prepared activation, then the down projection
    # (K split between workgroups), sampled outputs against the oracle
    ops = synth.llama3_8b_mlp(seed=2)
    x, h = ops["x"], ops["h"]
    print("gemm_prepared parity: 2048x14336x4096 (gate, up) and 2048x4096x14336 (down) sampled", flush=True)
    px = dfp4.gemm_prepare(dfp4.quantize(_dev(x)), weight=False)
    rng = np.random.default_rng(7)
    rows = np.sort(rng.choice(x.shape[0], 16, replace=False))
    for name in ("w_gate", "w_up"):
        w = ops[name]
        pw = dfp4.gemm_prepare(dfp4.quantize(_dev(w)), weight=True)
        out = dfp4.gemm_prepared(px, pw)
        torch.cuda.synchronize()
        cols = np.sort(rng.choice(w.shape[0], 128, replace=False))
        ref, absdot = _gemm_ref(synth.to_f64(x[rows]), synth.to_f64(w[cols]))
        _assert_gemm_close(out[rows][:, cols], ref, absdot, f"prepared {name} sampled")
    ph = dfp4.gemm_prepare(dfp4.quantize(_dev(h)), weight=False)
    pw = dfp4.gemm_prepare(dfp4.quantize(_dev(ops["w_down"])), weight=True)
    for rep in range(2):
        out = dfp4.gemm_prepared(ph, pw)
        torch.cuda.synchronize()
        cols = np.sort(rng.choice(4096, 64, replace=False))
        ref, absdot = _gemm_ref(synth.to_f64(h[rows]), synth.to_f64(ops["w_down"][cols]))
        _assert_gemm_close(out[rows][:, cols], ref, absdot, f"prepared down sampled rep {rep}")
    assert dfp4.gemm_declined_tiles(px) == 0 and dfp4.gemm_declined_tiles(ph) == 0


# --------------------------------------------------------------------------
# GEMM with requantizing epilogue
# --------------------------------------------------------------------------
def _requant_ref(a_bf16, w_bf16, mx=False):
    a64, w64 = synth.to_f64(a_bf16), synth.to_f64(w_bf16)
    if mx:
        prod = MX.mxfp4_dequantize(*MX.mxfp4_quantize(a64)) @ MX.mxfp4_dequantize(*MX.mxfp4_quantize(w64)).T
        return MX.mxfp4_quantize(O.round_to_bf16(prod))
    return O.dfp4_gemm_requant(O.dfp4_quantize(a64), O.dfp4_quantize(w64))


@pytest.mark.parametrize("M,N,K", [(600, 352, 512), (512, 128, 64), (130, 96, 1024)])
def test_gemm_requant_fused_tiles_bit_exact(M, N, K):
    # enough tiles that K is not split and moderate exponent spreads: every tile takes the
    # single-accumulator kernel, whose sums are exact, so the quantized result must equal the
    # oracle's bit for bit
    print(f"gemm_requant parity: {M}x{N}x{K}", flush=True)
    a = synth.gaussian_outlier_channels(M, K, max(1, K // 128), 50.0, 1.0, seed=300 + M)
    w = synth.gaussian(N, K, 0.02, seed=400 + N)
    qa, qw = dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w))
    q = dfp4.gemm_requant(qa, qw)
    torch.cuda.synchronize()
    _assert_quant_equal(q, _requant_ref(a, w), "requant")
    qm = dfp4.mxfp4_gemm_requant(dfp4.mxfp4_quantize(_dev(a)), dfp4.mxfp4_quantize(_dev(w)))
    torch.cuda.synchronize()
    codes, expo = _requant_ref(a, w, mx=True)
    assert np.array_equal(_np(qm.exponent), expo) and np.array_equal(_np(qm.codes), codes)


def test_gemm_requant_full_size_sampled_rows():
    ops = synth.llama3_8b_mlp(seed=2)
    x, w = ops["x"], ops["w_gate"]
    print("gemm_requant parity: 2048x14336x4096 sampled rows", flush=True)
    q = dfp4.gemm_requant(dfp4.quantize(_dev(x)), dfp4.quantize(_dev(w)))
    torch.cuda.synchronize()
    rows = np.sort(np.random.default_rng(6).choice(x.shape[0], 6, replace=False))
    codes, dialect, expo = _requant_ref(x[rows], w)
    assert np.array_equal(_np(q.exponent)[rows], expo)
    assert np.array_equal(_np(q.dialect)[rows], dialect)
    assert np.array_equal(_np(q.codes)[rows], codes)


def test_gemm_requant_split_k_bit_exact():
    # few tiles: K is split between workgroups whose exact int32 partial tiles are added before the
    # single conversion, so the requantized result must equal the oracle's bit for bit
    M, N, K = 100, 256, 4096
    print(f"gemm_requant parity: split K {M}x{N}x{K}", flush=True)
    a = synth.gaussian_outlier_channels(M, K, 20, 50.0, 1.0, seed=77)
    w = synth.gaussian(N, K, 0.02, seed=78)
    q = dfp4.gemm_requant(dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w)))
    torch.cuda.synchronize()
    _assert_quant_equal(q, _requant_ref(a, w), "requant split K")


@pytest.mark.parametrize("B,M,N,K", [(3, 600, 352, 128), (5, 40, 64, 256), (2, 2048, 2048, 128)])
def test_gemm_requant_batched(B, M, N, K):
    # attention-like batches: every problem's quantized scores against the oracle, bit for bit where the
    # sums are exact (more than 64 rows), to the fp32-accumulation bar otherwise
    print(f"gemm_requant_batched parity: {B} x {M}x{N}x{K}", flush=True)
    a = synth.gaussian_outlier_channels(B * M, K, 2, 30.0, 1.0, seed=310 + M)
    w = synth.gaussian_outlier_channels(B * N, K, 2, 30.0, 1.0, seed=311 + N)
    q = dfp4.gemm_requant_batched(dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w)), B, M, N)
    torch.cuda.synchronize()
    for b in (range(B) if M <= 600 else (0, B - 1)):
        rows = slice(b * M, (b + 1) * M) if M <= 600 else slice(b * M + 1000, b * M + 1032)
        ab = a[rows]
        wb = w[b * N:(b + 1) * N]
        if M > 64:
            codes, dialect, expo = _requant_ref(ab, wb)
            assert np.array_equal(_np(q.exponent)[rows], expo), f"problem {b}"
            assert np.array_equal(_np(q.dialect)[rows], dialect), f"problem {b}"
            assert np.array_equal(_np(q.codes)[rows], codes), f"problem {b}"
        else:
            ref, _ = _gemm_ref(synth.to_f64(ab), synth.to_f64(wb))
            codes, dialect, expo = O.dfp4_quantize(O.round_to_bf16(ref))
            same = np.array_equal(_np(q.codes)[rows], codes)
            # few rows accumulate in fp32: nearly all blocks reproduce the oracle's
            agree = (_np(q.exponent)[rows] == expo).mean()
            assert agree > 0.99 and (same or (_np(q.codes)[rows] == codes).mean() > 0.99)


def test_gemm_requant_handworked_block(golden_dir):
    # the hand-worked product of tests/golden (products on and just below a bf16 midpoint)
    import json, os
    g = json.load(open(os.path.join(golden_dir, "handworked_requant.json")))
    a = torch.zeros(1, 96)
    a[0, 0::32] = torch.tensor(g["a_blocks"])
    w = torch.zeros(32, 96)
    for j, row in enumerate(g["w_rows"]):
        w[j, 0::32] = torch.tensor(row)
    q = dfp4.gemm_requant(dfp4.quantize(_dev(a.to(torch.bfloat16))), dfp4.quantize(_dev(w.to(torch.bfloat16))))
    torch.cuda.synchronize()
    nib = _np(q.codes)[0]
    nib = np.stack([nib & 15, nib >> 4], axis=1).reshape(-1)
    assert int(q.exponent[0, 0]) == g["exponent_byte"] and int(q.dialect[0, 0]) == g["dialect"]
    assert list(nib[:8]) == g["codes"] and (nib[8:] == 0).all()


@pytest.mark.parametrize("M,N,K,why", [(16, 256, 512, "few rows"), (96, 160, 256, "declined tiles")])
def test_gemm_requant_fp32_accumulating_paths(M, N, K, why):
    # paths that add one fp32 term per block: the bf16 result may differ from the oracle's by one
    # bf16 ulp where the fp32 sum rounds across a bf16 midpoint.  Bar: every bf16 value within one
    # ulp of the oracle's, and every block whose 32 bf16 values all equal the oracle's carries the
    # oracle's exponent byte, dialect id and codes.
    print(f"gemm_requant parity: {why} {M}x{N}x{K}", flush=True)
    g = torch.Generator().manual_seed(M)
    a = torch.randn(M, K, generator=g)
    if why == "declined tiles":
        a = a * torch.exp2(torch.randint(-30, 30, (M, K // 32), generator=g).repeat_interleave(32, dim=1).float())
    a = a.to(torch.bfloat16)
    w = (torch.randn(N, K, generator=g) * 0.02).to(torch.bfloat16)
    qa, qw = dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w))
    q = dfp4.gemm_requant(qa, qw)
    gb = dfp4.gemm(qa, qw, dtype=torch.bfloat16)
    torch.cuda.synchronize()
    ref, absdot = _gemm_ref(synth.to_f64(a), synth.to_f64(w))
    rb = O.round_to_bf16(ref)
    got = gb.cpu().double().numpy()
    ulp = np.exp2(np.floor(np.log2(np.maximum(np.abs(rb), 1e-300))) - 7)
    assert (np.abs(got - rb) <= ulp + GEMM_RTOL * absdot).all()
    same = (got == rb).reshape(M, N // 32, 32).all(axis=2)
    assert same.mean() > 0.5, "too few blocks reproduce the oracle's bf16 values to say anything"
    codes, dialect, expo = O.dfp4_quantize(rb)
    assert np.array_equal(_np(q.exponent)[same], expo[same])
    assert np.array_equal(_np(q.dialect)[same], dialect[same])
    assert np.array_equal(_np(q.codes).reshape(M, N // 32, 16)[same], codes.reshape(M, N // 32, 16)[same])
    # the blocks that differ are quantizations of the bf16 values the GPU did compute
    cg, dg, eg = O.dfp4_quantize(got)
    assert np.array_equal(_np(q.codes), cg) and np.array_equal(_np(q.dialect), dg) and np.array_equal(_np(q.exponent), eg)


# --------------------------------------------------------------------------
# MXFP4 on the block-scaled matrix instruction
# --------------------------------------------------------------------------
@pytest.mark.parametrize("M,N,K", [(1, 1, 32), (70, 200, 160), (300, 130, 1056), (512, 512, 4096)])
def test_mxfp4_gemm_native(M, N, K):
    print(f"mxfp4_gemm_native parity: {M}x{N}x{K}", flush=True)
    a = synth.gaussian_outlier_channels(M, K, max(1, K // 100), 50.0, 1.0, seed=500 + M)
    w = synth.student_t(N, K, 3.0, seed=600 + N)
    qa, qw = dfp4.mxfp4_quantize(_dev(a)), dfp4.mxfp4_quantize(_dev(w))
    ref, absdot = _gemm_ref(synth.to_f64(a), synth.to_f64(w), mx=True)
    out = dfp4.mxfp4_gemm_native(qa, qw)
    torch.cuda.synchronize()
    _assert_gemm_close(out, ref, absdot, "native f32")
    outb = dfp4.mxfp4_gemm_native(qa, qw, dtype=torch.bfloat16)
    torch.cuda.synchronize()
    _assert_gemm_close(outb, ref, absdot, "native bf16", bf16=True)


def test_mxfp4_gemm_native_wide_exponents_and_full_size_sample():
    g = torch.Generator().manual_seed(16)
    scale = torch.exp2(torch.randint(-40, 40, (96, 8), generator=g).repeat_interleave(32, dim=1).float())
    a = (torch.randn(96, 256, generator=g) * scale).to(torch.bfloat16)
    w = (torch.randn(160, 256, generator=g) * scale[:1]).to(torch.bfloat16)
    out = dfp4.mxfp4_gemm_native(dfp4.mxfp4_quantize(_dev(a)), dfp4.mxfp4_quantize(_dev(w)))
    torch.cuda.synchronize()
    ref, absdot = _gemm_ref(synth.to_f64(a), synth.to_f64(w), mx=True)
    _assert_gemm_close(out, ref, absdot, "native wide")
    ops = synth.llama3_8b_mlp(seed=2)
    x, wg = ops["x"], ops["w_gate"]
    out = dfp4.mxfp4_gemm_native(dfp4.mxfp4_quantize(_dev(x)), dfp4.mxfp4_quantize(_dev(wg)))
    torch.cuda.synchronize()
    rng = np.random.default_rng(17)
    rows = np.sort(rng.choice(x.shape[0], 16, replace=False))
    cols = np.sort(rng.choice(wg.shape[0], 128, replace=False))
    ref, absdot = _gemm_ref(synth.to_f64(x[rows]), synth.to_f64(wg[cols]), mx=True)
    _assert_gemm_close(out[rows][:, cols], ref, absdot, "native full size sampled")


@pytest.mark.parametrize("M,N,K", [(1, 1, 32), (70, 200, 160), (300, 130, 1056), (512, 512, 4096)])
def test_dfp4_gemm_native(M, N, K):
    # DialectFP4 operands repacked to FP6 E2M3 (exact) on the block-scaled matrix instruction
    print(f"dfp4_gemm_native parity: {M}x{N}x{K}", flush=True)
    a = synth.gaussian_outlier_channels(M, K, max(1, K // 100), 50.0, 1.0, seed=700 + M)
    w = synth.student_t(N, K, 3.0, seed=800 + N)
    qa, qw = dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w))
    ref, absdot = _gemm_ref(synth.to_f64(a), synth.to_f64(w))
    out = dfp4.gemm_native(qa, qw)
    torch.cuda.synchronize()
    _assert_gemm_close(out, ref, absdot, "native fp6 f32")
    outb = dfp4.gemm_native(qa, qw, dtype=torch.bfloat16)
    torch.cuda.synchronize()
    _assert_gemm_close(outb, ref, absdot, "native fp6 bf16", bf16=True)


def test_dfp4_gemm_native_all_dialects_wide_exponents_and_full_size_sample():
    # every dialect and every index occurs; block exponents spread over tens of binades
    g = torch.Generator().manual_seed(18)
    scale = torch.exp2(torch.randint(-40, 40, (128, 16), generator=g).repeat_interleave(32, dim=1).float())
    a = (torch.randn(128, 512, generator=g) * scale).to(torch.bfloat16)
    w = (torch.randn(160, 512, generator=g) * scale[:1]).to(torch.bfloat16)
    qa, qw = dfp4.quantize(_dev(a)), dfp4.quantize_mse(_dev(w))
    assert len(torch.unique(qa.dialect)) == 16
    out = dfp4.gemm_native(qa, qw)
    torch.cuda.synchronize()
    ad = O.dfp4_dequantize(*O.dfp4_quantize(synth.to_f64(a)))
    wd = O.dfp4_dequantize(*O.dfp4_quantize_mse(synth.to_f64(w)))
    _assert_gemm_close(out, ad @ wd.T, np.abs(ad) @ np.abs(wd).T, "native fp6 wide")
    ops = synth.llama3_8b_mlp(seed=2)
    x, wg = ops["x"], ops["w_gate"]
    out = dfp4.gemm_native(dfp4.quantize(_dev(x)), dfp4.quantize(_dev(wg)))
    torch.cuda.synchronize()
    rng = np.random.default_rng(19)
    rows = np.sort(rng.choice(x.shape[0], 16, replace=False))
    cols = np.sort(rng.choice(wg.shape[0], 128, replace=False))
    ref, absdot = _gemm_ref(synth.to_f64(x[rows]), synth.to_f64(wg[cols]))
    _assert_gemm_close(out[rows][:, cols], ref, absdot, "native fp6 full size sampled")


def test_gemm_native_with_prepacked_weights():
    # weights arranged once in the instruction's register order; results identical to the call
    # that packs both operands
    M, N, K = 300, 520, 1056
    a = synth.gaussian_outlier_channels(M, K, 8, 50.0, 1.0, seed=901)
    w = synth.gaussian(N, K, 0.02, seed=902)
    qa, qw = dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w))
    wp = dfp4.native_pack(qw)
    out = dfp4.gemm_native_packed_w(qa, wp)
    both = dfp4.gemm_native(qa, qw)
    both_packed = dfp4.gemm_native_packed(dfp4.native_pack(qa), wp)
    torch.cuda.synchronize()
    assert torch.equal(out, both) and torch.equal(both_packed, both)
    ref, absdot = _gemm_ref(synth.to_f64(a), synth.to_f64(w))
    _assert_gemm_close(out, ref, absdot, "prepacked fp6")
    qam, qwm = dfp4.mxfp4_quantize(_dev(a)), dfp4.mxfp4_quantize(_dev(w))
    outm = dfp4.gemm_native_packed_w(qam, dfp4.native_pack(qwm, mx=True), dtype=torch.bfloat16)
    torch.cuda.synchronize()
    refm, absm = _gemm_ref(synth.to_f64(a), synth.to_f64(w), mx=True)
    _assert_gemm_close(outm, refm, absm, "prepacked fp4 bf16", bf16=True)


def test_gemm_random_edge_shapes_all_paths():
    # seeded sweep over awkward shapes (sizes around the tile boundaries, odd block counts) and three
    # input recipes; every GEMM path against the oracle, the requantizing one against its composition
    rng = np.random.default_rng(2024)
    for it in range(14):
        M = int(rng.choice([1, 31, 33, 65, 127, 129, 257, 300, 513, 700]))
        N = int(rng.choice([1, 7, 33, 96, 130, 256, 257, 520]))
        KB = int(rng.choice([1, 3, 8, 15, 17, 33, 65]))
        K, kind = KB * 32, int(rng.integers(0, 3))
        print(f"gemm sweep {it}: {M}x{N}x{K} recipe {kind}", flush=True)
        g = torch.Generator().manual_seed(int(rng.integers(1 << 30)))
        a = torch.randn(M, K, generator=g)
        if kind == 1:
            a[:, rng.integers(0, K, max(1, K // 100))] *= 50
        if kind == 2:
            a = a * torch.exp2(torch.randint(-12, 12, (M, KB), generator=g).repeat_interleave(32, dim=1).float())
        a = a.to(torch.bfloat16)
        w = (torch.randn(N, K, generator=g) * 0.02).to(torch.bfloat16)
        ref, absdot = _gemm_ref(synth.to_f64(a), synth.to_f64(w))
        qa, qw = dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w))
        _assert_gemm_close(dfp4.gemm(qa, qw), ref, absdot, f"int8 path {M}x{N}x{K}")
        _assert_gemm_close(dfp4.gemm_native(qa, qw), ref, absdot, f"native path {M}x{N}x{K}")
        if N % 32 == 0:
            rq = dfp4.gemm_requant(qa, qw)
            want = dfp4.quantize(dfp4.gemm(qa, qw, dtype=torch.bfloat16))
            torch.cuda.synchronize()
            assert torch.equal(rq.codes, want.codes) and torch.equal(rq.dialect, want.dialect)
            assert torch.equal(rq.exponent, want.exponent)
        refm, absm = _gemm_ref(synth.to_f64(a), synth.to_f64(w), mx=True)
        qam, qwm = dfp4.mxfp4_quantize(_dev(a)), dfp4.mxfp4_quantize(_dev(w))
        _assert_gemm_close(dfp4.mxfp4_gemm(qam, qwm), refm, absm, f"mx int8 path {M}x{N}x{K}")
        _assert_gemm_close(dfp4.mxfp4_gemm_native(qam, qwm), refm, absm, f"mx native path {M}x{N}x{K}")


@pytest.mark.parametrize("rows,K", [(1, 32), (70, 160), (300, 1056), (513, 4096), (64, 14336)])
def test_quantize_native_equals_quantize_then_pack(rows, K):
    # the quantizer that writes the matrix instruction's FP6 operand directly: byte-identical to
    # dfp4_quantize + dfp4_native_pack (both buffers start as zeros: the fused kernel leaves the
    # layout's padding rows untouched), also from a strided input
    print(f"quantize_native parity: {rows}x{K}", flush=True)
    x = synth.gaussian_outlier_channels(rows, K, max(1, K // 100), 50.0, 1.0, seed=rows + K).cuda()
    n = int(dfp4.load().dfp4_native_packed_bytes(rows, K))
    want = dfp4.native_pack(dfp4.quantize(x), buf=torch.zeros(n, dtype=torch.uint8, device="cuda"))
    got = dfp4.quantize_native(x)
    torch.cuda.synchronize()
    assert torch.equal(got.buf, want.buf), int((got.buf != want.buf).sum())
    wide = torch.zeros(rows, K + 64, dtype=torch.bfloat16, device="cuda")
    wide[:, 32:32 + K] = x
    got2 = dfp4.quantize_native(wide[:, 32:32 + K])
    torch.cuda.synchronize()
    assert torch.equal(got2.buf, want.buf)
    # and it multiplies to the oracle's product
    w = synth.gaussian(96, K, 0.02, seed=K)
    out = dfp4.gemm_native_packed(got, dfp4.native_pack(dfp4.quantize(_dev(w))))
    torch.cuda.synchronize()
    ref, absdot = _gemm_ref(synth.to_f64(x.cpu()), synth.to_f64(w))
    _assert_gemm_close(out, ref, absdot, "quantize_native product")


# --------------------------------------------------------------------------
# value cache with a high-precision residual chunk (Appendix C)
# --------------------------------------------------------------------------
def test_value_cache_appends_match_quantizing_the_transpose():
    from paper_2501_01144_amd.kvcache import ValueCache
    D, cap = 64, 256
    v = synth.gaussian_outlier_channels(200, D, 2, 30.0, 1.0, seed=41)
    cache = ValueCache(D, cap, "cuda")
    pos = 0
    for step in (1, 5, 26, 1, 64, 31, 40, 32):          # odd sizes: chunks complete at different points
        cache.append(v[pos:pos + step].cuda())
        pos += step
        torch.cuda.synchronize()
        assert cache.n_tokens == pos and cache.n_quantized == pos // 32 * 32
        nq = cache.n_quantized
        if nq:
            codes, dialect, expo = O.dfp4_quantize(synth.to_f64(v[:nq]).T.copy())
            assert np.array_equal(_np(cache.q.codes)[:, :nq // 2], codes)
            assert np.array_equal(_np(cache.q.dialect)[:, :nq // 32], dialect)
            assert np.array_equal(_np(cache.q.exponent)[:, :nq // 32], expo)
        assert not _np(cache.q.codes)[:, nq // 2:].any()                      # later blocks untouched
        assert torch.equal(cache.residual_values().cpu(), v[nq:pos])
    # P V over the whole capacity with zero-padded probabilities = product over the quantized tokens
    nq = cache.n_quantized
    p = torch.zeros(4, cap, dtype=torch.bfloat16)
    p[:, :nq] = synth.softmax_rows(4, nq, seed=42)
    out = dfp4.gemm(dfp4.quantize(_dev(p)), cache.q)
    torch.cuda.synchronize()
    ref, absdot = _gemm_ref(synth.to_f64(p[:, :nq]), synth.to_f64(v[:nq]).T.copy())
    _assert_gemm_close(out, ref, absdot, "P V through the cache")


# --------------------------------------------------------------------------
# blocks of 64
# --------------------------------------------------------------------------
@pytest.mark.parametrize("rows,K", [(1, 64), (7, 192), (33, 4096), (257, 1088)])
def test_quantize_block64(rows, K):
    print(f"quantize_b64 parity: {rows}x{K}", flush=True)
    for x in (synth.student_t(rows, K, 3.0, seed=rows + K),
              synth.gaussian_outlier_channels(rows, K, max(1, K // 100), 50.0, 1.0, seed=rows)):
        q = dfp4.quantize_b64(_dev(x))
        torch.cuda.synchronize()
        _assert_quant_equal(q, O.dfp4_quantize_block64(synth.to_f64(x)), "block 64")
    # strided input, and the result multiplies like any other quantized tensor
    wide = torch.zeros(rows, K + 64, dtype=torch.bfloat16, device="cuda")
    wide[:, 32:32 + K] = x.cuda()
    q2 = dfp4.quantize_b64(wide[:, 32:32 + K])
    torch.cuda.synchronize()
    _assert_quant_equal(q2, O.dfp4_quantize_block64(synth.to_f64(x)), "block 64 strided")
    w = synth.gaussian(40, K, 0.02, seed=K)
    out = dfp4.gemm(q, dfp4.quantize_b64(_dev(w)))
    torch.cuda.synchronize()
    ad = O.dfp4_dequantize(*O.dfp4_quantize_block64(synth.to_f64(x)))
    wd = O.dfp4_dequantize(*O.dfp4_quantize_block64(synth.to_f64(w)))
    _assert_gemm_close(out, ad @ wd.T, np.abs(ad) @ np.abs(wd).T, "block 64 product")


@pytest.mark.parametrize("M,N,K", [(5, 40, 64), (16, 4096, 4096), (33, 100, 1056), (64, 96, 256)])
def test_gemm_native_few_rows(M, N, K):
    # decode shapes on the block-scaled instruction: 32 W rows per workgroup, 16 waves share K
    print(f"native few rows parity: {M}x{N}x{K}", flush=True)
    a = synth.gaussian_outlier_channels(M, K, max(1, K // 200), 50.0, 1.0, seed=110 + M)
    w = synth.gaussian(N, K, 0.02, seed=210 + N)
    ref, absdot = _gemm_ref(synth.to_f64(a), synth.to_f64(w))
    wp = dfp4.native_pack(dfp4.quantize(_dev(w)))
    out = dfp4.gemm_native_packed(dfp4.quantize_native(_dev(a)), wp)
    torch.cuda.synchronize()
    _assert_gemm_close(out, ref, absdot, "native few rows f32")
    outb = dfp4.gemm_native(dfp4.quantize(_dev(a)), dfp4.quantize(_dev(w)), dtype=torch.bfloat16)
    torch.cuda.synchronize()
    _assert_gemm_close(outb, ref, absdot, "native few rows bf16", bf16=True)
    refm, absm = _gemm_ref(synth.to_f64(a), synth.to_f64(w), mx=True)
    outm = dfp4.mxfp4_gemm_native(dfp4.mxfp4_quantize(_dev(a)), dfp4.mxfp4_quantize(_dev(w)))
    torch.cuda.synchronize()
    _assert_gemm_close(outm, refm, absm, "native few rows mxfp4")


# --------------------------------------------------------------------------
# blocks of 16 and mixed block sizes (Section 4.2, Table 3)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("rows,K", [(1, 32), (7, 96), (33, 4096), (257, 1056), (2048, 4096)])
def test_quantize_and_dequantize_block16(rows, K):
    print(f"quantize parity: blocks of 16, {rows}x{K}", flush=True)
    x = torch.cat([synth.student_t(rows, K, 3.0, seed=60 + rows)[: rows - rows // 2],
                   synth.gaussian_outlier_channels(rows // 2, K, max(1, K // 100), 50.0, 1.0, seed=61 + rows)])
    q = dfp4.quantize_block(_dev(x), 16)
    torch.cuda.synchronize()
    assert q.dialect.shape == (rows, K // 16) and q.exponent.shape == (rows, K // 16)
    ref = O.dfp4_quantize_block16(synth.to_f64(x))
    _assert_quant_equal(q, ref, "block16")
    for dtype in (torch.float32, torch.bfloat16):
        back = dfp4.dequantize_block(q, 16, dtype=dtype)
        torch.cuda.synchronize()
        assert np.array_equal(back.cpu().double().numpy(), O.dfp4_dequantize_block(*ref, 16))
    # block sizes 32 and 64 through the same entry point
    _assert_quant_equal(dfp4.quantize_block(_dev(x), 32), O.dfp4_quantize(synth.to_f64(x)), "block32 via quantize_block")
    if K % 64 == 0:
        _assert_quant_equal(dfp4.quantize_block(_dev(x), 64), O.dfp4_quantize_block64(synth.to_f64(x)), "block64")


def test_quantize_block16_every_bf16_value_and_strided_rows():
    vals = synth.all_bf16_bit_patterns()                     # [2040, 32]: two blocks of 16 per row
    q = dfp4.quantize_block(_dev(vals), 16)
    torch.cuda.synchronize()
    _assert_quant_equal(q, O.dfp4_quantize_block16(synth.to_f64(vals)), "every bf16 value, blocks of 16")
    base = synth.gaussian_outlier_channels(70, 1024, 4, 30.0, 1.0, seed=67)
    qs = dfp4.quantize_block(_dev(base)[:, 128:128 + 512], 16)
    torch.cuda.synchronize()
    _assert_quant_equal(qs, O.dfp4_quantize_block16(synth.to_f64(base[:, 128:128 + 512].contiguous())), "strided, blocks of 16")


@pytest.mark.parametrize("M,N,K,ba,bw", [(70, 200, 160, 16, 16), (129, 257, 1024, 16, 32), (300, 130, 512, 32, 16),
                                         (64, 96, 256, 16, 64), (512, 256, 4096, 16, 16), (100, 100, 256, 64, 32)])
def test_gemm_mixed_block_sizes(M, N, K, ba, bw):
    print(f"gemm parity: blocks {ba} x {bw}, {M}x{N}x{K}", flush=True)
    a = synth.gaussian_outlier_channels(M, K, max(1, K // 100), 50.0, 1.0, seed=70 + M)
    w = synth.gaussian(N, K, 0.02, seed=71 + N)
    qa, qw = dfp4.quantize_block(_dev(a), ba), dfp4.quantize_block(_dev(w), bw)
    def oracle_q(x, b):
        x = synth.to_f64(x)
        return (O.dfp4_quantize_block16(x), 16) if b == 16 else ((O.dfp4_quantize_block64(x) if b == 64 else O.dfp4_quantize(x)), 32)
    (ra, la), (rw, lw) = oracle_q(a, ba), oracle_q(w, bw)
    ad, wd = O.dfp4_dequantize_block(*ra, la), O.dfp4_dequantize_block(*rw, lw)
    ref, absdot = O.dfp4_gemm_blocks(ra, la, rw, lw), np.abs(ad) @ np.abs(wd).T
    for dtype in (torch.float32, torch.bfloat16):
        out = dfp4.gemm_blocks(qa, ba, qw, bw, dtype=dtype)
        torch.cuda.synchronize()
        _assert_gemm_close(out, ref, absdot, f"blocks {ba}x{bw} {dtype}", bf16=dtype == torch.bfloat16)
