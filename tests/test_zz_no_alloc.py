"""dfp4_gemm_noalloc (the entry point that allocates nothing) against dfp4_gemm, through the C ABI:
same kernels on the library's own scratch array, so the outputs must be bit-identical; two calls in
a row, the second on a smaller input, so that stale scratch contents would show."""
import numpy as np
import pytest
import torch

from oracle import dfp4_oracle as O
from paper_2501_01144_amd import dfp4, synth

pytestmark = pytest.mark.gpu


def _case(M, N, K, seed):
    a = synth.gaussian_outlier_channels(M, K, max(1, K // 200), 50.0, 1.0, seed)
    w = synth.gaussian(N, K, 0.02, seed + 1)
    return a, w


def test_gemm_noalloc_matches_gemm_on_two_calls_in_a_row():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    dfp4.load()
    dev = torch.device("cuda:0")
    first = True
    for (M, N, K, dtype) in [(1100, 700, 2048, torch.float32), (300, 260, 512, torch.bfloat16)]:
        a, w = _case(M, N, K, 11 + M)
        qa, qw = dfp4.quantize(a.to(dev)), dfp4.quantize(w.to(dev))
        assert 0 < dfp4.gemm_workspace_bytes(M, N, K) <= dfp4.NOALLOC_SCRATCH_BYTES
        want = dfp4.gemm(qa, qw, dtype=dtype)
        got = torch.full((M, N), float("nan"), dtype=dtype, device=dev)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        dfp4.gemm_noalloc(qa, qw, got)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(got.view(torch.int32 if dtype == torch.float32 else torch.int16),
                           want.view(torch.int32 if dtype == torch.float32 else torch.int16)), (M, N, K)
        if first:
            # and against the oracle, to the GEMM's parity bar
            ad = O.dfp4_dequantize(*O.dfp4_quantize(synth.to_f64(a)))
            wd = O.dfp4_dequantize(*O.dfp4_quantize(synth.to_f64(w)))
            ref, absdot = ad @ wd.T, np.abs(ad) @ np.abs(wd).T
            assert (np.abs(got.cpu().double().numpy() - ref) <= 1e-5 * absdot).all()
            first = False


def test_gemm_noalloc_refuses_what_does_not_fit():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    lib = dfp4.load()
    M, N, K = 2048, 4096, 14336
    assert dfp4.gemm_workspace_bytes(M, N, K) > dfp4.NOALLOC_SCRATCH_BYTES
    dev = torch.device("cuda:0")
    qa, qw = dfp4.empty_qtensor(M, K, dev), dfp4.empty_qtensor(N, K, dev)
    out = torch.empty((M, N), dtype=torch.float32, device=dev)
    with pytest.raises(dfp4.Dfp4Error, match="workspace"):
        dfp4.gemm_noalloc(qa, qw, out)
    assert lib.dfp4_gemm_noalloc(qa.c(), qw.c(), out.data_ptr(), 0, N, None) == -5
