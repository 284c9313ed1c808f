"""MXFP4 comparison format (Section 4.1 "Baseline"; Appendix I) in float64 NumPy.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Blocks of 32 along K share
a power-of-two exponent e = floor(log2(block max)) - 2 (the same scaling the
paper uses when it compares block distributions with FP4 E2M1, Section 3.1);
each element is an FP4 E2M1 code: 1 sign bit + 3 bits indexing
{0, 0.5, 1, 1.5, 2, 3, 4, 6}.  The paper names the format only; the rounding
used here is the reading "round to nearest, ties to the even code, magnitudes
above 6 saturate to 6".  Layouts match the DialectFP4 oracle, without the
dialect array.
"""
import numpy as np

from .dfp4_oracle import BLOCK, EXP_BIAS, shared_exponent, pack_codes, unpack_codes

E2M1 = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])


def e2m1_index(s):
    """Nearest E2M1 magnitude; on a tie the even index; s >= 6 gives index 7."""
    dist = np.abs(s[..., None] - E2M1)
    best = dist.min(axis=-1, keepdims=True)
    is_best = dist == best
    even = (np.arange(8) % 2 == 0)
    # among the (one or two) nearest values prefer the even index
    prefer = is_best & even
    pick = np.where(prefer.any(axis=-1, keepdims=True), prefer, is_best)
    return np.argmax(pick, axis=-1)


def mxfp4_quantize(x):
    x = np.asarray(x, dtype=np.float64)
    assert x.ndim == 2 and x.shape[1] % BLOCK == 0
    assert np.isfinite(x).all()
    rows, K = x.shape
    xb = x.reshape(-1, BLOCK)
    mag = np.abs(xb)
    e = shared_exponent(mag.max(axis=1))
    s = np.ldexp(mag, (-e)[:, None].astype(np.int32))
    index = e2m1_index(s)
    codes = pack_codes(np.signbit(xb), index).reshape(rows, K // 2)
    return codes, (e + EXP_BIAS).astype(np.uint8).reshape(rows, K // BLOCK)


def mxfp4_dequantize(codes, exponent):
    rows = codes.shape[0]
    nib = unpack_codes(codes).reshape(rows, -1, BLOCK)
    mag = np.ldexp(E2M1[(nib & 7).astype(np.int64)],
                   (exponent.astype(np.int32) - EXP_BIAS)[:, :, None])
    return np.where((nib >> 3) == 1, -mag, mag).reshape(rows, -1)


def mxfp4_gemm(a_q, w_q):
    """out = A^ @ W^T over the dequantized operands, float64."""
    return mxfp4_dequantize(*a_q) @ mxfp4_dequantize(*w_q).T


def effective_bits(block, exponent_bits=5):
    """Appendix I: 4 element bits + one shared exponent per block."""
    return 4.0 + exponent_bits / block
