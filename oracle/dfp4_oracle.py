"""DialectFP4 oracle: quantize, dequantize, block-scaled matmul (float64 NumPy).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Every function follows the
paper's steps in the paper's order, on real numbers held exactly in float64:
inputs are bf16 values, every intermediate is a bf16 value times a power of
two, and every comparison is against a multiple of 0.25.

Arrays exchanged with callers (layouts are this build's choice, the paper
fixes none of them):
  codes     uint8 [rows, K/2]   element 2j in bits 3:0 of byte j, 2j+1 in bits 7:4;
                                a 4-bit code is (sign << 3) | index
  dialect   uint8 [rows, K/32]  dialect identifier 0..15
  exponent  uint8 [rows, K/32]  shared exponent e stored as e + 127
"""
import numpy as np

BLOCK = 32
EXP_BIAS = 127

# Section 3.1, "16-Dialect DialectFP4 Example": 16 dialects in 8 pairs, unit
# 0.5, each pair shares its largest magnitude and differs in one large value,
# the small values follow FP4 E2M1.  Stored as half-units (value = 0.5 * u),
# ascending, position = 3-bit index.  Rows 4 and 5 are printed in Sections
# 3.2/3.3; the other rows are a reconstruction (parity unpinned, see package
# docstring).  Pair p (dialects 2p, 2p+1) has largest magnitude 7.5 - 0.5 p;
# the even dialect holds the larger differing value (Appendix B).
FORMATBOOK_HALF_UNITS = np.array([
    [0, 1, 2, 3, 4, 6, 12, 15],   # d0   max 7.5
    [0, 1, 2, 3, 4, 6, 10, 15],   # d1
    [0, 1, 2, 3, 4, 6, 11, 14],   # d2   max 7.0
    [0, 1, 2, 3, 4, 6,  9, 14],   # d3
    [0, 1, 2, 3, 4, 6, 10, 13],   # d4   max 6.5  (Section 3.3 worked example)
    [0, 1, 2, 3, 4, 6,  8, 13],   # d5            (Section 3.2: 4.0 instead of 5.0)
    [0, 1, 2, 3, 4, 6,  9, 12],   # d6   max 6.0
    [0, 1, 2, 3, 4, 6,  8, 12],   # d7            = FP4 E2M1
    [0, 1, 2, 3, 4, 6,  9, 11],   # d8   max 5.5
    [0, 1, 2, 3, 4, 6,  8, 11],   # d9
    [0, 1, 2, 3, 4, 6,  8, 10],   # d10  max 5.0
    [0, 1, 2, 3, 4, 6,  7, 10],   # d11
    [0, 1, 2, 3, 4, 6,  8,  9],   # d12  max 4.5
    [0, 1, 2, 3, 4, 6,  7,  9],   # d13
    [0, 1, 2, 3, 4, 6,  7,  8],   # d14  max 4.0
    [0, 1, 2, 3, 4, 5,  6,  8],   # d15
], dtype=np.int64)

# representable magnitudes as real numbers, [16, 8]
FORMATBOOK = FORMATBOOK_HALF_UNITS.astype(np.float64) * 0.5


def shared_exponent(amax):
    """Section 3.1 / 3.2 preprocessing: e = floor(log2(block max)) - 2, so that
    the scaled block lies in [0, 8) with its maximum in [4, 8).

    With bf16 inputs the exponent needs 8 bits (the paper's 5 bits are for
    FP16): e is clamped to [-127, 127].  An all-zero block has no logarithm;
    it takes the smallest exponent, e = -127.
    """
    amax = np.asarray(amax, dtype=np.float64)
    _, ex = np.frexp(amax)                  # amax = m * 2**ex, m in [0.5, 1)
    e = ex.astype(np.int64) - 1 - 2         # floor(log2 amax) - 2, exact
    e = np.where(amax == 0.0, -EXP_BIAS, e)
    return np.clip(e, -EXP_BIAS, EXP_BIAS)


def beneficial_range(dialect):
    """Section 3.2, second stage: the interval in which the value that this
    dialect does not share with its pair partner is the nearest value among
    all values of the pair.  Half-open [lower midpoint, upper midpoint); for
    dialect 4 this is [4.5, 5.75) as printed in the paper.
    """
    mine = FORMATBOOK[dialect]
    other = FORMATBOOK[dialect ^ 1]
    differing = [v for v in mine if v not in other]
    assert len(differing) == 1
    v = differing[0]
    union = sorted(set(mine) | set(other))
    i = union.index(v)
    return (union[i - 1] + v) / 2.0, (v + union[i + 1]) / 2.0


def select_dialect(s):
    """Two-stage dialect selection (Section 3.2) for scaled magnitudes
    s [nblocks, 32] (each block already divided by 2**e).  Returns ids [nblocks].

    Stage 1: round the block maximum to a multiple of 0.5 (half up, as the
    paper rounds from the second fractional bit) and take the pair of
    dialects whose largest magnitude equals it.  A rounded maximum of 8.0
    has no pair and is taken as 7.5; a maximum below 4.0 can only occur when
    the exponent was clamped and is taken as 4.0.
    Stage 2: count the block's elements inside each dialect's beneficial
    range; the larger count wins, the even dialect wins ties.
    """
    smax = s.max(axis=1)
    rounded = np.floor(2.0 * smax + 0.5) / 2.0
    rounded = np.clip(rounded, 4.0, 7.5)
    pair = np.rint((7.5 - rounded) * 2.0).astype(np.int64)
    dialect = np.empty(s.shape[0], dtype=np.int64)
    for p in range(8):
        rows = np.nonzero(pair == p)[0]
        if rows.size == 0:
            continue
        lo_e, hi_e = beneficial_range(2 * p)
        lo_o, hi_o = beneficial_range(2 * p + 1)
        sp = s[rows]
        count_even = ((sp >= lo_e) & (sp < hi_e)).sum(axis=1)
        count_odd = ((sp >= lo_o) & (sp < hi_o)).sum(axis=1)
        dialect[rows] = 2 * p + (count_odd > count_even)
    return dialect


def nearest_index(s, dialect):
    """Section 3.3: each scaled magnitude goes to the nearest representable
    value of the block's dialect; a magnitude exactly halfway goes to the
    larger value (the paper's interval for 5.0 in dialect 4 is [4.0, 5.75)).
    s [nblocks, 32], dialect [nblocks] -> index [nblocks, 32] in 0..7.
    """
    vals = FORMATBOOK[dialect]                               # [nb, 8]
    dist = np.abs(s[:, :, None] - vals[:, None, :])          # [nb, 32, 8]
    # first minimum of the reversed axis = largest value among equal distances
    return 7 - np.argmin(dist[:, :, ::-1], axis=2)


def pack_codes(sign, index):
    """4-bit code = 1 sign bit + 3-bit index (Section 3.1); two per byte."""
    nib = ((sign.astype(np.uint8) << 3) | index.astype(np.uint8))
    nib = nib.reshape(nib.shape[0], -1)
    return (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)


def unpack_codes(codes):
    nib = np.empty((codes.shape[0], codes.shape[1] * 2), dtype=np.uint8)
    nib[:, 0::2] = codes & 0xF
    nib[:, 1::2] = codes >> 4
    return nib


def dfp4_quantize(x, chunk_blocks=1 << 15):
    """Online DialectFP4 quantization of x [rows, K] (K % 32 == 0) in blocks of
    32 along K.  x holds bf16 values (any float dtype that represents them
    exactly); non-finite inputs are outside the method.
    Returns (codes, dialect, exponent) as described in the module docstring.
    """
    x = np.asarray(x, dtype=np.float64)
    assert x.ndim == 2 and x.shape[1] % BLOCK == 0
    assert np.isfinite(x).all()
    rows, K = x.shape
    nb = rows * (K // BLOCK)
    xb = x.reshape(nb, BLOCK)
    index = np.empty((nb, BLOCK), dtype=np.uint8)
    dialect = np.empty(nb, dtype=np.uint8)
    exponent = np.empty(nb, dtype=np.uint8)
    for b0 in range(0, nb, chunk_blocks):
        blk = xb[b0:b0 + chunk_blocks]
        mag = np.abs(blk)
        e = shared_exponent(mag.max(axis=1))                 # preprocessing
        s = np.ldexp(mag, (-e)[:, None].astype(np.int32))    # exact scaling
        d = select_dialect(s)                                # two stages
        index[b0:b0 + chunk_blocks] = nearest_index(s, d)    # element rounding
        dialect[b0:b0 + chunk_blocks] = d
        exponent[b0:b0 + chunk_blocks] = e + EXP_BIAS
    sign = np.signbit(xb)                                    # -0.0 keeps its sign bit
    codes = pack_codes(sign, index).reshape(rows, K // 2)
    return codes, dialect.reshape(rows, K // BLOCK), exponent.reshape(rows, K // BLOCK)


def dfp4_quantize_block64(x, chunk_blocks=1 << 14):
    """DialectFP4 with blocks of 64 (Section 4.2, Table 3 varies the block size): the same steps
    on 64 consecutive elements -- one shared exponent, one dialect chosen from the votes
    of all 64.  Returned in the layout of the 32-element format: each block's exponent
    byte and dialect id appear twice (once per 32 elements), so that every consumer of
    the 32-element layout reads it unchanged."""
    x = np.asarray(x, dtype=np.float64)
    assert x.ndim == 2 and x.shape[1] % 64 == 0
    assert np.isfinite(x).all()
    rows, K = x.shape
    nb = rows * (K // 64)
    xb = x.reshape(nb, 64)
    index = np.empty((nb, 64), dtype=np.uint8)
    dialect = np.empty(nb, dtype=np.uint8)
    exponent = np.empty(nb, dtype=np.uint8)
    for b0 in range(0, nb, chunk_blocks):
        mag = np.abs(xb[b0:b0 + chunk_blocks])
        e = shared_exponent(mag.max(axis=1))
        s = np.ldexp(mag, (-e)[:, None].astype(np.int32))
        d = select_dialect(s)
        index[b0:b0 + chunk_blocks] = nearest_index(s, d)
        dialect[b0:b0 + chunk_blocks] = d
        exponent[b0:b0 + chunk_blocks] = e + EXP_BIAS
    codes = pack_codes(np.signbit(xb), index).reshape(rows, K // 2)
    return (codes, np.repeat(dialect.reshape(rows, K // 64), 2, axis=1),
            np.repeat(exponent.reshape(rows, K // 64), 2, axis=1))


def dfp4_quantize_block16(x, chunk_blocks=1 << 15):
    """DialectFP4 with blocks of 16 (Section 4.2, Table 3 varies the block size; smaller blocks
    for the sublayers most sensitive to quantization): the same steps on 16 consecutive elements.
    Returned with one exponent byte and one dialect id per 16 elements:
    codes [rows, K/2], dialect [rows, K/16], exponent [rows, K/16]."""
    x = np.asarray(x, dtype=np.float64)
    assert x.ndim == 2 and x.shape[1] % 16 == 0
    assert np.isfinite(x).all()
    rows, K = x.shape
    nb = rows * (K // 16)
    xb = x.reshape(nb, 16)
    index = np.empty((nb, 16), dtype=np.uint8)
    dialect = np.empty(nb, dtype=np.uint8)
    exponent = np.empty(nb, dtype=np.uint8)
    for b0 in range(0, nb, chunk_blocks):
        mag = np.abs(xb[b0:b0 + chunk_blocks])
        e = shared_exponent(mag.max(axis=1))
        s = np.ldexp(mag, (-e)[:, None].astype(np.int32))
        d = select_dialect(s)
        index[b0:b0 + chunk_blocks] = nearest_index(s, d)
        dialect[b0:b0 + chunk_blocks] = d
        exponent[b0:b0 + chunk_blocks] = e + EXP_BIAS
    codes = pack_codes(np.signbit(xb), index).reshape(rows, K // 2)
    return codes, dialect.reshape(rows, K // 16), exponent.reshape(rows, K // 16)


def dfp4_dequantize_block(codes, dialect, exponent, block):
    """Section 3.3 dequantization for a tensor whose dialect / exponent arrays hold one entry per
    `block` elements (16 or 32; blocks of 64 are stored in the 32-element layout)."""
    assert block in (16, 32)
    rows = codes.shape[0]
    nib = unpack_codes(codes).reshape(rows, -1, block)
    u = np.take_along_axis(FORMATBOOK_HALF_UNITS[dialect.astype(np.int64)],
                           (nib & 7).astype(np.int64), axis=2)
    mag = np.ldexp(0.5 * u.astype(np.float64),
                   (exponent.astype(np.int32) - EXP_BIAS)[:, :, None])
    return np.where((nib >> 3) == 1, -mag, mag).reshape(rows, -1)


def dfp4_gemm_blocks(a_q, block_a, w_q, block_w):
    """The block MAC of Section 3.3 for operands quantized with different block sizes (per-sublayer
    block-size mixes of Table 3): the sum over K of the dequantized values, in float64."""
    return dfp4_dequantize_block(*a_q, block_a) @ dfp4_dequantize_block(*w_q, block_w).T


def select_dialect_mse(s):
    """Dialect with the smallest squared error (Section 3.2: for weights, known in
    advance, the best dialect of a block can be found by computing the exact mean
    squared error of every dialect).  s [nblocks, 32] scaled magnitudes; returns ids.

    Every dialect rounds a magnitude below 0.25 to 0, so those elements add the same
    amount to all 16 errors and are left out of the comparison; the remaining terms
    (s - v)^2 are multiples of 2^-18 below 2^6, and their sums are exact in float64.
    Equal errors: the lowest dialect id (the paper does not say).
    """
    big = s >= 0.25
    err = np.empty((s.shape[0], 16), dtype=np.float64)
    for d in range(16):
        idx = nearest_index(s, np.full(s.shape[0], d, dtype=np.int64))
        v = np.take_along_axis(np.broadcast_to(FORMATBOOK[d], (s.shape[0], 8)), idx, axis=1)
        err[:, d] = (np.where(big, s - v, 0.0) ** 2).sum(axis=1)
    return np.argmin(err, axis=1)          # first minimum = lowest id


def dfp4_quantize_mse(x, chunk_blocks=1 << 13):
    """DialectFP4 quantization with MSE-based dialect selection (offline, for
    weights): same shared exponent, element rounding and layouts as dfp4_quantize;
    only the choice of the block's dialect differs."""
    x = np.asarray(x, dtype=np.float64)
    assert x.ndim == 2 and x.shape[1] % BLOCK == 0
    assert np.isfinite(x).all()
    rows, K = x.shape
    nb = rows * (K // BLOCK)
    xb = x.reshape(nb, BLOCK)
    index = np.empty((nb, BLOCK), dtype=np.uint8)
    dialect = np.empty(nb, dtype=np.uint8)
    exponent = np.empty(nb, dtype=np.uint8)
    for b0 in range(0, nb, chunk_blocks):
        blk = xb[b0:b0 + chunk_blocks]
        mag = np.abs(blk)
        e = shared_exponent(mag.max(axis=1))
        s = np.ldexp(mag, (-e)[:, None].astype(np.int32))
        d = select_dialect_mse(s)
        index[b0:b0 + chunk_blocks] = nearest_index(s, d)
        dialect[b0:b0 + chunk_blocks] = d
        exponent[b0:b0 + chunk_blocks] = e + EXP_BIAS
    sign = np.signbit(xb)
    codes = pack_codes(sign, index).reshape(rows, K // 2)
    return codes, dialect.reshape(rows, K // BLOCK), exponent.reshape(rows, K // BLOCK)


def dfp4_dequantize(codes, dialect, exponent):
    """Section 3.3 dequantization: index -> 4-bit unsigned integer u through the
    dialect's table, value = (-1)**sign * 0.5 * u * 2**e.  Returns float64 [rows, K]."""
    rows = codes.shape[0]
    nib = unpack_codes(codes).reshape(rows, -1, BLOCK)
    u = np.take_along_axis(FORMATBOOK_HALF_UNITS[dialect.astype(np.int64)],
                           (nib & 7).astype(np.int64), axis=2)
    mag = np.ldexp(0.5 * u.astype(np.float64),
                   (exponent.astype(np.int32) - EXP_BIAS)[:, :, None])
    out = np.where((nib >> 3) == 1, -mag, mag)
    return out.reshape(rows, -1)


def dfp4_gemm(a_q, w_q):
    """Section 3.3 block MAC: out[m, n] = sum over K of A^[m, k] * W^[n, k] with
    A^, W^ the dequantized operands (both blocked along K).  This equals the
    paper's per-block integer sums scaled by 2**(ea + ew - 2); accumulated in
    float64, where every term is an integer times a power of two.
    a_q, w_q are (codes, dialect, exponent) triples.  Returns float64 [M, N]."""
    a = dfp4_dequantize(*a_q)
    w = dfp4_dequantize(*w_q)
    assert a.shape[1] == w.shape[1]
    return a @ w.T


def round_to_bf16(x):
    """Round float64 values to float32 and then to bf16, both to nearest even (the
    precision chain of a bf16 result computed from an exact sum); returns float64."""
    u = np.asarray(x, dtype=np.float64).astype(np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def dfp4_gemm_requant(a_q, w_q):
    """Section 3.3: the result of a multiplication that feeds another one is quantized
    again.  out = quantize(bf16(A W^T)), blocks of 32 along N."""
    return dfp4_quantize(round_to_bf16(dfp4_gemm(a_q, w_q)))


def effective_bits(block, exponent_bits=5, dialect_bits=4):
    """Appendix I: element bits plus per-block overhead spread over the block."""
    return 4.0 + (exponent_bits + dialect_bits) / block
