"""ctypes binding of libdfp4.so: the same calls as include/dfp4.h, taking torch
tensors for device memory and the current torch stream.  Argument marshalling
only: every step of the path runs in the HIP kernels.  There is no fallback;
if the library is missing or a call fails, an exception is raised.
"""
import ctypes
import os
from dataclasses import dataclass

import torch

BLOCK = 32
F32, BF16 = 0, 1
_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libdfp4.so")
_lib = None


class Dfp4Error(RuntimeError):
    pass


class _CTensor(ctypes.Structure):
    _fields_ = [("codes", ctypes.c_void_p), ("dialect", ctypes.c_void_p), ("exponent", ctypes.c_void_p),
                ("rows", ctypes.c_int64), ("K", ctypes.c_int64)]


SYMBOLS = [
    "dfp4_quantize", "dfp4_quantize_b64", "dfp4_quantize_mse", "dfp4_quantize_t", "mxfp4_quantize_t", "dfp4_quantize_t_at", "dfp4_dequantize", "dfp4_gemm", "dfp4_gemm_batched", "dfp4_gemm_workspace_bytes", "dfp4_gemm_noalloc",
    "dfp4_quantize_block", "dfp4_dequantize_block", "dfp4_gemm_blocks",
    "dfp4_gemm_prepared_bytes", "dfp4_gemm_prepare", "mxfp4_gemm_prepare", "dfp4_gemm_prepared_workspace_bytes",
    "dfp4_gemm_prepared", "mxfp4_gemm_prepared", "dfp4_gemm_declined_tiles",
    "mxfp4_gemm_native", "dfp4_gemm_native", "dfp4_gemm_native_workspace_bytes", "dfp4_native_packed_bytes",
    "dfp4_quantize_native", "dfp4_native_pack", "mxfp4_native_pack", "dfp4_gemm_native_packed_w", "mxfp4_gemm_native_packed_w",
    "dfp4_gemm_native_packed", "mxfp4_gemm_native_packed", "dfp4_gemm_native_splitk_bytes",
    "dfp4_gemm_requant", "mxfp4_gemm_requant", "dfp4_gemm_requant_workspace_bytes", "dfp4_gemm_requant_batched",
    "mxfp4_quantize", "mxfp4_dequantize", "mxfp4_gemm", "dfp4_formatbook", "dfp4_strerror",
]


def lib_path():
    return _LIB_PATH


def load():
    """Load libdfp4.so (built by `python -m paper_2501_01144_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise Dfp4Error(f"{_LIB_PATH} not found: build it with `python -m paper_2501_01144_amd.build`")
    lib = ctypes.CDLL(_LIB_PATH)
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    lib.dfp4_quantize.argtypes = [vp, i64, i64, i64, _CTensor, vp]
    lib.mxfp4_quantize.argtypes = [vp, i64, i64, i64, _CTensor, vp]
    lib.dfp4_quantize_mse.argtypes = [vp, i64, i64, i64, _CTensor, vp]
    lib.dfp4_quantize_b64.argtypes = [vp, i64, i64, i64, _CTensor, vp]
    lib.dfp4_quantize_t.argtypes = [vp, i64, i64, i64, _CTensor, vp]
    lib.mxfp4_quantize_t.argtypes = [vp, i64, i64, i64, _CTensor, vp]
    lib.dfp4_quantize_t_at.argtypes = [vp, i64, i64, i64, _CTensor, i64, vp]
    lib.dfp4_quantize_t_at.restype = ci
    lib.dfp4_dequantize.argtypes = [_CTensor, vp, ci, i64, vp]
    lib.mxfp4_dequantize.argtypes = [_CTensor, vp, ci, i64, vp]
    lib.dfp4_gemm.argtypes = [_CTensor, _CTensor, vp, ci, i64, vp, ctypes.c_size_t, vp]
    lib.mxfp4_gemm.argtypes = [_CTensor, _CTensor, vp, ci, i64, vp, ctypes.c_size_t, vp]
    lib.dfp4_gemm_batched.argtypes = [_CTensor, _CTensor, vp, ci, i64, i64, i64, i64, i64, vp,
                                      ctypes.c_size_t, vp]
    lib.dfp4_quantize_block.argtypes = [vp, i64, i64, i64, ci, _CTensor, vp]
    lib.dfp4_quantize_block.restype = ci
    lib.dfp4_dequantize_block.argtypes = [_CTensor, ci, vp, ci, i64, vp]
    lib.dfp4_dequantize_block.restype = ci
    lib.dfp4_gemm_blocks.argtypes = [_CTensor, ci, _CTensor, ci, vp, ci, i64, vp, ctypes.c_size_t, vp]
    lib.dfp4_gemm_blocks.restype = ci
    lib.dfp4_gemm_prepared_bytes.argtypes = [i64, i64, ci]
    lib.dfp4_gemm_prepared_bytes.restype = ctypes.c_size_t
    lib.dfp4_gemm_prepared_workspace_bytes.argtypes = [i64, i64, i64]
    lib.dfp4_gemm_prepared_workspace_bytes.restype = ctypes.c_size_t
    for name in ("dfp4_gemm_prepare", "mxfp4_gemm_prepare"):
        getattr(lib, name).argtypes = [_CTensor, ci, vp, ctypes.c_size_t, vp]
        getattr(lib, name).restype = ci
    for name in ("dfp4_gemm_prepared", "mxfp4_gemm_prepared"):
        getattr(lib, name).argtypes = [_CTensor, vp, _CTensor, vp, vp, ci, i64, vp, ctypes.c_size_t, vp]
        getattr(lib, name).restype = ci
    lib.dfp4_gemm_declined_tiles.argtypes = [vp, i64, i64, ctypes.POINTER(ctypes.c_uint32)]
    lib.dfp4_gemm_declined_tiles.restype = ci
    lib.dfp4_gemm_noalloc.argtypes = [_CTensor, _CTensor, vp, ci, i64, vp]
    lib.dfp4_gemm_noalloc.restype = ci
    lib.dfp4_gemm_workspace_bytes.argtypes = [i64, i64, i64]
    lib.dfp4_gemm_workspace_bytes.restype = ctypes.c_size_t
    lib.mxfp4_gemm_native.argtypes = [_CTensor, _CTensor, vp, ci, i64, vp, ctypes.c_size_t, vp]
    lib.mxfp4_gemm_native.restype = ci
    lib.dfp4_gemm_native.argtypes = [_CTensor, _CTensor, vp, ci, i64, vp, ctypes.c_size_t, vp]
    lib.dfp4_gemm_native.restype = ci
    lib.dfp4_gemm_native_workspace_bytes.argtypes = [i64, i64, i64]
    lib.dfp4_gemm_native_workspace_bytes.restype = ctypes.c_size_t
    lib.dfp4_native_packed_bytes.argtypes = [i64, i64]
    lib.dfp4_native_packed_bytes.restype = ctypes.c_size_t
    lib.dfp4_quantize_native.argtypes = [vp, i64, i64, i64, vp, ctypes.c_size_t, vp]
    lib.dfp4_quantize_native.restype = ci
    for name in ("dfp4_native_pack", "mxfp4_native_pack"):
        getattr(lib, name).argtypes = [_CTensor, vp, ctypes.c_size_t, vp]
        getattr(lib, name).restype = ci
    for name in ("dfp4_gemm_native_packed", "mxfp4_gemm_native_packed"):
        getattr(lib, name).argtypes = [vp, i64, vp, i64, i64, vp, ci, i64, vp, ctypes.c_size_t, vp]
        getattr(lib, name).restype = ci
    lib.dfp4_gemm_native_splitk_bytes.argtypes = [i64, i64, i64]
    lib.dfp4_gemm_native_splitk_bytes.restype = ctypes.c_size_t
    for name in ("dfp4_gemm_native_packed_w", "mxfp4_gemm_native_packed_w"):
        getattr(lib, name).argtypes = [_CTensor, vp, i64, vp, ci, i64, vp, ctypes.c_size_t, vp]
        getattr(lib, name).restype = ci
    lib.dfp4_gemm_requant.argtypes = [_CTensor, _CTensor, _CTensor, vp, ctypes.c_size_t, vp]
    lib.mxfp4_gemm_requant.argtypes = [_CTensor, _CTensor, _CTensor, vp, ctypes.c_size_t, vp]
    lib.dfp4_gemm_requant_batched.argtypes = [_CTensor, _CTensor, _CTensor, i64, i64, i64, vp, ctypes.c_size_t, vp]
    lib.dfp4_gemm_requant_batched.restype = ci
    lib.dfp4_gemm_requant.restype = ci
    lib.mxfp4_gemm_requant.restype = ci
    lib.dfp4_gemm_requant_workspace_bytes.argtypes = [i64, i64, i64]
    lib.dfp4_gemm_requant_workspace_bytes.restype = ctypes.c_size_t
    lib.dfp4_formatbook.argtypes = [vp]
    lib.dfp4_strerror.argtypes = [ci]
    lib.dfp4_strerror.restype = ctypes.c_char_p
    for name in ("dfp4_quantize", "dfp4_quantize_b64", "dfp4_quantize_mse", "dfp4_quantize_t", "mxfp4_quantize_t", "mxfp4_quantize", "dfp4_dequantize", "mxfp4_dequantize", "dfp4_gemm",
                 "mxfp4_gemm", "dfp4_gemm_batched", "dfp4_formatbook"):
        getattr(lib, name).restype = ci
    _lib = lib
    return lib


def strerror(code):
    return load().dfp4_strerror(int(code)).decode()


def _check(rc, what):
    if rc != 0:
        raise Dfp4Error(f"{what} failed: {strerror(rc)} ({rc})")


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr() if t is not None and t.numel() > 0 else 0) if t is not None \
        else ctypes.c_void_p(0)


@dataclass
class QTensor:
    """A quantized [rows, K] tensor on the device (layouts in include/dfp4.h)."""
    codes: torch.Tensor            # uint8 [rows, K/2]
    dialect: torch.Tensor          # uint8 [rows, K/32] or None (MXFP4)
    exponent: torch.Tensor         # uint8 [rows, K/32]
    rows: int
    K: int

    def c(self):
        return _CTensor(_ptr(self.codes).value, _ptr(self.dialect).value, _ptr(self.exponent).value,
                        self.rows, self.K)


def empty_qtensor(rows, K, device, mx=False):
    return QTensor(torch.empty((rows, K // 2), dtype=torch.uint8, device=device),
                   None if mx else torch.empty((rows, K // BLOCK), dtype=torch.uint8, device=device),
                   torch.empty((rows, K // BLOCK), dtype=torch.uint8, device=device), rows, K)


def _quantize(fn, what, x, out, mx):
    assert x.dtype == torch.bfloat16 and x.dim() == 2 and x.is_cuda and x.stride(1) == 1
    rows, K = x.shape
    if out is None:
        out = empty_qtensor(rows, K, x.device, mx)
    ld = x.stride(0) if rows > 1 else K
    _check(fn(_ptr(x), rows, K, ld, out.c(), _stream()), what)
    return out


def quantize(x, out=None):
    """dfp4_quantize: bf16 [rows, K] (row stride allowed) -> QTensor."""
    return _quantize(load().dfp4_quantize, "dfp4_quantize", x, out, False)


def quantize_b64(x, out=None):
    """dfp4_quantize_b64: blocks of 64 elements, output in the layout of the 32-element format."""
    return _quantize(load().dfp4_quantize_b64, "dfp4_quantize_b64", x, out, False)


def quantize_block(x, block, out=None):
    """dfp4_quantize_block: block size 16, 32 or 64.  Blocks of 16 carry dialect / exponent arrays [rows, K/16]."""
    assert x.dtype == torch.bfloat16 and x.dim() == 2 and x.is_cuda and x.stride(1) == 1
    rows, K = x.shape
    if out is None:
        out = empty_qtensor(rows, K, x.device)
        if block == 16:
            out.dialect = torch.empty((rows, K // 16), dtype=torch.uint8, device=x.device)
            out.exponent = torch.empty((rows, K // 16), dtype=torch.uint8, device=x.device)
    ld = x.stride(0) if rows > 1 else K
    _check(load().dfp4_quantize_block(_ptr(x), rows, K, ld, block, out.c(), _stream()), "dfp4_quantize_block")
    return out


def dequantize_block(q, block, dtype=torch.float32, out=None):
    """dfp4_dequantize_block: the inverse of quantize_block for the same block size."""
    if out is None:
        out = torch.empty((q.rows, q.K), dtype=dtype, device=q.codes.device)
    ld = out.stride(0) if q.rows > 1 else q.K
    _check(load().dfp4_dequantize_block(q.c(), block, _ptr(out), F32 if out.dtype == torch.float32 else BF16, ld,
                                        _stream()), "dfp4_dequantize_block")
    return out


def gemm_blocks(a, block_a, w, block_w, dtype=torch.float32, out=None, workspace=None):
    """dfp4_gemm_blocks: product of operands quantized with block sizes block_a / block_w (16, 32 or 64)."""
    if out is None:
        out = torch.empty((a.rows, w.rows), dtype=dtype, device=a.codes.device)
    workspace, nbytes = _workspace(a.rows, w.rows, a.K, out.device, workspace)
    ldc = out.stride(0) if a.rows > 1 else w.rows
    _check(load().dfp4_gemm_blocks(a.c(), block_a, w.c(), block_w, _ptr(out), F32 if out.dtype == torch.float32 else BF16,
                                   ldc, _ptr(workspace), nbytes, _stream()), "dfp4_gemm_blocks")
    return out


def quantize_mse(x, out=None):
    """dfp4_quantize_mse: offline quantization, the dialect of each block chosen by squared error."""
    return _quantize(load().dfp4_quantize_mse, "dfp4_quantize_mse", x, out, False)


def _quantize_t(fn, what, x, out, mx):
    assert x.dtype == torch.bfloat16 and x.dim() == 2 and x.is_cuda and x.stride(1) == 1
    rows, cols = x.shape
    if out is None:
        out = empty_qtensor(cols, rows, x.device, mx)
    ld = x.stride(0) if rows > 1 else cols
    _check(fn(_ptr(x), rows, cols, ld, out.c(), _stream()), what)
    return out


def quantize_t(x, out=None):
    """dfp4_quantize_t: bf16 [rows, cols] -> QTensor of x^T (blocks of 32 along the rows of x)."""
    return _quantize_t(load().dfp4_quantize_t, "dfp4_quantize_t", x, out, False)


def quantize_t_at(x, out, row_offset):
    """dfp4_quantize_t_at: quantize `x` [rows, cols] (rows a multiple of 32) along its rows into the
    quantized transpose `out` [cols, capacity] at token `row_offset`."""
    assert x.dtype == torch.bfloat16 and x.dim() == 2 and x.is_cuda and x.stride(1) == 1
    rows, cols = x.shape
    ld = x.stride(0) if rows > 1 else cols
    _check(load().dfp4_quantize_t_at(_ptr(x), rows, cols, ld, out.c(), row_offset, _stream()), "dfp4_quantize_t_at")
    return out


def mxfp4_quantize_t(x, out=None):
    return _quantize_t(load().mxfp4_quantize_t, "mxfp4_quantize_t", x, out, True)


def mxfp4_quantize(x, out=None):
    return _quantize(load().mxfp4_quantize, "mxfp4_quantize", x, out, True)


def _dequantize(fn, what, q, dtype, out):
    if out is None:
        out = torch.empty((q.rows, q.K), dtype=dtype, device=q.codes.device)
    assert out.dtype in (torch.float32, torch.bfloat16) and out.stride(1) == 1
    ld = out.stride(0) if q.rows > 1 else q.K
    _check(fn(q.c(), _ptr(out), F32 if out.dtype == torch.float32 else BF16, ld, _stream()), what)
    return out


def dequantize(q, dtype=torch.float32, out=None):
    return _dequantize(load().dfp4_dequantize, "dfp4_dequantize", q, dtype, out)


def mxfp4_dequantize(q, dtype=torch.float32, out=None):
    return _dequantize(load().mxfp4_dequantize, "mxfp4_dequantize", q, dtype, out)


def gemm_workspace_bytes(M, N, K):
    return int(load().dfp4_gemm_workspace_bytes(M, N, K))


def _workspace(M, N, K, device, workspace, batch=1):
    need = gemm_workspace_bytes(M, N, K) * batch
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=device)
    return workspace, (workspace.numel() if workspace is not None else 0)


def _gemm(fn, what, a, w, dtype, out, workspace):
    if out is None:
        out = torch.empty((a.rows, w.rows), dtype=dtype, device=a.codes.device)
    assert out.dtype in (torch.float32, torch.bfloat16) and out.stride(1) == 1
    workspace, nbytes = _workspace(a.rows, w.rows, a.K, out.device, workspace)
    ldc = out.stride(0) if a.rows > 1 else w.rows
    _check(fn(a.c(), w.c(), _ptr(out), F32 if out.dtype == torch.float32 else BF16, ldc,
              _ptr(workspace), nbytes, _stream()), what)
    return out


def gemm(a, w, dtype=torch.float32, out=None, workspace=None):
    """dfp4_gemm: out[M, N] = A[M, K] * W[N, K]^T on quantized operands."""
    return _gemm(load().dfp4_gemm, "dfp4_gemm", a, w, dtype, out, workspace)


@dataclass
class PreparedOperand:
    """A quantized tensor together with its prepared form (dfp4_gemm_prepare)."""
    q: "QTensor"
    buf: torch.Tensor              # uint8, private layout; None when nothing is prepared for this operand
    weight: bool
    mx: bool


def gemm_prepare(q, weight, mx=False, buf=None):
    """dfp4_gemm_prepare / mxfp4_gemm_prepare: the per-operand work of the GEMM, done once."""
    need = int(load().dfp4_gemm_prepared_bytes(q.rows, q.K, 1 if weight else 0))
    if need == 0:
        return PreparedOperand(q, None, weight, mx)
    if buf is None:
        buf = torch.empty(need, dtype=torch.uint8, device=q.codes.device)
    fn = load().mxfp4_gemm_prepare if mx else load().dfp4_gemm_prepare
    _check(fn(q.c(), 1 if weight else 0, _ptr(buf), buf.numel(), _stream()), "gemm_prepare")
    return PreparedOperand(q, buf, weight, mx)


def gemm_prepared(a, w, dtype=torch.float32, out=None, workspace=None):
    """dfp4_gemm_prepared / mxfp4_gemm_prepared: a, w are PreparedOperands."""
    assert not a.weight and w.weight and a.mx == w.mx
    if out is None:
        out = torch.empty((a.q.rows, w.q.rows), dtype=dtype, device=a.q.codes.device)
    assert out.dtype in (torch.float32, torch.bfloat16) and out.stride(1) == 1
    need = int(load().dfp4_gemm_prepared_workspace_bytes(a.q.rows, w.q.rows, a.q.K))
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=out.device)
    fn = load().mxfp4_gemm_prepared if a.mx else load().dfp4_gemm_prepared
    ldc = out.stride(0) if a.q.rows > 1 else w.q.rows
    _check(fn(a.q.c(), _ptr(a.buf), w.q.c(), _ptr(w.buf), _ptr(out), F32 if out.dtype == torch.float32 else BF16,
              ldc, _ptr(workspace), workspace.numel() if workspace is not None else 0, _stream()), "gemm_prepared")
    return out


def gemm_declined_tiles(a):
    """dfp4_gemm_declined_tiles: tiles of products on this prepared A that took the per-block fp32 path."""
    n = ctypes.c_uint32(0)
    _check(load().dfp4_gemm_declined_tiles(_ptr(a.buf), a.q.rows, a.q.K, ctypes.byref(n)), "dfp4_gemm_declined_tiles")
    return int(n.value)


NOALLOC_SCRATCH_BYTES = 64 << 20


def gemm_noalloc(a, w, out):
    """dfp4_gemm_noalloc: dfp4_gemm on the library's own fixed scratch array; `out` must be given
    (nothing is allocated on either side of the boundary)."""
    assert out.dtype in (torch.float32, torch.bfloat16) and out.stride(1) == 1
    ldc = out.stride(0) if a.rows > 1 else w.rows
    _check(load().dfp4_gemm_noalloc(a.c(), w.c(), _ptr(out), F32 if out.dtype == torch.float32 else BF16, ldc,
                                    _stream()), "dfp4_gemm_noalloc")
    return out


def mxfp4_gemm(a, w, dtype=torch.float32, out=None, workspace=None):
    return _gemm(load().mxfp4_gemm, "mxfp4_gemm", a, w, dtype, out, workspace)


def _gemm_requant(fn, what, a, w, out, workspace, mx):
    if out is None:
        out = empty_qtensor(a.rows, w.rows, a.codes.device, mx)
    need = int(load().dfp4_gemm_requant_workspace_bytes(a.rows, w.rows, a.K))
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=a.codes.device)
    _check(fn(a.c(), w.c(), out.c(), _ptr(workspace), workspace.numel() if workspace is not None else 0, _stream()),
           what)
    return out


def gemm_requant(a, w, out=None, workspace=None):
    """dfp4_gemm_requant: quantize(bf16(A W^T)) in blocks of 32 along N -> QTensor [M, N]."""
    return _gemm_requant(load().dfp4_gemm_requant, "dfp4_gemm_requant", a, w, out, workspace, False)


def gemm_requant_batched(a, w, batch, M, N, out=None, workspace=None):
    """dfp4_gemm_requant_batched: a holds batch*M rows, w batch*N rows; returns the quantized [batch*M, N] result."""
    if out is None:
        out = empty_qtensor(batch * M, N, a.codes.device)
    need = int(load().dfp4_gemm_requant_workspace_bytes(M, N, a.K)) * batch
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=a.codes.device)
    ac, wc = a.c(), w.c()
    ac.rows, wc.rows = M, N
    _check(load().dfp4_gemm_requant_batched(ac, wc, out.c(), batch, M, N, _ptr(workspace), workspace.numel(), _stream()),
           "dfp4_gemm_requant_batched")
    return out


def mxfp4_gemm_requant(a, w, out=None, workspace=None):
    return _gemm_requant(load().mxfp4_gemm_requant, "mxfp4_gemm_requant", a, w, out, workspace, True)


def _gemm_native(fn, what, a, w, dtype, out, workspace):
    if out is None:
        out = torch.empty((a.rows, w.rows), dtype=dtype, device=a.codes.device)
    assert out.dtype in (torch.float32, torch.bfloat16) and out.stride(1) == 1
    need = int(load().dfp4_gemm_native_workspace_bytes(a.rows, w.rows, a.K))
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=out.device)
    ldc = out.stride(0) if a.rows > 1 else w.rows
    _check(fn(a.c(), w.c(), _ptr(out), F32 if out.dtype == torch.float32 else BF16, ldc, _ptr(workspace),
              workspace.numel() if workspace is not None else 0, _stream()), what)
    return out


def gemm_native(a, w, dtype=torch.float32, out=None, workspace=None):
    """dfp4_gemm_native: DialectFP4 product on the block-scaled matrix instruction (FP6 E2M3 operands)."""
    return _gemm_native(load().dfp4_gemm_native, "dfp4_gemm_native", a, w, dtype, out, workspace)


def mxfp4_gemm_native(a, w, dtype=torch.float32, out=None, workspace=None):
    """mxfp4_gemm_native: the MXFP4 product on the block-scaled matrix instruction (FP4 operands)."""
    return _gemm_native(load().mxfp4_gemm_native, "mxfp4_gemm_native", a, w, dtype, out, workspace)


@dataclass
class PackedWeights:
    """A quantized [rows, K] tensor in the matrix instruction's register order (dfp4_native_pack)."""
    buf: torch.Tensor
    rows: int
    K: int
    mx: bool


def native_pack(w, mx=False, buf=None):
    """dfp4_native_pack / mxfp4_native_pack: pack a quantized tensor (weights: once)."""
    n = int(load().dfp4_native_packed_bytes(w.rows, w.K))
    if buf is None:
        buf = torch.empty(max(n, 256), dtype=torch.uint8, device=w.codes.device)
    fn = load().mxfp4_native_pack if mx else load().dfp4_native_pack
    _check(fn(w.c(), _ptr(buf), buf.numel(), _stream()), "native_pack")
    return PackedWeights(buf, w.rows, w.K, mx)


def quantize_native(x, buf=None):
    """dfp4_quantize_native: bf16 [rows, K] -> packed FP6 operand of the block-scaled matrix instruction."""
    assert x.dtype == torch.bfloat16 and x.dim() == 2 and x.is_cuda and x.stride(1) == 1
    rows, K = x.shape
    n = int(load().dfp4_native_packed_bytes(rows, K))
    if buf is None:
        buf = torch.zeros(max(n, 256), dtype=torch.uint8, device=x.device)
    ld = x.stride(0) if rows > 1 else K
    _check(load().dfp4_quantize_native(_ptr(x), rows, K, ld, _ptr(buf), buf.numel(), _stream()), "dfp4_quantize_native")
    return PackedWeights(buf, rows, K, False)


def gemm_native_packed_w(a, wp, dtype=torch.float32, out=None, workspace=None):
    """dfp4_gemm_native_packed_w / mxfp4_gemm_native_packed_w: A quantized, W packed beforehand."""
    if out is None:
        out = torch.empty((a.rows, wp.rows), dtype=dtype, device=a.codes.device)
    assert out.dtype in (torch.float32, torch.bfloat16) and out.stride(1) == 1 and a.K == wp.K
    need = int(load().dfp4_native_packed_bytes(a.rows, a.K)) + \
        int(load().dfp4_gemm_native_splitk_bytes(a.rows, wp.rows, a.K))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=out.device)
    fn = load().mxfp4_gemm_native_packed_w if wp.mx else load().dfp4_gemm_native_packed_w
    ldc = out.stride(0) if a.rows > 1 else wp.rows
    _check(fn(a.c(), _ptr(wp.buf), wp.rows, _ptr(out), F32 if out.dtype == torch.float32 else BF16, ldc,
              _ptr(workspace), workspace.numel(), _stream()), "gemm_native_packed_w")
    return out


def gemm_native_packed(ap, wp, dtype=torch.float32, out=None, workspace=None):
    """dfp4_gemm_native_packed / mxfp4_gemm_native_packed: both operands packed beforehand."""
    if out is None:
        out = torch.empty((ap.rows, wp.rows), dtype=dtype, device=ap.buf.device)
    need = int(load().dfp4_gemm_native_splitk_bytes(ap.rows, wp.rows, ap.K))
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=out.device)
    assert out.dtype in (torch.float32, torch.bfloat16) and out.stride(1) == 1 and ap.K == wp.K and ap.mx == wp.mx
    fn = load().mxfp4_gemm_native_packed if wp.mx else load().dfp4_gemm_native_packed
    ldc = out.stride(0) if ap.rows > 1 else wp.rows
    _check(fn(_ptr(ap.buf), ap.rows, _ptr(wp.buf), wp.rows, ap.K, _ptr(out),
              F32 if out.dtype == torch.float32 else BF16, ldc, _ptr(workspace),
              workspace.numel() if workspace is not None else 0, _stream()), "gemm_native_packed")
    return out


def gemm_batched(a, w, batch, M, N, dtype=torch.float32, out=None, workspace=None):
    """dfp4_gemm_batched: a holds batch*M rows, w batch*N rows (problem after problem);
    out [batch, M, N]."""
    if out is None:
        out = torch.empty((batch, M, N), dtype=dtype, device=a.codes.device)
    assert out.is_contiguous()
    ac, wc = a.c(), w.c()
    ac.rows, wc.rows = M, N
    workspace, nbytes = _workspace(M, N, a.K, out.device, workspace, batch)
    _check(load().dfp4_gemm_batched(ac, wc, _ptr(out), F32 if out.dtype == torch.float32 else BF16, N,
                                    batch, M, N, M * N, _ptr(workspace), nbytes, _stream()),
           "dfp4_gemm_batched")
    return out


def formatbook():
    """The library's formatbook as a 16 x 8 list of half-unit magnitudes."""
    buf = (ctypes.c_uint8 * 128)()
    _check(load().dfp4_formatbook(ctypes.cast(buf, ctypes.c_void_p)), "dfp4_formatbook")
    return [[int(buf[d * 8 + j]) for j in range(8)] for d in range(16)]
