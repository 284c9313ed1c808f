"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every function include/dfp4.h declares, reports the formatbook the oracle
uses, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from oracle import dfp4_oracle as O
from paper_2501_01144_amd import dfp4

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(dfp4.lib_path()):
        from paper_2501_01144_amd.build import build_library
        build_library(verbose=False)
    return dfp4.load()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "dfp4.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:dfp4|mxfp4)_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert len(names) >= 10
    assert sorted(dfp4.SYMBOLS) == names
    for n in names:
        assert getattr(lib, n) is not None


def test_formatbook_matches_the_oracle_table(lib):
    assert dfp4.formatbook() == O.FORMATBOOK_HALF_UNITS.tolist()


def test_strerror(lib):
    assert dfp4.strerror(0) == "ok"
    for code in range(-6, 0):
        assert dfp4.strerror(code) not in ("ok", "unknown error")
    assert dfp4.strerror(-99) == "unknown error"


def _t(codes=0, dialect=0, exponent=0, rows=0, K=0):
    return dfp4._CTensor(codes, dialect, exponent, rows, K)


def test_argument_errors_are_reported_without_a_device(lib):
    vp = ctypes.c_void_p
    # K not a multiple of 32, negative rows, ld < K, mismatched out shape
    assert lib.dfp4_quantize(vp(16), 4, 48, 48, _t(16, 16, 16, 4, 48), vp(0)) == -2
    assert lib.dfp4_quantize(vp(16), -1, 64, 64, _t(16, 16, 16, -1, 64), vp(0)) == -2
    assert lib.dfp4_quantize(vp(16), 4, 64, 32, _t(16, 16, 16, 4, 64), vp(0)) == -2
    assert lib.dfp4_quantize(vp(16), 4, 64, 64, _t(16, 16, 16, 4, 32), vp(0)) == -2
    # null pointers
    assert lib.dfp4_quantize(vp(0), 4, 64, 64, _t(16, 16, 16, 4, 64), vp(0)) == -1
    assert lib.dfp4_quantize(vp(16), 4, 64, 64, _t(16, 0, 16, 4, 64), vp(0)) == -1
    assert lib.mxfp4_quantize(vp(16), 4, 64, 64, _t(0, 0, 16, 4, 64), vp(0)) == -1
    # alignment: x must be 16-byte aligned, ld a multiple of 8
    assert lib.dfp4_quantize(vp(8), 4, 64, 64, _t(16, 16, 16, 4, 64), vp(0)) == -3
    assert lib.dfp4_quantize(vp(16), 4, 64, 68, _t(16, 16, 16, 4, 64), vp(0)) == -3
    # dtype
    assert lib.dfp4_dequantize(_t(16, 16, 16, 4, 64), vp(16), 7, 64, vp(0)) == -4
    assert lib.dfp4_gemm(_t(16, 16, 16, 4, 64), _t(16, 16, 16, 4, 64), vp(16), 9, 4, vp(0), 0, vp(0)) == -4
    # gemm: mismatched K, ldc < N, null output
    assert lib.dfp4_gemm(_t(16, 16, 16, 4, 64), _t(16, 16, 16, 4, 96), vp(16), 0, 4, vp(0), 0, vp(0)) == -2
    assert lib.dfp4_gemm(_t(16, 16, 16, 4, 64), _t(16, 16, 16, 8, 64), vp(16), 0, 4, vp(0), 0, vp(0)) == -2
    assert lib.dfp4_gemm(_t(16, 16, 16, 4, 64), _t(16, 16, 16, 4, 64), vp(0), 0, 4, vp(0), 0, vp(0)) == -1
    # empty problems succeed as no-ops
    assert lib.dfp4_quantize(vp(0), 0, 64, 64, _t(0, 0, 0, 0, 64), vp(0)) == 0
    assert lib.dfp4_gemm(_t(0, 0, 0, 0, 64), _t(16, 16, 16, 4, 64), vp(0), 0, 4, vp(0), 0, vp(0)) == 0
    assert lib.dfp4_formatbook(vp(0)) == -1


def test_binding_refuses_to_run_without_the_library(monkeypatch):
    monkeypatch.setattr(dfp4, "_lib", None)
    monkeypatch.setattr(dfp4, "_LIB_PATH", "/nonexistent/libdfp4.so")
    with pytest.raises(dfp4.Dfp4Error):
        dfp4.load()


def test_header_compiles_as_c99(tmp_path):
    # the boundary is a C ABI: the public header must be plain C
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    header = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "dfp4.h")
    src = tmp_path / "t.c"
    src.write_text('#include "%s"\nint main(void) { return dfp4_strerror(0) == 0; }\n' % header)
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-c", str(src), "-o",
                    str(tmp_path / "t.o")], check=True)


def test_argument_errors_of_the_later_entry_points(lib):
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    q = _t(16, 16, 16, 64, 64)
    # MSE and transposing quantizers: same checks as dfp4_quantize; the transposing one needs rows % 32 == 0
    assert lib.dfp4_quantize_mse(vp(16), 4, 48, 48, _t(16, 16, 16, 4, 48), vp(0)) == -2
    assert lib.dfp4_quantize_mse(vp(0), 4, 64, 64, _t(16, 16, 16, 4, 64), vp(0)) == -1
    assert lib.dfp4_quantize_t(vp(16), 48, 64, 64, _t(16, 16, 16, 64, 48), vp(0)) == -2
    assert lib.dfp4_quantize_t(vp(16), 64, 64, 64, _t(16, 16, 16, 64, 32), vp(0)) == -2
    assert lib.dfp4_quantize_t(vp(8), 64, 64, 64, q, vp(0)) == -3
    assert lib.mxfp4_quantize_t(vp(16), 64, 64, 64, _t(0, 0, 16, 64, 64), vp(0)) == -1
    # requantizing GEMM: N must be a multiple of 32, the output shape [M, N], a workspace is required
    a, w = _t(16, 16, 16, 64, 64), _t(16, 16, 16, 48, 64)
    assert lib.dfp4_gemm_requant(a, w, _t(16, 16, 16, 64, 48), vp(256), sz(1 << 30), vp(0)) == -2
    w = _t(16, 16, 16, 64, 64)
    assert lib.dfp4_gemm_requant(a, w, _t(16, 16, 16, 64, 32), vp(256), sz(1 << 30), vp(0)) == -2
    assert lib.dfp4_gemm_requant(a, w, _t(0, 16, 16, 64, 64), vp(256), sz(1 << 30), vp(0)) == -1
    assert lib.dfp4_gemm_requant(a, w, q, vp(0), sz(0), vp(0)) == -5
    assert lib.dfp4_gemm_requant_workspace_bytes(64, 64, 64) > lib.dfp4_gemm_workspace_bytes(64, 64, 64)
    # native family: packed sizes, workspace and alignment checks
    need = lib.dfp4_native_packed_bytes(64, 64)
    assert need > 0 and lib.dfp4_native_packed_bytes(0, 64) == 0
    assert lib.dfp4_native_pack(a, vp(256), sz(need - 1), vp(0)) == -5
    assert lib.dfp4_native_pack(a, vp(128), sz(need), vp(0)) == -3
    assert lib.dfp4_native_pack(_t(16, 0, 16, 64, 64), vp(256), sz(need), vp(0)) == -1
    assert lib.mxfp4_native_pack(_t(16, 0, 16, 64, 48), vp(256), sz(need), vp(0)) == -2
    assert lib.dfp4_quantize_native(vp(16), 64, 64, 64, vp(256), sz(need - 1), vp(0)) == -5
    assert lib.dfp4_quantize_native(vp(16), 64, 64, 32, vp(256), sz(need), vp(0)) == -2
    assert lib.dfp4_gemm_native(a, w, vp(16), 0, 64, vp(256), sz(need), vp(0)) == -5          # two operands do not fit
    assert lib.dfp4_gemm_native(a, _t(16, 16, 16, 64, 96), vp(16), 0, 64, vp(256), sz(1 << 30), vp(0)) == -2
    assert lib.dfp4_gemm_native(a, w, vp(16), 3, 64, vp(256), sz(1 << 30), vp(0)) == -4
    assert lib.dfp4_gemm_native_packed_w(a, vp(0), 64, vp(16), 0, 64, vp(256), sz(1 << 30), vp(0)) == -1
    assert lib.dfp4_gemm_native_packed(vp(256), 64, vp(256), 64, 48, vp(16), 0, 64, vp(0), sz(0), vp(0)) == -2
    assert lib.dfp4_gemm_native_packed(vp(256), 64, vp(128), 64, 64, vp(16), 0, 64, vp(0), sz(0), vp(0)) == -3
    assert lib.dfp4_gemm_native_packed(vp(256), 0, vp(256), 64, 64, vp(16), 0, 64, vp(0), sz(0), vp(0)) == 0


def test_gemm_noalloc_argument_errors(lib):
    vp = ctypes.c_void_p
    # a product whose workspace exceeds the library's fixed scratch array is refused before anything else
    big_a, big_w = _t(16, 16, 16, 2048, 14336), _t(16, 16, 16, 4096, 14336)
    assert lib.dfp4_gemm_workspace_bytes(2048, 4096, 14336) > (64 << 20)
    assert lib.dfp4_gemm_noalloc(big_a, big_w, vp(16), 0, 4096, vp(0)) == -5
    assert b"workspace" in lib.dfp4_strerror(-5)
    # the other checks are those of dfp4_gemm
    assert lib.dfp4_gemm_noalloc(_t(16, 16, 16, 4, 64), _t(16, 16, 16, 4, 96), vp(16), 0, 4, vp(0)) == -2
    assert lib.dfp4_gemm_noalloc(_t(16, 16, 16, 4, 64), _t(16, 16, 16, 4, 64), vp(16), 9, 4, vp(0)) == -4
    assert lib.dfp4_gemm_noalloc(_t(16, 16, 16, 4, 64), _t(16, 16, 16, 4, 64), vp(0), 0, 4, vp(0)) == -1
    assert lib.dfp4_gemm_noalloc(_t(0, 0, 0, 0, 64), _t(16, 16, 16, 4, 64), vp(0), 0, 4, vp(0)) == 0


def test_block_size_entry_points_argument_errors(lib):
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    q = _t(16, 16, 16, 4, 64)
    assert lib.dfp4_quantize_block(vp(16), 4, 64, 64, 8, q, vp(0)) == -2          # block size not 16 / 32 / 64
    assert lib.dfp4_quantize_block(vp(16), 4, 96, 96, 64, _t(16, 16, 16, 4, 96), vp(0)) == -2   # K % 64
    assert lib.dfp4_quantize_block(vp(0), 4, 64, 64, 16, q, vp(0)) == -1
    assert lib.dfp4_quantize_block(vp(16), 0, 64, 64, 16, _t(0, 0, 0, 0, 64), vp(0)) == 0
    assert lib.dfp4_dequantize_block(q, 48, vp(16), 0, 64, vp(0)) == -2
    assert lib.dfp4_dequantize_block(q, 16, vp(16), 5, 64, vp(0)) == -4
    assert lib.dfp4_gemm_blocks(q, 16, _t(16, 16, 16, 4, 96), 16, vp(16), 0, 4, vp(0), sz(0), vp(0)) == -2
    assert lib.dfp4_gemm_blocks(q, 16, q, 24, vp(16), 0, 4, vp(0), sz(0), vp(0)) == -2
    assert lib.dfp4_gemm_blocks(q, 16, q, 16, vp(0), 0, 4, vp(0), sz(0), vp(0)) == -1


def test_gemm_requant_batched_argument_errors(lib):
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    a, w = _t(16, 16, 16, 64, 64), _t(16, 16, 16, 64, 64)
    assert lib.dfp4_gemm_requant_batched(a, w, _t(16, 16, 16, 64, 64), 2, 64, 64, vp(256), sz(1 << 30), vp(0)) == -2   # out.rows != batch * M
    assert lib.dfp4_gemm_requant_batched(a, w, _t(16, 16, 16, 128, 64), 2, 64, 64, vp(0), sz(0), vp(0)) == -5
    assert lib.dfp4_gemm_requant_batched(a, w, _t(16, 16, 16, 128, 64), -1, 64, 64, vp(256), sz(1 << 30), vp(0)) == -2
    assert lib.dfp4_gemm_requant_batched(a, w, _t(16, 16, 16, 0, 64), 0, 64, 64, vp(0), sz(0), vp(0)) == 0
