// extern "C" entry points of libdfp4 (see include/dfp4.h): argument checks
// and dispatch to the kernels.  No device memory is allocated here.
#include <mutex>

#include "common.h"
#include "formatbook.h"

namespace dfp4 {

int device_cu_count() {
    static std::mutex mu;
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    std::lock_guard<std::mutex> lock(mu);
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

int check_quant_args(const void* dense, int64_t rows, int64_t K, int64_t ld, const dfp4_tensor& q,
                     bool need_dialect) {
    if (rows < 0 || K < 0 || K % kBlock != 0 || ld < K || q.rows != rows || q.K != K) return DFP4_ERR_SHAPE;
    if (rows == 0 || K == 0) return DFP4_OK;
    if (!dense || !q.codes || !q.exponent || (need_dialect && !q.dialect)) return DFP4_ERR_NULL;
    if (ld % 8 != 0 || !aligned(dense, 16) || !aligned(q.codes, 4)) return DFP4_ERR_ALIGN;
    return DFP4_OK;
}

static int check_gemm_args(const dfp4_tensor& A, const dfp4_tensor& W, const void* out, int out_dtype,
                           int64_t ldc, bool need_dialect, const void* workspace, size_t workspace_bytes) {
    if (A.rows < 0 || W.rows < 0 || A.K < 0 || A.K != W.K || A.K % kBlock != 0) return DFP4_ERR_SHAPE;
    if (out_dtype != DFP4_F32 && out_dtype != DFP4_BF16) return DFP4_ERR_DTYPE;
    if (A.rows == 0 || W.rows == 0) return DFP4_OK;
    if (ldc < W.rows) return DFP4_ERR_SHAPE;
    if (!out) return DFP4_ERR_NULL;
    if (A.K > 0) {
        if (!A.codes || !A.exponent || !W.codes || !W.exponent) return DFP4_ERR_NULL;
        if (need_dialect && (!A.dialect || !W.dialect)) return DFP4_ERR_NULL;
        if (!aligned(A.codes, 16) || !aligned(W.codes, 16)) return DFP4_ERR_ALIGN;
    }
    const size_t need = gemm_workspace_bytes(A.rows, W.rows, A.K);
    if (need > 0) {
        if (!workspace || workspace_bytes < need) return DFP4_ERR_WORKSPACE;
        if (!aligned(workspace, 256)) return DFP4_ERR_ALIGN;
    }
    return gemm_shape_check(A, W, ldc, 1, false);
}

// Device memory of dfp4_gemm_noalloc: one array per GPU, part of the library's code object, so
// that the call needs no allocation at all.  Every call on a GPU shares that GPU's array.
static __device__ __align__(256) uint8_t scratch[DFP4_NOALLOC_SCRATCH_BYTES];

// Address of `scratch` on the current device (looked up once per device, with that device current;
// in host code the array's name is only a handle for this lookup, never an address).
static int noalloc_scratch(void** out) {
    static std::mutex mu;
    static void* ptr[64] = {nullptr};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return DFP4_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return DFP4_ERR_LAUNCH;
        }
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return DFP4_OK;
}

}  // namespace dfp4

using namespace dfp4;

extern "C" {

int dfp4_quantize(const void* x_bf16, int64_t rows, int64_t K, int64_t ld_elems, dfp4_tensor out,
                  void* stream) {
    const int rc = check_quant_args(x_bf16, rows, K, ld_elems, out, true);
    if (rc != DFP4_OK) return rc;
    return launch_quantize(false, x_bf16, rows, K, ld_elems, out, static_cast<hipStream_t>(stream));
}

// x [rows, cols] quantized along its rows into rows [row_offset, row_offset + rows) of the K axis of `out`
// (the quantized transpose [cols, out.K])
static int quantize_t_common(bool mx, const void* x, int64_t rows, int64_t cols, int64_t ld, dfp4_tensor out,
                             int64_t row_offset, void* stream) {
    if (rows < 0 || cols < 0 || rows % kBlock != 0 || cols % 8 != 0 || ld < cols || out.rows != cols ||
        row_offset < 0 || row_offset % kBlock != 0 || out.K % kBlock != 0 || row_offset + rows > out.K)
        return DFP4_ERR_SHAPE;
    if (rows == 0 || cols == 0) return DFP4_OK;
    if (!x || !out.codes || !out.exponent || (!mx && !out.dialect)) return DFP4_ERR_NULL;
    if (ld % 8 != 0 || !aligned(x, 16) || !aligned(out.codes, 4)) return DFP4_ERR_ALIGN;
    if (out.K / kBlock >= ((int64_t)1 << 31) / (cols > 0 ? cols : 1)) return DFP4_ERR_SHAPE;
    return launch_quantize_t(mx, x, rows, cols, ld, out, row_offset, static_cast<hipStream_t>(stream));
}

int dfp4_quantize_t(const void* x_bf16, int64_t rows, int64_t cols, int64_t ld_elems, dfp4_tensor out,
                    void* stream) {
    if (out.K != rows) return DFP4_ERR_SHAPE;
    return quantize_t_common(false, x_bf16, rows, cols, ld_elems, out, 0, stream);
}

int mxfp4_quantize_t(const void* x_bf16, int64_t rows, int64_t cols, int64_t ld_elems, dfp4_tensor out,
                     void* stream) {
    if (out.K != rows) return DFP4_ERR_SHAPE;
    return quantize_t_common(true, x_bf16, rows, cols, ld_elems, out, 0, stream);
}

int dfp4_quantize_t_at(const void* x_bf16, int64_t rows, int64_t cols, int64_t ld_elems, dfp4_tensor out,
                       int64_t row_offset, void* stream) {
    return quantize_t_common(false, x_bf16, rows, cols, ld_elems, out, row_offset, stream);
}

int dfp4_quantize_mse(const void* x_bf16, int64_t rows, int64_t K, int64_t ld_elems, dfp4_tensor out,
                      void* stream) {
    const int rc = check_quant_args(x_bf16, rows, K, ld_elems, out, true);
    if (rc != DFP4_OK) return rc;
    return launch_quantize_mse(x_bf16, rows, K, ld_elems, out, static_cast<hipStream_t>(stream));
}

int dfp4_quantize_b64(const void* x_bf16, int64_t rows, int64_t K, int64_t ld_elems, dfp4_tensor out,
                      void* stream) {
    if (K % 64 != 0) return DFP4_ERR_SHAPE;
    const int rc = check_quant_args(x_bf16, rows, K, ld_elems, out, true);
    if (rc != DFP4_OK) return rc;
    return launch_quantize(false, x_bf16, rows, K, ld_elems, out, static_cast<hipStream_t>(stream), true);
}

static bool block_size_ok(int b) { return b == 16 || b == 32 || b == 64; }

int dfp4_quantize_block(const void* x_bf16, int64_t rows, int64_t K, int64_t ld_elems, int block_size, dfp4_tensor out,
                        void* stream) {
    if (!block_size_ok(block_size) || (block_size == 64 && K % 64 != 0)) return DFP4_ERR_SHAPE;
    const int rc = check_quant_args(x_bf16, rows, K, ld_elems, out, true);
    if (rc != DFP4_OK) return rc;
    return launch_quantize(false, x_bf16, rows, K, ld_elems, out, static_cast<hipStream_t>(stream), block_size == 64,
                           block_size == 16);
}

int dfp4_dequantize_block(dfp4_tensor in, int block_size, void* y, int y_dtype, int64_t ld_elems, void* stream) {
    if (!block_size_ok(block_size)) return DFP4_ERR_SHAPE;
    if (y_dtype != DFP4_F32 && y_dtype != DFP4_BF16) return DFP4_ERR_DTYPE;
    const int rc = check_quant_args(y, in.rows, in.K, ld_elems, in, true);
    if (rc != DFP4_OK) return rc;
    return launch_dequantize(false, in, y, y_dtype, ld_elems, static_cast<hipStream_t>(stream), block_size == 16);
}

int dfp4_gemm_blocks(dfp4_tensor A, int block_a, dfp4_tensor W, int block_w, void* out, int out_dtype, int64_t ldc,
                     void* workspace, size_t workspace_bytes, void* stream) {
    if (!block_size_ok(block_a) || !block_size_ok(block_w)) return DFP4_ERR_SHAPE;
    if (block_a != 16 && block_w != 16)               // blocks of 32 and 64 share the 32-element layout
        return dfp4_gemm(A, W, out, out_dtype, ldc, workspace, workspace_bytes, stream);
    const int rc = check_gemm_args(A, W, out, out_dtype, ldc, true, reinterpret_cast<void*>(uintptr_t{256}), ~(size_t)0);
    if (rc != DFP4_OK) return rc;
    return launch_gemm_block16(A, block_a == 16, W, block_w == 16, out, out_dtype, ldc, static_cast<hipStream_t>(stream));
}

int mxfp4_quantize(const void* x_bf16, int64_t rows, int64_t K, int64_t ld_elems, dfp4_tensor out,
                   void* stream) {
    const int rc = check_quant_args(x_bf16, rows, K, ld_elems, out, false);
    if (rc != DFP4_OK) return rc;
    return launch_quantize(true, x_bf16, rows, K, ld_elems, out, static_cast<hipStream_t>(stream));
}

static int dequantize_common(bool mx, dfp4_tensor in, void* y, int y_dtype, int64_t ld, void* stream) {
    if (y_dtype != DFP4_F32 && y_dtype != DFP4_BF16) return DFP4_ERR_DTYPE;
    const int rc = check_quant_args(y, in.rows, in.K, ld, in, !mx);
    if (rc != DFP4_OK) return rc;
    return launch_dequantize(mx, in, y, y_dtype, ld, static_cast<hipStream_t>(stream));
}

int dfp4_dequantize(dfp4_tensor in, void* y, int y_dtype, int64_t ld_elems, void* stream) {
    return dequantize_common(false, in, y, y_dtype, ld_elems, stream);
}

int mxfp4_dequantize(dfp4_tensor in, void* y, int y_dtype, int64_t ld_elems, void* stream) {
    return dequantize_common(true, in, y, y_dtype, ld_elems, stream);
}

int dfp4_gemm(dfp4_tensor A, dfp4_tensor W, void* out, int out_dtype, int64_t ldc, void* workspace,
              size_t workspace_bytes, void* stream) {
    const int rc = check_gemm_args(A, W, out, out_dtype, ldc, true, workspace, workspace_bytes);
    if (rc != DFP4_OK) return rc;
    return launch_gemm(false, A, W, out, out_dtype, ldc, 1, 0, 0, 0, workspace, workspace_bytes,
                       static_cast<hipStream_t>(stream));
}

int dfp4_gemm_noalloc(dfp4_tensor A, dfp4_tensor W, void* out, int out_dtype, int64_t ldc, void* stream) {
    if (A.rows < 0 || W.rows < 0 || A.K < 0) return DFP4_ERR_SHAPE;
    // the size check comes first: a product that does not fit is refused whatever else is wrong with it
    if (gemm_workspace_bytes(A.rows, W.rows, A.K) > (size_t)DFP4_NOALLOC_SCRATCH_BYTES) return DFP4_ERR_WORKSPACE;
    // argument checks first (with a stand-in for the workspace pointer), then the scratch array's address
    int rc = check_gemm_args(A, W, out, out_dtype, ldc, true, reinterpret_cast<void*>(uintptr_t{256}),
                             DFP4_NOALLOC_SCRATCH_BYTES);
    if (rc != DFP4_OK) return rc;
    if (A.rows == 0 || W.rows == 0) return DFP4_OK;
    void* ws = nullptr;
    rc = noalloc_scratch(&ws);
    if (rc != DFP4_OK) return rc;
    return launch_gemm(false, A, W, out, out_dtype, ldc, 1, 0, 0, 0, ws, DFP4_NOALLOC_SCRATCH_BYTES,
                       static_cast<hipStream_t>(stream));
}

int mxfp4_gemm(dfp4_tensor A, dfp4_tensor W, void* out, int out_dtype, int64_t ldc, void* workspace,
               size_t workspace_bytes, void* stream) {
    const int rc = check_gemm_args(A, W, out, out_dtype, ldc, false, workspace, workspace_bytes);
    if (rc != DFP4_OK) return rc;
    return launch_gemm(true, A, W, out, out_dtype, ldc, 1, 0, 0, 0, workspace, workspace_bytes,
                       static_cast<hipStream_t>(stream));
}

int dfp4_gemm_batched(dfp4_tensor A, dfp4_tensor W, void* out, int out_dtype, int64_t ldc, int64_t batch,
                      int64_t strideA_rows, int64_t strideW_rows, int64_t strideC, void* workspace,
                      size_t workspace_bytes, void* stream) {
    if (batch < 0 || strideA_rows < 0 || strideW_rows < 0 || strideC < 0) return DFP4_ERR_SHAPE;
    const int rc = check_gemm_args(A, W, out, out_dtype, ldc, true, workspace, workspace_bytes);
    if (rc != DFP4_OK) return rc;
    if (batch > 0 && workspace_bytes / (size_t)batch < gemm_workspace_bytes(A.rows, W.rows, A.K)) return DFP4_ERR_WORKSPACE;
    return launch_gemm(false, A, W, out, out_dtype, ldc, batch, strideA_rows, strideW_rows, strideC,
                       workspace, workspace_bytes, static_cast<hipStream_t>(stream));
}

size_t dfp4_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    if (M < 0 || N < 0 || K < 0) return 0;
    return gemm_workspace_bytes(M, N, K);
}

size_t dfp4_gemm_prepared_bytes(int64_t rows, int64_t K, int is_weight) {
    if (rows < 0 || K < 0 || K % kBlock != 0) return 0;
    return gemm_prepared_bytes(rows, K, is_weight != 0);
}

static int gemm_prepare_common(bool mx, dfp4_tensor T, int is_weight, void* prepared, size_t bytes, void* stream) {
    if (T.rows < 0 || T.K < 0 || T.K % kBlock != 0) return DFP4_ERR_SHAPE;
    const size_t need = gemm_prepared_bytes(T.rows, T.K, is_weight != 0);
    if (need == 0) return DFP4_OK;                    // nothing to prepare: the products of this operand read it as it is
    if (!T.codes || !T.exponent || (!mx && !T.dialect)) return DFP4_ERR_NULL;
    if (!prepared || bytes < need) return DFP4_ERR_WORKSPACE;
    if (!aligned(T.codes, 16) || !aligned(prepared, 256)) return DFP4_ERR_ALIGN;
    return launch_gemm_prepare(mx, T, is_weight != 0, prepared, static_cast<hipStream_t>(stream));
}

int dfp4_gemm_prepare(dfp4_tensor T, int is_weight, void* prepared, size_t bytes, void* stream) {
    return gemm_prepare_common(false, T, is_weight, prepared, bytes, stream);
}

int mxfp4_gemm_prepare(dfp4_tensor T, int is_weight, void* prepared, size_t bytes, void* stream) {
    return gemm_prepare_common(true, T, is_weight, prepared, bytes, stream);
}

size_t dfp4_gemm_prepared_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    if (M < 0 || N < 0 || K < 0) return 0;
    return gemm_prepared_workspace_bytes(M, N, K);
}

static int gemm_prepared_common(bool mx, dfp4_tensor A, void* a_prepared, dfp4_tensor W, const void* w_prepared,
                                void* out, int out_dtype, int64_t ldc, void* workspace, size_t workspace_bytes,
                                void* stream) {
    // the checks of dfp4_gemm, with the prepared-path workspace (partial tiles only) in place of its own
    int rc = check_gemm_args(A, W, out, out_dtype, ldc, !mx, reinterpret_cast<void*>(uintptr_t{256}), ~(size_t)0);
    if (rc != DFP4_OK) return rc;
    if (A.rows == 0 || W.rows == 0) return DFP4_OK;
    if (gemm_prepared_bytes(A.rows, A.K, false) > 0 && (!a_prepared || !w_prepared)) return DFP4_ERR_NULL;   // K <= 16384
    if ((a_prepared && !aligned(a_prepared, 256)) || (w_prepared && !aligned(w_prepared, 256))) return DFP4_ERR_ALIGN;
    const size_t need = gemm_prepared_workspace_bytes(A.rows, W.rows, A.K);
    if (need > 0) {
        if (!workspace || workspace_bytes < need) return DFP4_ERR_WORKSPACE;
        if (!aligned(workspace, 256)) return DFP4_ERR_ALIGN;
    }
    return launch_gemm_prepared(mx, A, a_prepared, W, w_prepared, out, out_dtype, ldc, workspace, workspace_bytes,
                                static_cast<hipStream_t>(stream));
}

int dfp4_gemm_prepared(dfp4_tensor A, void* a_prepared, dfp4_tensor W, const void* w_prepared, void* out, int out_dtype,
                       int64_t ldc, void* workspace, size_t workspace_bytes, void* stream) {
    return gemm_prepared_common(false, A, a_prepared, W, w_prepared, out, out_dtype, ldc, workspace, workspace_bytes,
                                stream);
}

int mxfp4_gemm_prepared(dfp4_tensor A, void* a_prepared, dfp4_tensor W, const void* w_prepared, void* out,
                        int out_dtype, int64_t ldc, void* workspace, size_t workspace_bytes, void* stream) {
    return gemm_prepared_common(true, A, a_prepared, W, w_prepared, out, out_dtype, ldc, workspace, workspace_bytes,
                                stream);
}

int dfp4_gemm_declined_tiles(const void* a_prepared, int64_t M, int64_t K, uint32_t* count) {
    if (!count) return DFP4_ERR_NULL;
    *count = 0;
    if (M < 0 || K < 0 || K % kBlock != 0) return DFP4_ERR_SHAPE;
    if (gemm_prepared_bytes(M, K, false) == 0) return DFP4_OK;
    if (!a_prepared) return DFP4_ERR_NULL;
    const uint8_t* src = static_cast<const uint8_t*>(a_prepared) + gemm_prepared_declined_offset(M, K);
    if (hipMemcpy(count, src, sizeof(uint32_t), hipMemcpyDeviceToHost) != hipSuccess) {
        (void)hipGetLastError();
        return DFP4_ERR_LAUNCH;
    }
    return DFP4_OK;
}

// Native block-scaled GEMM.  w_packed == nullptr: both operands are packed into the workspace
// (A first, then W); otherwise only A is, and W comes packed (dfp4_native_pack / mxfp4_native_pack).
static int gemm_native_common(bool fp6, dfp4_tensor A, const dfp4_tensor* W, const void* w_packed, int64_t N,
                              void* out, int out_dtype, int64_t ldc, void* workspace, size_t workspace_bytes,
                              void* stream) {
    if (A.rows < 0 || N < 0 || A.K < 0 || A.K % kBlock != 0) return DFP4_ERR_SHAPE;
    if (W && (W->K != A.K || W->rows != N)) return DFP4_ERR_SHAPE;
    if (out_dtype != DFP4_F32 && out_dtype != DFP4_BF16) return DFP4_ERR_DTYPE;
    if (A.rows == 0 || N == 0) return DFP4_OK;
    if (ldc < N || A.K == 0) return DFP4_ERR_SHAPE;
    if (!out || !A.codes || !A.exponent || (fp6 && !A.dialect)) return DFP4_ERR_NULL;
    if (W && (!W->codes || !W->exponent || (fp6 && !W->dialect))) return DFP4_ERR_NULL;
    if (!W && !w_packed) return DFP4_ERR_NULL;
    if (!aligned(A.codes, 16) || (W && !aligned(W->codes, 16)) || (w_packed && !aligned(w_packed, 256)))
        return DFP4_ERR_ALIGN;
    const size_t a_bytes = native_packed_bytes(A.rows, A.K, fp6);
    const size_t w_bytes = W ? native_packed_bytes(N, A.K, fp6) : 0;
    const size_t need = a_bytes + w_bytes + native_splitk_bytes(A.rows, N, A.K);
    if (!workspace || workspace_bytes < need) return DFP4_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return DFP4_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int rc = launch_native_pack(fp6, A, workspace, a_bytes, st);
    if (rc != DFP4_OK) return rc;
    const void* wp = w_packed;
    if (W) {
        void* dst = static_cast<uint8_t*>(workspace) + a_bytes;
        rc = launch_native_pack(fp6, *W, dst, w_bytes, st);
        if (rc != DFP4_OK) return rc;
        wp = dst;
    }
    return launch_gemm_native_packed(fp6, workspace, wp, A.rows, N, A.K, out, out_dtype, ldc,
                                     static_cast<uint8_t*>(workspace) + a_bytes + w_bytes, need - a_bytes - w_bytes, st);
}

int mxfp4_gemm_native(dfp4_tensor A, dfp4_tensor W, void* out, int out_dtype, int64_t ldc, void* workspace,
                      size_t workspace_bytes, void* stream) {
    return gemm_native_common(false, A, &W, nullptr, W.rows, out, out_dtype, ldc, workspace, workspace_bytes, stream);
}

int dfp4_gemm_native(dfp4_tensor A, dfp4_tensor W, void* out, int out_dtype, int64_t ldc, void* workspace,
                     size_t workspace_bytes, void* stream) {
    return gemm_native_common(true, A, &W, nullptr, W.rows, out, out_dtype, ldc, workspace, workspace_bytes, stream);
}

int mxfp4_gemm_native_packed_w(dfp4_tensor A, const void* w_packed, int64_t N, void* out, int out_dtype,
                               int64_t ldc, void* workspace, size_t workspace_bytes, void* stream) {
    return gemm_native_common(false, A, nullptr, w_packed, N, out, out_dtype, ldc, workspace, workspace_bytes, stream);
}

int dfp4_gemm_native_packed_w(dfp4_tensor A, const void* w_packed, int64_t N, void* out, int out_dtype,
                              int64_t ldc, void* workspace, size_t workspace_bytes, void* stream) {
    return gemm_native_common(true, A, nullptr, w_packed, N, out, out_dtype, ldc, workspace, workspace_bytes, stream);
}

static int gemm_native_packed_common(bool fp6, const void* a_packed, int64_t M, const void* w_packed, int64_t N,
                                     int64_t K, void* out, int out_dtype, int64_t ldc, void* workspace,
                                     size_t workspace_bytes, void* stream) {
    if (M < 0 || N < 0 || K <= 0 || K % kBlock != 0) return DFP4_ERR_SHAPE;
    if (out_dtype != DFP4_F32 && out_dtype != DFP4_BF16) return DFP4_ERR_DTYPE;
    if (M == 0 || N == 0) return DFP4_OK;
    if (ldc < N) return DFP4_ERR_SHAPE;
    if (!out || !a_packed || !w_packed) return DFP4_ERR_NULL;
    if (!aligned(a_packed, 256) || !aligned(w_packed, 256)) return DFP4_ERR_ALIGN;
    if (workspace && !aligned(workspace, 256)) return DFP4_ERR_ALIGN;
    return launch_gemm_native_packed(fp6, a_packed, w_packed, M, N, K, out, out_dtype, ldc, workspace,
                                     workspace ? workspace_bytes : 0, static_cast<hipStream_t>(stream));
}

int dfp4_gemm_native_packed(const void* a_packed, int64_t M, const void* w_packed, int64_t N, int64_t K, void* out,
                            int out_dtype, int64_t ldc, void* workspace, size_t workspace_bytes, void* stream) {
    return gemm_native_packed_common(true, a_packed, M, w_packed, N, K, out, out_dtype, ldc, workspace,
                                     workspace_bytes, stream);
}

int mxfp4_gemm_native_packed(const void* a_packed, int64_t M, const void* w_packed, int64_t N, int64_t K, void* out,
                             int out_dtype, int64_t ldc, void* workspace, size_t workspace_bytes, void* stream) {
    return gemm_native_packed_common(false, a_packed, M, w_packed, N, K, out, out_dtype, ldc, workspace,
                                     workspace_bytes, stream);
}

size_t dfp4_gemm_native_splitk_bytes(int64_t M, int64_t N, int64_t K) {
    if (M < 0 || N < 0 || K < 0) return 0;
    return native_splitk_bytes(M, N, K);
}

static int native_pack_common(bool fp6, dfp4_tensor T, void* packed, size_t bytes, void* stream) {
    if (T.rows < 0 || T.K < 0 || T.K % kBlock != 0) return DFP4_ERR_SHAPE;
    if (T.rows == 0 || T.K == 0) return DFP4_OK;
    if (!packed || !T.codes || !T.exponent || (fp6 && !T.dialect)) return DFP4_ERR_NULL;
    if (!aligned(T.codes, 16) || !aligned(packed, 256)) return DFP4_ERR_ALIGN;
    if (bytes < native_packed_bytes(T.rows, T.K, fp6)) return DFP4_ERR_WORKSPACE;
    return launch_native_pack(fp6, T, packed, bytes, static_cast<hipStream_t>(stream));
}

int dfp4_quantize_native(const void* x_bf16, int64_t rows, int64_t K, int64_t ld_elems, void* packed, size_t bytes,
                         void* stream) {
    if (rows < 0 || K < 0 || K % kBlock != 0 || ld_elems < K) return DFP4_ERR_SHAPE;
    if (rows == 0 || K == 0) return DFP4_OK;
    if (!x_bf16 || !packed) return DFP4_ERR_NULL;
    if (ld_elems % 8 != 0 || !aligned(x_bf16, 16) || !aligned(packed, 256)) return DFP4_ERR_ALIGN;
    if (bytes < native_packed_bytes(rows, K, true)) return DFP4_ERR_WORKSPACE;
    return launch_quantize_native(x_bf16, rows, K, ld_elems, packed, native_scale_offset(rows, K, true),
                                  static_cast<hipStream_t>(stream));
}

int dfp4_native_pack(dfp4_tensor T, void* packed, size_t bytes, void* stream) {
    return native_pack_common(true, T, packed, bytes, stream);
}

int mxfp4_native_pack(dfp4_tensor T, void* packed, size_t bytes, void* stream) {
    return native_pack_common(false, T, packed, bytes, stream);
}

size_t dfp4_native_packed_bytes(int64_t rows, int64_t K) {
    if (rows < 0 || K < 0) return 0;
    return native_packed_bytes(rows, K, true);               // covers the FP4 form as well
}

size_t dfp4_gemm_native_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    if (M < 0 || N < 0 || K < 0) return 0;
    return gemm_native_workspace_bytes(M, N, K, true);       // covers the FP4 form as well
}

// out: quantized [batch * M, N] (problem after problem); A.rows = M and W.rows = N per problem
static int gemm_requant_common(bool mx, dfp4_tensor A, dfp4_tensor W, dfp4_tensor out, int64_t batch,
                               int64_t strideA_rows, int64_t strideW_rows, void* workspace, size_t workspace_bytes,
                               void* stream) {
    if (batch < 0 || strideA_rows < 0 || strideW_rows < 0) return DFP4_ERR_SHAPE;
    if (A.rows < 0 || W.rows < 0 || A.K < 0 || A.K != W.K || A.K % kBlock != 0 || W.rows % kBlock != 0 ||
        out.rows != A.rows * batch || out.K != W.rows)
        return DFP4_ERR_SHAPE;
    if (A.rows == 0 || W.rows == 0 || batch == 0) return DFP4_OK;
    if (!out.codes || !out.exponent || (!mx && !out.dialect)) return DFP4_ERR_NULL;
    if (!aligned(out.codes, 4)) return DFP4_ERR_ALIGN;
    // per problem: the plain GEMM's workspace, then the bf16 [M, N] temporaries of all problems
    const size_t gemm_ws = (size_t)((gemm_workspace_bytes(A.rows, W.rows, A.K) + 255) & ~(size_t)255) * (size_t)batch;
    const size_t temp_bytes = (size_t)(((A.rows * W.rows * 2) + 255) & ~(int64_t)255) * (size_t)batch;
    if (!workspace || workspace_bytes < gemm_ws + temp_bytes) return DFP4_ERR_WORKSPACE;
    void* temp = static_cast<uint8_t*>(workspace) + gemm_ws;
    int rc = check_gemm_args(A, W, temp, DFP4_BF16, W.rows, !mx, workspace, gemm_ws > 0 ? gemm_ws : 1);
    if (rc != DFP4_OK) return rc;
    rc = gemm_shape_check(A, W, W.rows, batch, true);
    if (rc != DFP4_OK) return rc;
    return launch_gemm(mx, A, W, temp, DFP4_BF16, W.rows, batch, strideA_rows, strideW_rows, A.rows * W.rows, workspace,
                       gemm_ws, static_cast<hipStream_t>(stream), &out);
}

int dfp4_gemm_requant(dfp4_tensor A, dfp4_tensor W, dfp4_tensor out, void* workspace, size_t workspace_bytes,
                      void* stream) {
    return gemm_requant_common(false, A, W, out, 1, 0, 0, workspace, workspace_bytes, stream);
}

int mxfp4_gemm_requant(dfp4_tensor A, dfp4_tensor W, dfp4_tensor out, void* workspace, size_t workspace_bytes,
                       void* stream) {
    return gemm_requant_common(true, A, W, out, 1, 0, 0, workspace, workspace_bytes, stream);
}

int dfp4_gemm_requant_batched(dfp4_tensor A, dfp4_tensor W, dfp4_tensor out, int64_t batch, int64_t strideA_rows,
                              int64_t strideW_rows, void* workspace, size_t workspace_bytes, void* stream) {
    return gemm_requant_common(false, A, W, out, batch, strideA_rows, strideW_rows, workspace, workspace_bytes, stream);
}

size_t dfp4_gemm_requant_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    if (M < 0 || N < 0 || K < 0) return 0;
    return gemm_requant_workspace_bytes(M, N, K);
}

int dfp4_formatbook(uint8_t* out) {
    if (!out) return DFP4_ERR_NULL;
    for (int d = 0; d < kDialects; ++d)
        for (int j = 0; j < 8; ++j) out[d * 8 + j] = kBook[d][j];
    return DFP4_OK;
}

const char* dfp4_strerror(int code) {
    switch (code) {
        case DFP4_OK: return "ok";
        case DFP4_ERR_NULL: return "null pointer";
        case DFP4_ERR_SHAPE: return "bad shape (K % 32, negative size, mismatched K, ld < K or size above limit)";
        case DFP4_ERR_ALIGN: return "misaligned pointer or leading dimension";
        case DFP4_ERR_DTYPE: return "unknown dtype";
        case DFP4_ERR_WORKSPACE: return "workspace missing or too small";
        case DFP4_ERR_LAUNCH: return "kernel launch failed";
        default: return "unknown error";
    }
}

}  // extern "C"
