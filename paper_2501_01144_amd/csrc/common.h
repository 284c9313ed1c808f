// Shared host-side helpers of libdfp4 (argument checks, device properties).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/dfp4.h"

namespace dfp4 {

// Number of compute units of the current device (cached per device).
int device_cu_count();

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

inline int check_launch() {
    return hipGetLastError() == hipSuccess ? DFP4_OK : DFP4_ERR_LAUNCH;
}

// Argument checks shared by the quantize / dequantize entry points.
int check_quant_args(const void* dense, int64_t rows, int64_t K, int64_t ld, const dfp4_tensor& q,
                     bool need_dialect);

// kernels (defined in the .hip files)
int launch_quantize(bool mx, const void* x, int64_t rows, int64_t K, int64_t ld, dfp4_tensor out,
                    hipStream_t stream, bool wide = false, bool narrow = false);
int launch_quantize_t(bool mx, const void* x, int64_t rows, int64_t cols, int64_t ld, dfp4_tensor out,
                      int64_t row_offset, hipStream_t stream);
int launch_quantize_native(const void* x, int64_t rows, int64_t K, int64_t ld, void* packed, size_t sc_offset,
                           hipStream_t stream);
size_t native_scale_offset(int64_t rows, int64_t K, bool fp6);
int launch_quantize_mse(const void* x, int64_t rows, int64_t K, int64_t ld, dfp4_tensor out, hipStream_t stream);
int launch_dequantize(bool mx, dfp4_tensor in, void* y, int y_dtype, int64_t ld, hipStream_t stream, bool narrow = false);
int launch_gemm_block16(dfp4_tensor A, bool a16, dfp4_tensor W, bool w16, void* out, int out_dtype, int64_t ldc,
                        hipStream_t stream);
int launch_gemm(bool mx, dfp4_tensor A, dfp4_tensor W, void* out, int out_dtype, int64_t ldc,
                int64_t batch, int64_t strideA_rows, int64_t strideW_rows, int64_t strideC,
                void* workspace, size_t workspace_bytes, hipStream_t stream, const dfp4_tensor* rq = nullptr);
size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);
int gemm_shape_check(dfp4_tensor A, dfp4_tensor W, int64_t ldc, int64_t batch, bool rq);
size_t gemm_prepared_bytes(int64_t rows, int64_t K, bool weight);
size_t gemm_prepared_workspace_bytes(int64_t M, int64_t N, int64_t K);
size_t gemm_prepared_declined_offset(int64_t M, int64_t K);
int launch_gemm_prepare(bool mx, dfp4_tensor T, bool weight, void* prepared, hipStream_t stream);
int launch_gemm_prepared(bool mx, dfp4_tensor A, void* a_prepared, dfp4_tensor W, const void* w_prepared, void* out,
                         int out_dtype, int64_t ldc, void* workspace, size_t workspace_bytes, hipStream_t stream);
size_t gemm_requant_workspace_bytes(int64_t M, int64_t N, int64_t K);
size_t native_packed_bytes(int64_t rows, int64_t K, bool fp6);
size_t gemm_native_workspace_bytes(int64_t M, int64_t N, int64_t K, bool fp6);
int launch_native_pack(bool fp6, dfp4_tensor T, void* packed, size_t bytes, hipStream_t stream);
int launch_gemm_native_packed(bool fp6, const void* a_packed, const void* w_packed, int64_t M, int64_t N, int64_t K,
                              void* out, int out_dtype, int64_t ldc, void* splitk, size_t splitk_bytes,
                              hipStream_t stream);
size_t native_splitk_bytes(int64_t M, int64_t N, int64_t K);

}  // namespace dfp4
