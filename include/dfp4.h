/*
 * dfp4.h - C ABI of libdfp4: BlockDialect / DialectFP4 hot path on AMD MI355X (gfx950).
 *
 * The library implements, as HIP kernels, the per-block online quantizer of
 * the paper (Section 3.2: preprocessing and two-stage dialect selection;
 * Section 3.3: rounding to the selected dialect), its inverse (Section 3.3,
 * dequantization through the table of representable values) and the
 * block-scaled integer matrix multiply that consumes quantized operands
 * (Section 3.3: 4-bit integer products accumulated as integers inside a
 * block pair, one exponent sum per block pair, floating-point accumulation
 * across blocks), plus the MXFP4 format the paper compares against
 * (Section 4.1, baseline).
 *
 * Conventions for every call
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     never allocates, frees or keeps user memory and never synchronizes.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream) of the current device.
 *   - Return value: DFP4_OK (0), or a negative DFP4_ERR_* code.  Arguments, shapes and
 *     workspace sizes are checked before the first kernel is enqueued, so on any error
 *     other than DFP4_ERR_LAUNCH nothing has been enqueued; DFP4_ERR_LAUNCH (the HIP
 *     runtime refused a launch) may leave earlier kernels of the same call enqueued.
 *     dfp4_strerror() names a code.
 *   - A block is 32 consecutive elements along K (the contraction dimension,
 *     Appendix C: every operand is quantized along its multiplication
 *     dimension).  K must be a multiple of 32.
 *   - Inputs must be finite; the method does not define NaN or infinity.
 *
 * Storage of a quantized tensor [rows, K]  (Section 3.1: 1 sign bit + 3-bit
 * index per element, 4-bit dialect identifier and a shared exponent per block;
 * the byte layout is this library's choice)
 *   codes    uint8 [rows, K/2]   element 2j in bits 3:0 of byte j, element 2j+1
 *                                in bits 7:4; a 4-bit code is (sign << 3) | index,
 *                                index = ascending rank of the magnitude in the
 *                                dialect (0 -> 0.0, 7 -> largest)
 *   dialect  uint8 [rows, K/32]  dialect identifier 0..15 (absent for MXFP4)
 *   exponent uint8 [rows, K/32]  shared exponent e stored as e + 127, with
 *                                e = clamp(floor(log2(block max)) - 2, -127, 127);
 *                                an all-zero block stores 0
 *   All three arrays are dense row-major (no padding between rows).
 */
#ifndef DFP4_H
#define DFP4_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DFP4_BLOCK 32

enum {
    DFP4_OK = 0,
    DFP4_ERR_NULL = -1,       /* a required pointer is NULL */
    DFP4_ERR_SHAPE = -2,      /* K % 32 != 0, negative size, A.K != W.K, ld < K, size above limit */
    DFP4_ERR_ALIGN = -3,      /* pointer or leading dimension not aligned as documented */
    DFP4_ERR_DTYPE = -4,      /* unknown dtype selector */
    DFP4_ERR_WORKSPACE = -5,  /* workspace missing or too small */
    DFP4_ERR_LAUNCH = -6      /* the HIP runtime refused the launch */
};

enum { DFP4_F32 = 0, DFP4_BF16 = 1 };

typedef struct dfp4_tensor {
    uint8_t* codes;     /* device, [rows, K/2],  4-byte aligned */
    uint8_t* dialect;   /* device, [rows, K/32]; ignored (may be NULL) by mxfp4_* */
    uint8_t* exponent;  /* device, [rows, K/32] */
    int64_t rows;
    int64_t K;
} dfp4_tensor;

/*
 * Online DialectFP4 quantization (Section 3.2 and 3.3).
 *   x_bf16   device, bf16 [rows, K] row-major with leading dimension ld_elems
 *            (elements, >= K, multiple of 8); 16-byte aligned.
 *   out      receives codes / dialect / exponent; out.rows and out.K must equal
 *            rows and K.
 * Per block: shared exponent from the block maximum; 5-bit magnitudes
 * floor(4|x|/2^e); stage 1 picks the dialect pair whose largest value equals the
 * block maximum rounded (half up) to a multiple of 0.5 (a rounded maximum of 8.0
 * uses the 7.5 pair); stage 2 counts elements in each dialect's beneficial
 * range, the larger count wins and the even dialect wins ties; each element
 * takes the index of the nearest value of the chosen dialect, halfway cases
 * going to the larger value.  rows == 0 is a no-op.
 */
int dfp4_quantize(const void* x_bf16, int64_t rows, int64_t K, int64_t ld_elems,
                  dfp4_tensor out, void* stream);

/*
 * DialectFP4 with blocks of 64 elements (Section 4.2, Table 3 varies the block size): one shared
 * exponent and one dialect per 64 consecutive elements along K (K a multiple of 64), chosen
 * by the same steps from all 64.  The output keeps the layout of the 32-element format --
 * the exponent byte and the dialect id of a block are written for both of its halves -- so
 * dfp4_dequantize and every GEMM entry point consume it unchanged.
 */
int dfp4_quantize_b64(const void* x_bf16, int64_t rows, int64_t K, int64_t ld_elems,
                      dfp4_tensor out, void* stream);

/*
 * Block size as an argument (Section 4.2, Table 3: blocks of 16, 32 or 64, and smaller blocks for
 * only the sublayers most sensitive to quantization, so that operands of one model -- and the
 * two operands of one product -- may use different sizes).  block_size is 16, 32 or 64.
 *   32   as dfp4_quantize / dfp4_dequantize / dfp4_gemm
 *   64   as dfp4_quantize_b64: stored in the 32-element layout (K a multiple of 64)
 *   16   one shared exponent and one dialect per 16 consecutive elements, chosen by the same
 *        steps from those 16: the tensor's dialect and exponent arrays are [rows, K/16]
 *        (codes unchanged); K must still be a multiple of 32
 * dfp4_gemm_blocks multiplies operands of any two block sizes.  Where either is 16 the product is
 * computed as the paper's MAC states it, one fp32 scale-and-add per pair of 16-element blocks
 * (the exact single-accumulator path needs one exponent per 32 elements; this path runs at about a
 * tenth of its rate and needs no workspace); otherwise the call is dfp4_gemm.
 */
int dfp4_quantize_block(const void* x_bf16, int64_t rows, int64_t K, int64_t ld_elems, int block_size,
                        dfp4_tensor out, void* stream);
int dfp4_dequantize_block(dfp4_tensor in, int block_size, void* y, int y_dtype, int64_t ld_elems, void* stream);
int dfp4_gemm_blocks(dfp4_tensor A, int block_a, dfp4_tensor W, int block_w, void* out, int out_dtype,
                     int64_t ldc, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Transposing quantizers (Appendix C: every operand is blocked along the dimension
 * it is multiplied over): x [rows, cols] row-major (leading dimension ld_elems) is
 * quantized in blocks of 32 along its ROWS; `out` is the quantized transpose,
 * out.rows = cols, out.K = rows, bit-identical to dfp4_quantize / mxfp4_quantize
 * applied to x^T.  For V of the attention product P V: stored [sequence, head
 * dim], contracted over the sequence.  rows must be a multiple of 32, cols and
 * ld_elems multiples of 8, x 16-byte aligned.
 */
int dfp4_quantize_t(const void* x_bf16, int64_t rows, int64_t cols, int64_t ld_elems,
                    dfp4_tensor out, void* stream);
int mxfp4_quantize_t(const void* x_bf16, int64_t rows, int64_t cols, int64_t ld_elems,
                     dfp4_tensor out, void* stream);
/*
 * The same into a longer tensor (Appendix C, value cache: values are stored in 4-bit chunks
 * of one block of tokens; only the most recent, incomplete chunk stays in high precision and
 * is quantized once it holds 32 tokens): x holds `rows` consecutive tokens (a multiple of 32)
 * starting at token `row_offset` (a multiple of 32); `out` is the quantized transpose of the
 * whole sequence, out.rows = cols, out.K = capacity in tokens >= row_offset + rows.  Only the
 * blocks of these tokens are written.
 */
int dfp4_quantize_t_at(const void* x_bf16, int64_t rows, int64_t cols, int64_t ld_elems,
                       dfp4_tensor out, int64_t row_offset, void* stream);

/*
 * Offline DialectFP4 quantization with MSE-based dialect selection (Section 3.2:
 * for tensors known in advance, such as weights, the best dialect of a block is
 * found by computing the squared error of every dialect).  Arguments, layouts,
 * shared exponent and element rounding as dfp4_quantize; the block's dialect is
 * the one whose 32 rounded values have the smallest sum of squared errors, the
 * lowest id among equal sums.  Not meant for the online path: it does 16 rounds
 * of quantization per block.
 */
int dfp4_quantize_mse(const void* x_bf16, int64_t rows, int64_t K, int64_t ld_elems,
                      dfp4_tensor out, void* stream);

/*
 * Dequantization (Section 3.3): y[r, k] = (-1)^sign * 0.5 * u[dialect][index] * 2^e.
 *   y        device, [rows, K] with leading dimension ld_elems (>= K, multiple of 8),
 *            16-byte aligned; y_dtype selects DFP4_F32 or DFP4_BF16 (both exact).
 */
int dfp4_dequantize(dfp4_tensor in, void* y, int y_dtype, int64_t ld_elems, void* stream);

/*
 * Block-scaled matrix multiply (Section 3.3): out = A * W^T,
 *   out[m, n] = sum over blocks kb of 2^(ea[m,kb] + ew[n,kb] - 2) *
 *               sum over k in kb of (+-ua[m,k]) * (+-uw[n,k])
 * with u the 4-bit unsigned integers (half-units) the codes index.  The inner
 * sums run on the int8 matrix cores with int32 accumulation and are exact.
 * Where the block exponents of a tile span at most 12 binades per row the
 * outer sum is exact as well (exponent offsets folded into the int8 operands,
 * one conversion to fp32 at the end); otherwise it is accumulated in fp32,
 * one addition per block.  That slower per-block path also takes every product
 * with K > 16384 and, at its own pace, every product with M <= 64 (few rows);
 * 512 x 128 output tiles whose exponents spread further are computed that way by
 * the workgroup that finds them (dfp4_gemm_declined_tiles counts them).
 *   A        quantized [M, K]; W quantized [N, K] (both blocked along K)
 *   out      device, [M, N] row-major, leading dimension ldc (elements, N <= ldc < 2^27);
 *            out_dtype DFP4_F32 or DFP4_BF16 (round to nearest even)
 *   workspace, workspace_bytes   device scratch of at least
 *            dfp4_gemm_workspace_bytes(M, N, K) bytes, 256-byte aligned; may be
 *            NULL when that size is 0.  Contents are undefined afterwards.
 * M == 0 or N == 0 is a no-op.
 */
int dfp4_gemm(dfp4_tensor A, dfp4_tensor W, void* out, int out_dtype, int64_t ldc,
              void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same product for `batch` independent problems of equal shape (attention
 * score and context matmuls, Appendix C).  Problem b uses
 *   A.codes + b * strideA_rows * K/2, A.dialect/exponent + b * strideA_rows * K/32
 * (and likewise W with strideW_rows), and out + b * strideC elements.
 * A.rows = M and W.rows = N are the per-problem sizes.
 *   workspace   at least batch * dfp4_gemm_workspace_bytes(M, N, K) bytes.
 */
int dfp4_gemm_batched(dfp4_tensor A, dfp4_tensor W, void* out, int out_dtype, int64_t ldc,
                      int64_t batch, int64_t strideA_rows, int64_t strideW_rows, int64_t strideC,
                      void* workspace, size_t workspace_bytes, void* stream);

size_t dfp4_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);

/*
 * The same product with the per-operand work of dfp4_gemm done ahead (Section 3.3: the cost
 * of preparing a quantized activation block is amortized over the many weight blocks it is
 * multiplied with; weights are known in advance).  dfp4_gemm spends part of every call on
 * each operand alone: per-row reference exponents, per-block tables, and for A the 4-bit
 * codes expanded through the dialect tables to the int8 operands of the matrix cores.
 * dfp4_gemm_prepare does that once per tensor:
 *   is_weight != 0   T is a W operand [N, K] (offline, once per weight matrix)
 *   is_weight == 0   T is an A operand [M, K] (online, once per activation tensor, however
 *                    many products consume it: gate and up projections share one)
 *   prepared         device, 256-byte aligned, at least dfp4_gemm_prepared_bytes(rows, K,
 *                    is_weight) bytes; the layout is private to the library (for a weight:
 *                    a copy of the codes and three table words per block, both in the order
 *                    the kernels read them, about 0.9 bytes per element).  A size of 0
 *                    means nothing is prepared for this operand (K > 16384): NULL may be
 *                    passed then.
 * dfp4_gemm_prepared multiplies.  The quantized tensors are still passed: paths that do not
 * use the prepared form read them.  a_prepared is written to (arrival counters of tiles
 * whose K is split between workgroups), so one prepared A serves one product at a time:
 * products on one stream are ordered by the stream, products that may overlap in time need
 * their own prepared copy.  Results are bit-identical to dfp4_gemm, except possibly for
 * products with at most 64 rows of A: there both take the exact scheme (one rounding of the
 * exact sum) where the exponents allow it, but dfp4_gemm decides that per 32 x 32 output
 * tile from the tile's own rows, and a tile it cannot take gets one fp32 term per block.
 *   workspace   at least dfp4_gemm_prepared_workspace_bytes(M, N, K) bytes (partial tiles
 *               where K is split; 0 for products with many output tiles), 256-byte aligned
 * Limits: ceil(rows / 512) * (K/32 + 1) * 49152 < 2^31 for A, rows * K / 2 < 2^31 for W
 * (DFP4_ERR_SHAPE; dfp4_gemm itself cuts larger products into pieces).
 */
size_t dfp4_gemm_prepared_bytes(int64_t rows, int64_t K, int is_weight);
int dfp4_gemm_prepare(dfp4_tensor T, int is_weight, void* prepared, size_t bytes, void* stream);
int mxfp4_gemm_prepare(dfp4_tensor T, int is_weight, void* prepared, size_t bytes, void* stream);
size_t dfp4_gemm_prepared_workspace_bytes(int64_t M, int64_t N, int64_t K);
int dfp4_gemm_prepared(dfp4_tensor A, void* a_prepared, dfp4_tensor W, const void* w_prepared, void* out,
                       int out_dtype, int64_t ldc, void* workspace, size_t workspace_bytes, void* stream);
int mxfp4_gemm_prepared(dfp4_tensor A, void* a_prepared, dfp4_tensor W, const void* w_prepared, void* out,
                        int out_dtype, int64_t ldc, void* workspace, size_t workspace_bytes, void* stream);
/*
 * Diagnostic: number of 512 x 128 output tiles that products on this prepared A ([M, K]) have
 * computed on the per-block fp32 path since it was prepared (exponent spread beyond what the
 * exact path folds into its operands).  `count` is a HOST pointer.  Synchronizes with the device.
 */
int dfp4_gemm_declined_tiles(const void* a_prepared, int64_t M, int64_t K, uint32_t* count);

/*
 * dfp4_gemm for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same product,
 * same kernels and bit-identical results; the workspace is an array of
 * DFP4_NOALLOC_SCRATCH_BYTES that is part of the library's device code (each GPU the
 * library runs on holds its own copy until the process ends).  The call allocates and
 * frees nothing.  Products with dfp4_gemm_workspace_bytes(M, N, K) above that size are
 * refused with DFP4_ERR_WORKSPACE (64 MiB covers M = 2048, N = 14336, K = 4096).
 * All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU
 * (different streams, different threads) race and must be ordered by the caller; calls on
 * one stream are ordered by the stream.  Every call initializes what it reads, so nothing
 * carries over from one call to the next.
 */
#define DFP4_NOALLOC_SCRATCH_BYTES (64 << 20)
int dfp4_gemm_noalloc(dfp4_tensor A, dfp4_tensor W, void* out, int out_dtype, int64_t ldc, void* stream);

/*
 * Matrix multiply on the block-scaled matrix instruction of the GPU
 * (v_mfma_scale_f32_32x32x64_f8f6f4): out = A * W^T as dfp4_gemm / mxfp4_gemm, but
 * with the power-of-two block scales applied and the sum accumulated in fp32 by
 * the hardware.  dfp4_gemm_native repacks the DialectFP4 operands to FP6 E2M3,
 * in which every DialectFP4 value is exact; mxfp4_gemm_native uses the MXFP4
 * codes as they are (FP4 E2M1).  The exponent bytes are the scales (E8M0).
 * Results agree with dfp4_gemm / mxfp4_gemm within the rounding of fp32
 * accumulation (the tolerance of the parity tests), not bit for bit.
 *   workspace   at least dfp4_gemm_native_workspace_bytes(M, N, K) bytes, 256-byte
 *            aligned: both operands in the instruction's register order
 */
int dfp4_gemm_native(dfp4_tensor A, dfp4_tensor W, void* out, int out_dtype, int64_t ldc,
                     void* workspace, size_t workspace_bytes, void* stream);
int mxfp4_gemm_native(dfp4_tensor A, dfp4_tensor W, void* out, int out_dtype, int64_t ldc,
                      void* workspace, size_t workspace_bytes, void* stream);
size_t dfp4_gemm_native_workspace_bytes(int64_t M, int64_t N, int64_t K);

/*
 * The same with W arranged in the instruction's register order beforehand (weights:
 * once, offline).  dfp4_native_pack / mxfp4_native_pack write the packed form of a
 * quantized [rows, K] tensor into `packed` (device, 256-byte aligned, at least
 * dfp4_native_packed_bytes(rows, K) bytes; the layout is private to the library).
 * The *_packed_w calls take A quantized and W packed (N = number of rows of W); their
 * workspace holds the packed A and, where K is split between workgroups (few output
 * tiles), their fp32 partial tiles: dfp4_native_packed_bytes(M, K) +
 * dfp4_gemm_native_splitk_bytes(M, N, K) bytes.
 */
size_t dfp4_native_packed_bytes(int64_t rows, int64_t K);
/* Online DialectFP4 quantization (as dfp4_quantize) straight into the packed form: equal to
 * dfp4_quantize followed by dfp4_native_pack, except that the layout's padding rows are left
 * untouched (they only reach outputs that are never stored).  x as for dfp4_quantize. */
int dfp4_quantize_native(const void* x_bf16, int64_t rows, int64_t K, int64_t ld_elems, void* packed,
                         size_t bytes, void* stream);
int dfp4_native_pack(dfp4_tensor T, void* packed, size_t bytes, void* stream);
int mxfp4_native_pack(dfp4_tensor T, void* packed, size_t bytes, void* stream);
int dfp4_gemm_native_packed_w(dfp4_tensor A, const void* w_packed, int64_t N, void* out, int out_dtype,
                              int64_t ldc, void* workspace, size_t workspace_bytes, void* stream);
int mxfp4_gemm_native_packed_w(dfp4_tensor A, const void* w_packed, int64_t N, void* out, int out_dtype,
                               int64_t ldc, void* workspace, size_t workspace_bytes, void* stream);
/* Both operands packed beforehand ([M, K] and [N, K] before packing).  An activation that
 * feeds several products (gate and up projections) is packed once.  workspace: at least
 * dfp4_gemm_native_splitk_bytes(M, N, K) bytes (0 for most shapes), or NULL: then K is never
 * split, whatever the number of tiles. */
int dfp4_gemm_native_packed(const void* a_packed, int64_t M, const void* w_packed, int64_t N, int64_t K,
                            void* out, int out_dtype, int64_t ldc, void* workspace,
                            size_t workspace_bytes, void* stream);
int mxfp4_gemm_native_packed(const void* a_packed, int64_t M, const void* w_packed, int64_t N, int64_t K,
                             void* out, int out_dtype, int64_t ldc, void* workspace,
                             size_t workspace_bytes, void* stream);
size_t dfp4_gemm_native_splitk_bytes(int64_t M, int64_t N, int64_t K);

/*
 * Matrix multiply with requantizing epilogue (Section 3.3: the result of a
 * multiplication is quantized again when it feeds the next one):
 *   out = quantize(bf16(A * W^T))   in blocks of 32 along N,
 * bit-identical to dfp4_gemm with DFP4_BF16 output followed by dfp4_quantize
 * (mxfp4_gemm / mxfp4_quantize for the MXFP4 variant), without the bf16 [M, N]
 * round trip through memory for tiles the single-accumulator kernel computes.
 *   out      quantized [M, N]: out.rows = A.rows, out.K = W.rows (a multiple of 32)
 *   workspace   at least dfp4_gemm_requant_workspace_bytes(M, N, K) bytes, 256-byte
 *            aligned (it includes a bf16 [M, N] temporary used by the paths that
 *            are not fused: few rows, split K, declined tiles)
 */
int dfp4_gemm_requant(dfp4_tensor A, dfp4_tensor W, dfp4_tensor out, void* workspace,
                      size_t workspace_bytes, void* stream);
int mxfp4_gemm_requant(dfp4_tensor A, dfp4_tensor W, dfp4_tensor out, void* workspace,
                       size_t workspace_bytes, void* stream);
size_t dfp4_gemm_requant_workspace_bytes(int64_t M, int64_t N, int64_t K);
/*
 * The same for `batch` independent problems of equal shape (Appendix C: the attention products
 * are quantized along their multiplication dimensions too, so the scores Q K^T feed the next
 * product as a quantized tensor).  Problem b reads A and W as dfp4_gemm_batched does; `out` is
 * the quantized [batch * M, N] result, problem after problem (out.rows = batch * M, out.K = N).
 *   workspace   at least batch * dfp4_gemm_requant_workspace_bytes(M, N, K) bytes
 */
int dfp4_gemm_requant_batched(dfp4_tensor A, dfp4_tensor W, dfp4_tensor out, int64_t batch, int64_t strideA_rows,
                              int64_t strideW_rows, void* workspace, size_t workspace_bytes, void* stream);

/*
 * MXFP4 comparison path (Section 4.1, baseline): FP4 E2M1 elements
 * {0, 0.5, 1, 1.5, 2, 3, 4, 6} with the same shared exponent; elements are
 * rounded to nearest, ties to the even code, magnitudes above 6 saturate.
 * Same layouts; the dialect member of dfp4_tensor is ignored.
 */
int mxfp4_quantize(const void* x_bf16, int64_t rows, int64_t K, int64_t ld_elems,
                   dfp4_tensor out, void* stream);
int mxfp4_dequantize(dfp4_tensor in, void* y, int y_dtype, int64_t ld_elems, void* stream);
int mxfp4_gemm(dfp4_tensor A, dfp4_tensor W, void* out, int out_dtype, int64_t ldc,
               void* workspace, size_t workspace_bytes, void* stream);

/*
 * The formatbook in use (Section 3.1): out[d * 8 + i] = half-unit magnitude
 * (value = 0.5 * out[...]) of index i in dialect d, ascending.  `out` is a HOST
 * pointer to 128 bytes.
 */
int dfp4_formatbook(uint8_t* out);

const char* dfp4_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* DFP4_H */
