// Block-scaled integer GEMM on DialectFP4 / MXFP4 operands for gfx950
// (paper Section 3.3): out = A * W^T with
//   out[m,n] = sum_kb 2^(ea[m,kb]+ew[n,kb]-2) * sum_{k in kb} (+-ua)(+-uw).
// The inner sum over one block of 32 is exactly one v_mfma_i32_32x32x32_i8:
// 4-bit codes are expanded to signed int8 half-units through the dialect's
// 8-entry table (v_perm_b32 = four lookups per instruction), the int32 block
// sums are exact, and each is scaled by its exponent pair and added in fp32.
//
// The order of the 32 elements inside an MFMA operand does not matter as
// long as A and W use the same order; both go through unpack16() below.
#include "common.h"
#include "formatbook.h"

namespace dfp4 {

// book rows as two dwords of magnitudes and two dwords of negated magnitudes
struct SignedBook { uint32_t pos[kDialects][2]; uint32_t neg[kDialects][2]; };
constexpr SignedBook make_signed_book() {
    SignedBook b{};
    for (int d = 0; d < kDialects; ++d)
        for (int j = 0; j < 8; ++j) {
            b.pos[d][j / 4] |= (uint32_t)kBook[d][j] << (8 * (j % 4));
            b.neg[d][j / 4] |= (uint32_t)((256 - kBook[d][j]) & 0xff) << (8 * (j % 4));
        }
    return b;
}
__device__ const SignedBook g_signed_book = make_signed_book();

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kTileM = 128, kTileN = 128;

// 8 codes (one dword) -> 8 signed int8: returns {even elements, odd elements}
__device__ __forceinline__ void unpack8(uint32_t c, uint32_t plo, uint32_t phi, uint32_t nlo,
                                        uint32_t nhi, uint32_t& even, uint32_t& odd) {
    const uint32_t ie = c & 0x07070707u, io = (c >> 4) & 0x07070707u;
    const uint32_t pe = __builtin_amdgcn_perm(phi, plo, ie), po = __builtin_amdgcn_perm(phi, plo, io);
    const uint32_t ne = __builtin_amdgcn_perm(nhi, nlo, ie), no = __builtin_amdgcn_perm(nhi, nlo, io);
    const uint32_t se = (c >> 3) & 0x01010101u, so = (c >> 7) & 0x01010101u;
    const uint32_t me = (se << 8) - se, mo = (so << 8) - so;      // 0xff per negative byte
    even = (ne & me) | (pe & ~me);
    odd = (no & mo) | (po & ~mo);
}

__device__ __forceinline__ v4i unpack16(uint2 c, uint32_t d) {
    const uint32_t plo = g_signed_book.pos[d][0], phi = g_signed_book.pos[d][1];
    const uint32_t nlo = g_signed_book.neg[d][0], nhi = g_signed_book.neg[d][1];
    uint32_t a, b, e, f;
    unpack8(c.x, plo, phi, nlo, nhi, a, b);
    unpack8(c.y, plo, phi, nlo, nhi, e, f);
    return v4i{(int)a, (int)b, (int)e, (int)f};
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Reference-quality kernel: one workgroup = 128 x 128 outputs, 4 waves of 64 x 64,
// operands read straight from global memory, one flush per block of 32.
template <bool MX, bool BF16>
__global__ __launch_bounds__(kThreads) void gemm_block_kernel(
    const uint8_t* __restrict__ a_codes, const uint8_t* __restrict__ a_dial,
    const uint8_t* __restrict__ a_exp, const uint8_t* __restrict__ w_codes,
    const uint8_t* __restrict__ w_dial, const uint8_t* __restrict__ w_exp, void* __restrict__ out,
    int M, int N, int KB, int64_t ldc, int64_t strideA_rows, int64_t strideW_rows, int64_t strideC) {
    __shared__ uint8_t s_exp[2][kTileM + kTileN];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * kTileM, n0 = blockIdx.x * kTileN;
    const int64_t bz = blockIdx.z;
    const int64_t a_row0 = bz * strideA_rows, w_row0 = bz * strideW_rows;
    const int half = lane >> 5, l32 = lane & 31;

    int64_t a_row[2], w_row[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        a_row[i] = a_row0 + min(m0 + wm * 64 + i * 32 + l32, M - 1);
        w_row[i] = w_row0 + min(n0 + wn * 64 + i * 32 + l32, N - 1);
    }
    // exponent staging: thread t < 128 fetches an A row's byte, t >= 128 a W row's byte
    const int t = threadIdx.x;
    const int64_t e_row = t < kTileM ? a_row0 + min(m0 + t, M - 1) : w_row0 + min(n0 + t - kTileM, N - 1);
    const uint8_t* e_src = (t < kTileM ? a_exp : w_exp) + e_row * KB;

    float acc[2][2][16];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    for (int kb = 0; kb < KB; ++kb) {
        uint8_t* se = s_exp[kb & 1];
        se[t] = e_src[kb];
        v4i a[2], b[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uint2 ca = *reinterpret_cast<const uint2*>(a_codes + (a_row[i] * KB + kb) * 16 + half * 8);
            const uint2 cw = *reinterpret_cast<const uint2*>(w_codes + (w_row[i] * KB + kb) * 16 + half * 8);
            const uint32_t da = MX ? 7u : ((uint32_t)a_dial[a_row[i] * KB + kb] & 15u);
            const uint32_t dw = MX ? 7u : ((uint32_t)w_dial[w_row[i] * KB + kb] & 15u);
            a[i] = unpack16(ca, da);
            b[i] = unpack16(cw, dw);
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                v16i p = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                p = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], p, 0, 0, 0);
                const int ew = se[kTileM + wn * 64 + j * 32 + l32];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = 8 * (r >> 2) + 4 * half + (r & 3);
                    const int ea = se[wm * 64 + i * 32 + row];
                    acc[i][j][r] += ldexpf((float)p[r], ea + ew - 256);
                }
            }
    }

#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + wn * 64 + j * 32 + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                if (m < M && n < N) {
                    const int64_t o = bz * strideC + (int64_t)m * ldc + n;
                    if constexpr (BF16)
                        static_cast<uint16_t*>(out)[o] = f32_to_bf16_rne(acc[i][j][r]);
                    else
                        static_cast<float*>(out)[o] = acc[i][j][r];
                }
            }
        }
}

}  // namespace

size_t gemm_workspace_bytes(int64_t, int64_t, int64_t) { return 0; }

int launch_gemm(bool mx, dfp4_tensor A, dfp4_tensor W, void* out, int out_dtype, int64_t ldc,
                int64_t batch, int64_t strideA_rows, int64_t strideW_rows, int64_t strideC,
                void* /*workspace*/, size_t /*workspace_bytes*/, hipStream_t stream) {
    const int64_t M = A.rows, N = W.rows, KB = A.K / kBlock;
    if (M == 0 || N == 0 || batch == 0) return DFP4_OK;
    if (M >= (1 << 30) || N >= (1 << 30) || KB >= (1 << 26) || batch > 65535) return DFP4_ERR_SHAPE;
    dim3 grid((unsigned)((N + kTileN - 1) / kTileN), (unsigned)((M + kTileM - 1) / kTileM), (unsigned)batch);
    if (grid.y > 65535) return DFP4_ERR_SHAPE;
#define DFP4_LAUNCH(MXV, BV)                                                                        \
    hipLaunchKernelGGL((gemm_block_kernel<MXV, BV>), grid, dim3(kThreads), 0, stream, A.codes,      \
                       A.dialect, A.exponent, W.codes, W.dialect, W.exponent, out, (int)M, (int)N,  \
                       (int)KB, ldc, strideA_rows, strideW_rows, strideC)
    if (mx) {
        if (out_dtype == DFP4_BF16) DFP4_LAUNCH(true, true); else DFP4_LAUNCH(true, false);
    } else {
        if (out_dtype == DFP4_BF16) DFP4_LAUNCH(false, true); else DFP4_LAUNCH(false, false);
    }
#undef DFP4_LAUNCH
    return check_launch();
}

}  // namespace dfp4
