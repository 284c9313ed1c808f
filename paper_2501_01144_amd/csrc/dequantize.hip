// DialectFP4 / MXFP4 dequantizer for gfx950 (paper Section 3.3, Figure 6):
// 3-bit index -> 4-bit unsigned integer u through the dialect's table,
// value = (-1)^sign * u * 2^(e-1).  One lane expands one dword of codes
// (8 elements); the dialect's 8 table bytes sit in two registers and
// v_perm_b32 does four lookups per instruction.  Both output types hold the
// values exactly (u has 4 significant bits).
#include "common.h"
#include "formatbook.h"

namespace dfp4 {

static_assert(kBook[7][6] == kE2M1[6] && kBook[7][7] == kE2M1[7] && kBook[7][5] == kE2M1[5],
              "MXFP4 dequantization reuses dialect 7 (FP4 E2M1)");

// book rows packed as two little-endian dwords each
struct BookWords { uint32_t w[kDialects][2]; };
constexpr BookWords make_book_words() {
    BookWords b{};
    for (int d = 0; d < kDialects; ++d)
        for (int j = 0; j < 8; ++j) b.w[d][j / 4] |= (uint32_t)kBook[d][j] << (8 * (j % 4));
    return b;
}
__device__ const BookWords g_book_words = make_book_words();

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ uint32_t as_u(float f) { return __builtin_bit_cast(uint32_t, f); }

template <bool MX, bool BF16, bool CONTIG>
__global__ __launch_bounds__(kThreads) void dequantize_kernel(
    const uint32_t* __restrict__ codes, const uint8_t* __restrict__ dialect,
    const uint8_t* __restrict__ exponent, void* __restrict__ y, int64_t ld, uint32_t blocks_per_row,
    uint32_t nblocks, uint32_t narrow /* 1: one exponent byte and dialect id per 16 elements */) {
    const uint64_t nlanes = (uint64_t)nblocks * 4u;
    const uint64_t stride = (uint64_t)gridDim.x * kThreads;
    for (uint64_t g = (uint64_t)blockIdx.x * kThreads + threadIdx.x; g < nlanes; g += stride) {
        const uint32_t b = (uint32_t)(g >> 2), sub = (uint32_t)(g & 3u);
        const uint32_t c = codes[g];
        const size_t mb = narrow ? (size_t)b * 2u + (sub >> 1) : (size_t)b;
        const int e = (int)exponent[mb] - 128;             // 0.5 u 2^(byte-127) = u 2^(byte-128)
        const uint32_t d = MX ? 7u : ((uint32_t)dialect[mb] & 15u);
        const uint32_t lo = g_book_words.w[d][0], hi = g_book_words.w[d][1];
        const uint32_t mag_even = __builtin_amdgcn_perm(hi, lo, c & 0x07070707u);
        const uint32_t mag_odd = __builtin_amdgcn_perm(hi, lo, (c >> 4) & 0x07070707u);
        uint32_t v[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t ue = (mag_even >> (8 * j)) & 0xffu, uo = (mag_odd >> (8 * j)) & 0xffu;
            v[2 * j] = as_u(ldexpf((float)ue, e)) | ((c << (28 - 8 * j)) & 0x80000000u);
            v[2 * j + 1] = as_u(ldexpf((float)uo, e)) | ((c << (24 - 8 * j)) & 0x80000000u);
        }
        int64_t off;
        if constexpr (CONTIG) {
            off = (int64_t)b * kBlock + sub * 8;
        } else {
            const uint32_t row = b / blocks_per_row;
            off = (int64_t)row * ld + (int64_t)(b - row * blocks_per_row) * kBlock + sub * 8;
        }
        if constexpr (BF16) {
            uint4 o;
            o.x = (v[0] >> 16) | (v[1] & 0xffff0000u);
            o.y = (v[2] >> 16) | (v[3] & 0xffff0000u);
            o.z = (v[4] >> 16) | (v[5] & 0xffff0000u);
            o.w = (v[6] >> 16) | (v[7] & 0xffff0000u);
            *reinterpret_cast<uint4*>(static_cast<uint16_t*>(y) + off) = o;
        } else {
            uint4* p = reinterpret_cast<uint4*>(static_cast<float*>(y) + off);
            p[0] = make_uint4(v[0], v[1], v[2], v[3]);
            p[1] = make_uint4(v[4], v[5], v[6], v[7]);
        }
    }
}

}  // namespace

int launch_dequantize(bool mx, dfp4_tensor in, void* y, int y_dtype, int64_t ld, hipStream_t stream, bool narrow) {
    const int64_t nblocks64 = in.rows * (in.K / kBlock);
    if (nblocks64 == 0) return DFP4_OK;
    if (nblocks64 >= (int64_t)1 << 31) return DFP4_ERR_SHAPE;
    const uint32_t nblocks = (uint32_t)nblocks64;
    const uint64_t nlanes = (uint64_t)nblocks * 4u;
    const uint64_t want = (nlanes + kThreads - 1) / kThreads;
    const uint64_t cap = (uint64_t)device_cu_count() * 16u;
    const uint32_t grid = (uint32_t)(want < cap ? want : cap);
    const bool contig = (ld == in.K);
    const uint32_t kb = (uint32_t)(in.K / kBlock);
    const uint32_t* cp = reinterpret_cast<const uint32_t*>(in.codes);
#define DFP4_LAUNCH(MXV, BV, CV)                                                                  \
    hipLaunchKernelGGL((dequantize_kernel<MXV, BV, CV>), dim3(grid), dim3(kThreads), 0, stream, cp, \
                       in.dialect, in.exponent, y, ld, kb, nblocks, narrow ? 1u : 0u)
#define DFP4_PICK(MXV)                                                             \
    do {                                                                           \
        if (y_dtype == DFP4_BF16) {                                                \
            if (contig) DFP4_LAUNCH(MXV, true, true); else DFP4_LAUNCH(MXV, true, false);   \
        } else {                                                                   \
            if (contig) DFP4_LAUNCH(MXV, false, true); else DFP4_LAUNCH(MXV, false, false); \
        }                                                                          \
    } while (0)
    if (mx) DFP4_PICK(true); else DFP4_PICK(false);
#undef DFP4_PICK
#undef DFP4_LAUNCH
    return check_launch();
}

}  // namespace dfp4
