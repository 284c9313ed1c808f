// DialectFP4 values in the FP6 E2M3 operand format of the block-scaled matrix instruction,
// and the layout of a packed operand (see gemm_native.hip).  Shared by the packing kernel and
// by the quantizer that writes the packed form directly.
#pragma once
#include "common.h"
#include "formatbook.h"

namespace dfp4 {
namespace {

// E2M3 bit pattern of the magnitude 0.5 u, u = 0..15 (all exact: step 1/8 below 1, 1/4 below 4, 1/2 below 8)
constexpr uint8_t e2m3_of_half_units(int u) {
    return u < 2 ? (uint8_t)(4 * u) : u < 4 ? (uint8_t)(8 + 4 * (u - 2)) : u < 8 ? (uint8_t)(16 + 2 * (u - 4))
                                                                                 : (uint8_t)(24 + (u - 8));
}
struct Fp6Book { uint32_t w[kDialects][2]; };   // [dialect] -> 8 six-bit magnitudes, one per byte
constexpr Fp6Book make_fp6_book() {
    Fp6Book b{};
    for (int d = 0; d < kDialects; ++d)
        for (int j = 0; j < 8; ++j) b.w[d][j / 4] |= (uint32_t)e2m3_of_half_units(kBook[d][j]) << (8 * (j % 4));
    return b;
}
static __device__ const Fp6Book g_fp6_book = make_fp6_book();

// 8 codes (one dword) -> 48 bits: 8 six-bit values, element j in bits [6 j, 6 j + 6)
__device__ __forceinline__ uint64_t pack6(uint32_t c, uint32_t tlo, uint32_t thi) {
    const uint32_t ie = c & 0x07070707u, io = (c >> 4) & 0x07070707u;
    const uint32_t e = __builtin_amdgcn_perm(thi, tlo, ie) | ((c << 2) & 0x20202020u);   // elements 0, 2, 4, 6
    const uint32_t o = __builtin_amdgcn_perm(thi, tlo, io) | ((c >> 2) & 0x20202020u);   // elements 1, 3, 5, 7
    const uint32_t lo24 = (e & 0x3fu) | ((o & 0x3fu) << 6) | (((e >> 8) & 0x3fu) << 12) | (((o >> 8) & 0x3fu) << 18);
    const uint32_t hi24 = ((e >> 16) & 0x3fu) | (((o >> 16) & 0x3fu) << 6) | ((e >> 24) << 12) | ((o >> 24) << 18);
    return (uint64_t)lo24 | ((uint64_t)hi24 << 24);
}

// Packed FP6 operand: per (32-row tile, step) 1792 bytes = 64 lanes x 16 bytes (registers 0..3) followed by
// 64 lanes x 12 bytes (registers 4, 5, one unused dword); lane = 32 * (block % 2) + row % 32.
constexpr int kFp6ChunkBytes = 1792;

}  // namespace
}  // namespace dfp4
