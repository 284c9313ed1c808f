// Per-block arithmetic of the DialectFP4 / MXFP4 quantizers (paper Sections 3.2, 3.3),
// shared by the quantizer kernels and by the GEMM's requantizing epilogue.
// Mapping: four consecutive lanes own one block of 32; each lane holds 8 elements as
// four dwords of two bf16 (one 16-byte load).  Block reductions are two DPP
// quad-permute steps, so all four lanes of a quad must be active.
#pragma once
#include "common.h"
#include "formatbook.h"

namespace dfp4 {

// lookup tables derived from the formatbook at compile time (one copy per translation unit)
static __device__ const QuantTables g_quant_tables = make_quant_tables();

namespace {

typedef unsigned short us2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float as_f(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u(float f) { return __builtin_bit_cast(uint32_t, f); }

// value of the lane's quad neighbour: XOR 1 (0xB1) and XOR 2 (0x4E)
template <int CTRL>
__device__ __forceinline__ uint32_t quad(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}

__device__ __forceinline__ uint32_t sign_nibbles(const uint32_t (&w)[4]) {
    // bf16 sign bits (bit 15 / bit 31 of dword j) -> bit 3 / bit 7 of code byte j.
    // v_perm_b32 gathers the high byte of every bf16: p = {w_a.b3, w_b.b3, w_a.b1, w_b.b1}
    const uint32_t p0 = __builtin_amdgcn_perm(w[1], w[0], 0x05010703u);
    const uint32_t p1 = __builtin_amdgcn_perm(w[3], w[2], 0x05010703u);
    const uint32_t hi = __builtin_amdgcn_perm(p1, p0, 0x05040100u);   // odd elements of dwords 0..3
    const uint32_t lo = __builtin_amdgcn_perm(p1, p0, 0x07060302u);   // even elements of dwords 0..3
    return (hi & 0x80808080u) | ((lo >> 4) & 0x08080808u);
}

// value of the lane that mirrors this one inside its group of 8 lanes (lane i <-> 7 - i): after a
// reduction over the quad it is the other quad's result
__device__ __forceinline__ uint32_t other_quad(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xf, 0xf, true);
}

// Block maximum over the quad's 32 elements (WIDE: over the 64 elements of two neighbouring quads),
// as bf16 bits (sign cleared).
template <bool WIDE = false>
__device__ __forceinline__ uint32_t block_amax_bits(const uint32_t (&w)[4]) {
    float m = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        m = __builtin_fmaxf(m, __builtin_fabsf(as_f(w[j] << 16)));
        m = __builtin_fmaxf(m, __builtin_fabsf(as_f(w[j])));
    }
    // non-negative floats order like their bit patterns
    uint32_t u = as_u(m);
    u = max(u, quad<0xB1>(u));
    u = max(u, quad<0x4E>(u));
    if constexpr (WIDE) u = max(u, other_quad(u));
    return u >> 16;
}

// Maximum over the 16 elements of two neighbouring lanes (blocks of 16), as bf16 bits (sign cleared).
__device__ __forceinline__ uint32_t pair_amax_bits(const uint32_t (&w)[4]) {
    float m = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        m = __builtin_fmaxf(m, __builtin_fabsf(as_f(w[j] << 16)));
        m = __builtin_fmaxf(m, __builtin_fabsf(as_f(w[j])));
    }
    uint32_t u = as_u(m);
    u = max(u, quad<0xB1>(u));
    return u >> 16;
}

// One lane's share (8 elements) of one DialectFP4 block.  WIDE: blocks of 64 elements (two
// neighbouring quads share the exponent and the dialect; Section 4.2, Table 3 varies the block size).
template <bool WIDE = false>
__device__ __forceinline__ void dfp4_pass(const uint4& wv, const uint8_t* __restrict__ lut_s,
                                          const uint8_t* __restrict__ lut_q, uint32_t& code,
                                          uint32_t& ebyte, uint32_t& dial) {
    const uint32_t w[4] = {wv.x, wv.y, wv.z, wv.w};
    const uint32_t ab = block_amax_bits<WIDE>(w);
    // exponent byte = biased exponent of the maximum, minus 2, floored at 0
    const int byte = max((int)(ab >> 7) - 2, 0);
    const int n = 129 - byte;                       // 4 |x| / 2^e = |x| * 2^n
    // stage 1: block maximum rounded half-up to a multiple of 0.5 selects the pair
    const uint32_t tmax = (uint32_t)ldexpf(as_f(ab << 16), n);
    const uint32_t r = min(max((tmax + 1u) >> 1, 8u), 15u);
    const uint32_t pair = 15u - r;
    uint32_t key[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t t0 = (uint32_t)ldexpf(__builtin_fabsf(as_f(w[j] << 16)), n);
        const uint32_t t1 = (uint32_t)ldexpf(__builtin_fabsf(as_f(w[j])), n);
        key[j] = t0 | (t1 << 5);
    }
    // stage 2: votes of this lane's 8 elements (even dialect +1, odd dialect -1), then of the
    // quad; the odd dialect needs strictly more votes
    const int8_t* s = reinterpret_cast<const int8_t*>(lut_s) + pair * 1024u;
    uint32_t v = (uint32_t)((int)s[key[0]] + (int)s[key[1]] + (int)s[key[2]] + (int)s[key[3]]);
    v += quad<0xB1>(v);
    v += quad<0x4E>(v);
    if constexpr (WIDE) v += other_quad(v);
    dial = 2u * pair + (v >> 31);
    const uint8_t* q = lut_q + dial * 1024u;
    const us2 qe = {q[key[0]], q[key[2]]}, qo = {q[key[1]], q[key[3]]};   // bytes 0, 2 and bytes 1, 3
    code = (__builtin_bit_cast(uint32_t, qe) | (__builtin_bit_cast(uint32_t, qo) << 8)) | sign_nibbles(w);
    ebyte = (uint32_t)byte;
}

// The same with tables keyed by ONE 5-bit magnitude (768 bytes in all instead of 24 KiB: twice the
// lookups, but a workgroup fills them with a single load): lut_i[d * 32 + t] = index of t under
// dialect d, lut_v[p * 32 + t] = vote of t in pair p (+1 even dialect, -1 odd, as int8).
// NARROW: blocks of 16 elements (Section 4.2, Table 3): two neighbouring lanes own a block, so the
// maximum and the votes are reduced over the lane pair only.
template <bool NARROW = false>
__device__ __forceinline__ void dfp4_pass_small(const uint4& wv, const uint8_t* __restrict__ lut_v,
                                                const uint8_t* __restrict__ lut_i, uint32_t& code,
                                                uint32_t& ebyte, uint32_t& dial) {
    const uint32_t w[4] = {wv.x, wv.y, wv.z, wv.w};
    const uint32_t ab = NARROW ? pair_amax_bits(w) : block_amax_bits<false>(w);
    const int byte = max((int)(ab >> 7) - 2, 0);
    const int n = 129 - byte;
    const uint32_t tmax = (uint32_t)ldexpf(as_f(ab << 16), n);
    const uint32_t r = min(max((tmax + 1u) >> 1, 8u), 15u);
    const uint32_t pair = 15u - r;
    uint32_t t[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        t[2 * j] = (uint32_t)ldexpf(__builtin_fabsf(as_f(w[j] << 16)), n);
        t[2 * j + 1] = (uint32_t)ldexpf(__builtin_fabsf(as_f(w[j])), n);
    }
    const int8_t* sv = reinterpret_cast<const int8_t*>(lut_v) + pair * 32u;
    int votes = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) votes += (int)sv[t[j]];
    uint32_t v = (uint32_t)votes;
    v += quad<0xB1>(v);
    if constexpr (!NARROW) v += quad<0x4E>(v);
    dial = 2u * pair + (v >> 31);
    const uint8_t* q = lut_i + dial * 32u;
    uint32_t c = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) c |= (uint32_t)q[t[j]] << (4 * j);
    code = c | sign_nibbles(w);
    ebyte = (uint32_t)byte;
}

// One lane's share of one MXFP4 block: E2M1, round to nearest, ties to even code.
__device__ __forceinline__ void mxfp4_pass(const uint4& wv, const uint8_t* __restrict__ lut_mx,
                                           uint32_t& code, uint32_t& ebyte) {
    const uint32_t w[4] = {wv.x, wv.y, wv.z, wv.w};
    const uint32_t ab = block_amax_bits(w);
    const int byte = max((int)(ab >> 7) - 2, 0);
    const int n = 129 - byte;
    uint32_t c = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float v0 = ldexpf(__builtin_fabsf(as_f(w[j] << 16)), n);
        const float v1 = ldexpf(__builtin_fabsf(as_f(w[j] & 0xffff0000u)), n);
        const uint32_t t0 = (uint32_t)v0, t1 = (uint32_t)v1;
        const uint32_t k0 = 2u * t0 + ((float)t0 != v0 ? 1u : 0u);
        const uint32_t k1 = 2u * t1 + ((float)t1 != v1 ? 1u : 0u);
        c |= ((uint32_t)lut_mx[k0] | ((uint32_t)lut_mx[k1] << 4)) << (8 * j);
    }
    code = c | sign_nibbles(w);
    ebyte = (uint32_t)byte;
}

}  // namespace
}  // namespace dfp4
