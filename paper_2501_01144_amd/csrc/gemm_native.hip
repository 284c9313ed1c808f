// Block-scaled GEMM on the CDNA4 scaled matrix instruction
// (v_mfma_scale_f32_32x32x64_f8f6f4): out = A * W^T with one power-of-two scale per
// 32 elements along K applied by the hardware, fp32 accumulation.
//
// Two operand formats:
//   FP4 (E2M1)  MXFP4 tensors are multiplied as they are: the 4-bit code (sign, 3-bit
//               index into {0, .5, 1, 1.5, 2, 3, 4, 6}) is the E2M1 bit pattern and the
//               exponent byte e + 127 is the E8M0 scale.
//   FP6 (E2M3)  every DialectFP4 value 0.5 u (u <= 15) is an E2M3 number, so the codes of
//               both operands are repacked to 6 bits through the dialect tables and the
//               same kernel multiplies them; the exponent byte is again the scale.
// (Section 3.3 of the paper builds its MAC from integer products because its values are
// not a standard format; on this GPU a standard format covers them.)
//
// Operand layout of the instruction (checked on the hardware): lane l supplies row or
// column l % 32 and the 32 consecutive K elements of block l / 32 of the pair, element j
// in bits [w j, w j + w) of its operand registers (w = 4 or 6); the scale is the byte of
// the scale register that op_sel names, 2^(byte - 127).  Output as the other 32x32 MFMAs:
// register x of lane (h, c) is row 8 (x / 4) + 4 h + x % 4, column c.
//
// Two kernels.  native_pack_kernel rewrites an operand in the order the matrix instruction
// wants it (per 32-row tile and step, 64 lanes x 16 or 24 bytes, plus one dword of four
// scale bytes per lane and group of four tiles), so that the multiply kernel's loads are
// whole 1 KiB lines.  gemm_native_kernel: 256 x 256 outputs per workgroup, four waves as
// 2 x 2, each 128 x 128 (16 accumulator tiles = 256 registers, one wave per SIMD); operands
// go from global memory straight to registers, one step (a pair of blocks) ahead; no LDS,
// no barrier.  For weights the packing could be done once, offline.
#include "common.h"
#include "formatbook.h"

namespace dfp4 {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kFmtFp6 = 2, kFmtFp4 = 4;      // format codes of the instruction (E2M3, E2M1)

__device__ __forceinline__ uint16_t f32_to_bf16_rne_n(float f) {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Packed operands (written by native_pack_kernel): rows padded to a multiple of 128,
// S = ceil(KB / 2) steps, a missing second block is all zeros.
//   lo  [row tile of 32][step][lane][16 bytes]   registers 0..3 of the lane
//   hi  [row tile of 32][step][lane][ 8 bytes]   registers 4..5 (FP6 only)
//   sc  [group of 4 row tiles][step][lane] dword: byte t = scale byte of row tile 4 g + t
struct PackedOperand {
    uint4* lo;
    uint2* hi;
    uint32_t* sc;
};

struct NativeParams {
    PackedOperand a, w;
    void* out;
    int M, N, S;
    int64_t ldc;
};

struct PackParams {
    const uint8_t *codes, *dial, *expo;
    PackedOperand dst;
    int rows, KB, S, tiles;        // tiles = padded rows / 32
};

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
__device__ const Fp6Book g_fp6_book = make_fp6_book();

// 8 codes (one dword) -> 48 bits: 8 six-bit values, element j in bits [6 j, 6 j + 6)
__device__ __forceinline__ uint64_t pack6(uint32_t c, uint32_t tlo, uint32_t thi) {
    const uint32_t ie = c & 0x07070707u, io = (c >> 4) & 0x07070707u;
    const uint32_t e = __builtin_amdgcn_perm(thi, tlo, ie) | ((c << 2) & 0x20202020u);   // elements 0, 2, 4, 6
    const uint32_t o = __builtin_amdgcn_perm(thi, tlo, io) | ((c >> 2) & 0x20202020u);   // elements 1, 3, 5, 7
    const uint32_t lo24 = (e & 0x3fu) | ((o & 0x3fu) << 6) | (((e >> 8) & 0x3fu) << 12) | (((o >> 8) & 0x3fu) << 18);
    const uint32_t hi24 = ((e >> 16) & 0x3fu) | (((o >> 16) & 0x3fu) << 6) | ((e >> 24) << 12) | ((o >> 24) << 18);
    return (uint64_t)lo24 | ((uint64_t)hi24 << 24);
}

// One wave per (row tile, step); lane (kh, c) takes row 32 tile + c, block 2 step + kh.
template <int FMT>
__global__ __launch_bounds__(256) void native_pack_kernel(PackParams p) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int kh = lane >> 5, c = lane & 31;
    const int tile = blockIdx.y, s = blockIdx.x * 4 + wave;
    if (s >= p.S) return;
    const int row = tile * 32 + c, kb = 2 * s + kh;
    const bool on = row < p.rows && kb < p.KB;
    uint4 codes = make_uint4(0, 0, 0, 0);
    uint32_t eb = 0, dl = 7;
    if (on) {
        const int64_t blk = (int64_t)row * p.KB + kb;
        codes = *reinterpret_cast<const uint4*>(p.codes + blk * 16);
        eb = p.expo[blk];
        if constexpr (FMT == kFmtFp6) dl = p.dial ? ((uint32_t)p.dial[blk] & 15u) : 7u;
    }
    const int64_t slot = ((int64_t)tile * p.S + s) * 64 + lane;
    if constexpr (FMT == kFmtFp4) {
        p.dst.lo[slot] = codes;                 // the MXFP4 code is the E2M1 bit pattern
    } else {
        const uint32_t tlo = g_fp6_book.w[dl][0], thi = g_fp6_book.w[dl][1];
        const uint64_t p0 = pack6(codes.x, tlo, thi), p1 = pack6(codes.y, tlo, thi);
        const uint64_t p2 = pack6(codes.z, tlo, thi), p3 = pack6(codes.w, tlo, thi);
        uint4 lo;
        lo.x = (uint32_t)p0;
        lo.y = (uint32_t)(p0 >> 32) | ((uint32_t)p1 << 16);
        lo.z = (uint32_t)(p1 >> 16);
        lo.w = (uint32_t)p2;
        p.dst.lo[slot] = lo;
        p.dst.hi[slot] = make_uint2((uint32_t)(p2 >> 32) | ((uint32_t)p3 << 16), (uint32_t)(p3 >> 16));
    }
    reinterpret_cast<uint8_t*>(p.dst.sc)[(((int64_t)(tile >> 2) * p.S + s) * 64 + lane) * 4 + (tile & 3)] = (uint8_t)eb;
}

template <int FMT>
struct Operand {
    v8i v[4];        // four 32-row (or 32-column) tiles
    int s;           // their four scale bytes
};

template <int FMT>
__device__ __forceinline__ void load_operand(const PackedOperand& src, int tile0, int S, int s, int lane,
                                             Operand<FMT>& o) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int64_t slot = ((int64_t)(tile0 + t) * S + s) * 64 + lane;
        const uint4 lo = src.lo[slot];
        o.v[t] = v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, 0, 0, 0, 0};
        if constexpr (FMT == kFmtFp6) {
            const uint2 hi = src.hi[slot];
            o.v[t][4] = (int)hi.x;
            o.v[t][5] = (int)hi.y;
        }
    }
    o.s = (int)src.sc[((int64_t)(tile0 >> 2) * S + s) * 64 + lane];
}

template <int FMT, bool BF16>
__global__ __launch_bounds__(256, 1) void gemm_native_kernel(NativeParams p) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kh = lane >> 5, c = lane & 31;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * 256 + wm * 128, n0 = blockIdx.x * 256 + wn * 128;
    if (m0 >= p.M || n0 >= p.N) return;        // wave-uniform; the kernel has no barrier
    const int S = p.S;
    v16f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int x = 0; x < 16; ++x) acc[i][j][x] = 0.0f;

    Operand<FMT> a, b, an, bn;
    load_operand<FMT>(p.a, m0 >> 5, S, 0, lane, a);
    load_operand<FMT>(p.w, n0 >> 5, S, 0, lane, b);
    for (int s = 0; s < S; ++s) {
        const int sn = min(s + 1, S - 1);       // the last step reloads itself (unused)
        load_operand<FMT>(p.a, m0 >> 5, S, sn, lane, an);
        load_operand<FMT>(p.w, n0 >> 5, S, sn, lane, bn);
#define DFP4_NATIVE_ROW(I)                                                                                    \
        acc[I][0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a.v[I], b.v[0], acc[I][0], FMT, FMT, I, a.s, 0, b.s); \
        acc[I][1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a.v[I], b.v[1], acc[I][1], FMT, FMT, I, a.s, 1, b.s); \
        acc[I][2] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a.v[I], b.v[2], acc[I][2], FMT, FMT, I, a.s, 2, b.s); \
        acc[I][3] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a.v[I], b.v[3], acc[I][3], FMT, FMT, I, a.s, 3, b.s);
        DFP4_NATIVE_ROW(0) DFP4_NATIVE_ROW(1) DFP4_NATIVE_ROW(2) DFP4_NATIVE_ROW(3)
#undef DFP4_NATIVE_ROW
        a = an;
        b = bn;
    }

    // epilogue: fp32 (or bf16, round to nearest even) [M, N]
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + j * 32 + c;
#pragma unroll
            for (int x = 0; x < 16; ++x) {
                const int m = m0 + i * 32 + 8 * (x >> 2) + 4 * kh + (x & 3);
                if (m < p.M && n < p.N) {
                    const int64_t o = (int64_t)m * p.ldc + n;
                    if constexpr (BF16)
                        static_cast<uint16_t*>(p.out)[o] = f32_to_bf16_rne_n(acc[i][j][x]);
                    else
                        static_cast<float*>(p.out)[o] = acc[i][j][x];
                }
            }
        }
}

struct NativeLayout { int64_t a_lo, a_hi, a_sc, w_lo, w_hi, w_sc, total; };
inline int64_t up256(int64_t x) { return (x + 255) & ~(int64_t)255; }
inline NativeLayout native_layout(int64_t M, int64_t N, int64_t KB, bool fp6) {
    const int64_t S = (KB + 1) / 2, tm = (M + 127) / 128 * 4, tn = (N + 127) / 128 * 4;
    NativeLayout l{};
    l.a_lo = 0;
    l.a_hi = up256(l.a_lo + tm * S * 1024);
    l.a_sc = up256(l.a_hi + (fp6 ? tm * S * 512 : 0));
    l.w_lo = up256(l.a_sc + (tm / 4) * S * 256);
    l.w_hi = up256(l.w_lo + tn * S * 1024);
    l.w_sc = up256(l.w_hi + (fp6 ? tn * S * 512 : 0));
    l.total = up256(l.w_sc + (tn / 4) * S * 256);
    return l;
}

}  // namespace

size_t gemm_native_workspace_bytes(int64_t M, int64_t N, int64_t K, bool fp6) {
    if (M == 0 || N == 0) return 0;
    return (size_t)native_layout(M, N, K / kBlock, fp6).total;
}

// fp6 = false: MXFP4 operands on the FP4 form of the instruction; true: DialectFP4 (or MXFP4,
// dialect pointer null) operands repacked to FP6 E2M3.
int launch_gemm_native(bool fp6, dfp4_tensor A, dfp4_tensor W, void* out, int out_dtype, int64_t ldc,
                       void* workspace, size_t workspace_bytes, hipStream_t stream) {
    const int64_t M = A.rows, N = W.rows, KB = A.K / kBlock;
    if (M == 0 || N == 0) return DFP4_OK;
    if (M >= (1 << 30) || N >= (1 << 30) || KB >= (1 << 26) || KB == 0) return KB == 0 ? DFP4_ERR_SHAPE : DFP4_ERR_SHAPE;
    const NativeLayout lay = native_layout(M, N, KB, fp6);
    if ((size_t)lay.total > workspace_bytes) return DFP4_ERR_WORKSPACE;
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    const int S = (int)((KB + 1) / 2);
    NativeParams p{};
    p.a = PackedOperand{reinterpret_cast<uint4*>(ws + lay.a_lo), reinterpret_cast<uint2*>(ws + lay.a_hi),
                        reinterpret_cast<uint32_t*>(ws + lay.a_sc)};
    p.w = PackedOperand{reinterpret_cast<uint4*>(ws + lay.w_lo), reinterpret_cast<uint2*>(ws + lay.w_hi),
                        reinterpret_cast<uint32_t*>(ws + lay.w_sc)};
    p.out = out; p.M = (int)M; p.N = (int)N; p.S = S; p.ldc = ldc;
    for (int side = 0; side < 2; ++side) {
        const dfp4_tensor& T = side ? W : A;
        PackParams q{};
        q.codes = T.codes; q.dial = T.dialect; q.expo = T.exponent;
        q.dst = side ? p.w : p.a;
        q.rows = (int)T.rows; q.KB = (int)KB; q.S = S; q.tiles = (int)((T.rows + 127) / 128 * 4);
        dim3 gp((unsigned)((S + 3) / 4), (unsigned)q.tiles);
        if (gp.y > 65535) return DFP4_ERR_SHAPE;
        if (fp6) hipLaunchKernelGGL((native_pack_kernel<kFmtFp6>), gp, dim3(256), 0, stream, q);
        else hipLaunchKernelGGL((native_pack_kernel<kFmtFp4>), gp, dim3(256), 0, stream, q);
    }
    dim3 grid((unsigned)((N + 255) / 256), (unsigned)((M + 255) / 256));
    if (grid.y > 65535) return DFP4_ERR_SHAPE;
    const bool bf16 = out_dtype == DFP4_BF16;
    if (fp6) {
        if (bf16) hipLaunchKernelGGL((gemm_native_kernel<kFmtFp6, true>), grid, dim3(256), 0, stream, p);
        else hipLaunchKernelGGL((gemm_native_kernel<kFmtFp6, false>), grid, dim3(256), 0, stream, p);
    } else {
        if (bf16) hipLaunchKernelGGL((gemm_native_kernel<kFmtFp4, true>), grid, dim3(256), 0, stream, p);
        else hipLaunchKernelGGL((gemm_native_kernel<kFmtFp4, false>), grid, dim3(256), 0, stream, p);
    }
    return check_launch();
}

}  // namespace dfp4
