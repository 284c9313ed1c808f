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
// Kernels.  native_pack_kernel rewrites an operand in the order the matrix instruction
// wants it (per 32-row tile and step, 64 lanes x 16 bytes, for FP6 followed by 64 lanes x 12
// bytes of which 8 are used, plus one dword of four scale bytes per lane and group of four
// tiles), so that the multiply kernel's loads are whole lines; weights are packed once,
// offline, and quantize_native_kernel (quantize.hip) writes an activation in this form
// directly.  gemm_native_kernel: 256 x 256 outputs per workgroup, four waves as 2 x 2, each
// 128 x 128 (16 accumulator tiles = 256 registers, one wave per SIMD), or 128 x 256 per
// workgroup when there are few tiles; operands go global -> LDS by direct loads three (FP6)
// or seven (FP4) steps ahead, LDS -> registers one step ahead, one barrier per step; the
// main loop is generated assembly (gen_native_loop.py).  With very few tiles K is split
// between workgroups and native_reduce_kernel adds their fp32 partial tiles in a fixed order.
#include <type_traits>
#include "common.h"
#include "formatbook.h"
#include "fp6_pack.h"
#include "gemm_native_asm.inc"

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

// Packed operands (written by native_pack_kernel): rows padded to a multiple of 256,
// S = ceil(KB / 2) steps, a missing second block is all zeros.
//   bits [row tile of 32][step][64 lanes x 16 bytes]                    FP4: registers 0..3 of the lane
//        [row tile of 32][step][64 lanes x 16 bytes | 64 lanes x 12 bytes]   FP6: registers 0..3 | 4, 5, pad
//   sc   [group of 4 row tiles][step][lane] dword: byte t = scale byte of row tile 4 g + t
// Both arrays end with eight steps of slack: the loop loads up to seven steps ahead.
struct PackedOperand {
    uint8_t* bits;
    uint32_t* sc;
};

struct NativeParams {
    PackedOperand a, w;
    void* out;
    int M, N, S;
    int64_t ldc;
    int ksplit;              // workgroups sharing a tile (each a range of steps); partial tiles go to `part`
    float* part;             // [ksplit][M][N] fp32
};

struct PackParams {
    const uint8_t *codes, *dial, *expo;
    PackedOperand dst;
    int rows, KB, S;
};

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
    const int64_t chunk = (int64_t)tile * p.S + s;
    if constexpr (FMT == kFmtFp4) {
        reinterpret_cast<uint4*>(p.dst.bits)[chunk * 64 + lane] = codes;     // the MXFP4 code is the E2M1 bit pattern
    } else {
        const uint32_t tlo = g_fp6_book.w[dl][0], thi = g_fp6_book.w[dl][1];
        const uint64_t p0 = pack6(codes.x, tlo, thi), p1 = pack6(codes.y, tlo, thi);
        const uint64_t p2 = pack6(codes.z, tlo, thi), p3 = pack6(codes.w, tlo, thi);
        uint32_t* d0 = reinterpret_cast<uint32_t*>(p.dst.bits + chunk * 1792 + lane * 16);
        d0[0] = (uint32_t)p0;
        d0[1] = (uint32_t)(p0 >> 32) | ((uint32_t)p1 << 16);
        d0[2] = (uint32_t)(p1 >> 16);
        d0[3] = (uint32_t)p2;
        uint32_t* d1 = reinterpret_cast<uint32_t*>(p.dst.bits + chunk * 1792 + 1024 + lane * 12);
        d1[0] = (uint32_t)(p2 >> 32) | ((uint32_t)p3 << 16);
        d1[1] = (uint32_t)(p3 >> 16);
        d1[2] = 0;
    }
    reinterpret_cast<uint8_t*>(p.dst.sc)[(((int64_t)(tile >> 2) * p.S + s) * 64 + lane) * 4 + (tile & 3)] = (uint8_t)eb;
}

// TA = 32-row tiles per wave: 4 (256 x 256 per workgroup) or 2 (128 x 256, for products with few tiles)
template <int FMT, bool BF16, int TA>
__global__ __launch_bounds__(256, 1) void gemm_native_kernel(NativeParams p) {
    constexpr bool kFp6 = FMT == kFmtFp6;
    constexpr int kTileLds = kFp6 ? 2048 : 1024, kStage = (2 * TA + 8) * kTileLds + 1024, kStages = kFp6 ? 4 : 8;
    constexpr int kRowsWg = 64 * TA, kRowsWave = 32 * TA;
    constexpr int kGStride = kFp6 ? 1792 : 1024;             // global bytes per (tile, step)
    __shared__ __attribute__((aligned(16))) uint8_t s_stage[kStages * kStage];
    const int tid = threadIdx.x, lane = tid & 63;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane(tid >> 6);
    const int kh = lane >> 5, c = lane & 31;
    const int wm = (int)wave >> 1, wn = (int)wave & 1;
    // this workgroup's range of steps (split K: blockIdx.z)
    const int per = (p.S + p.ksplit - 1) / p.ksplit;
    const int s_lo = (int)blockIdx.z * per, S = min(p.S, s_lo + per) - s_lo;
    {
        const uint32_t lds = (uint32_t)__builtin_amdgcn_readfirstlane(
            (int)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)&s_stage[0]);
        const uint32_t tstride = (uint32_t)p.S * (uint32_t)kGStride;      // bytes per tile
        // this wave fetches A tiles 2w, 2w+1 and B tiles 2w, 2w+1 of the workgroup's 8 + 8, and scale chunk w
        const uint64_t ab = reinterpret_cast<uint64_t>(p.a.bits) +
                            ((uint64_t)blockIdx.y * (2 * TA) + (TA == 4 ? 2 * wave : wave)) * tstride;
        const uint64_t bb = reinterpret_cast<uint64_t>(p.w.bits) + ((uint64_t)blockIdx.x * 8 + 2 * wave) * tstride;
        const uint64_t sb = wave < 2
            ? reinterpret_cast<uint64_t>(p.a.sc) + (TA == 4 ? (uint64_t)blockIdx.y * 2 + wave : (uint64_t)blockIdx.y) * (uint64_t)p.S * 256
            : reinterpret_cast<uint64_t>(p.w.sc) + ((uint64_t)blockIdx.x * 2 + (wave - 2)) * (uint64_t)p.S * 256;
        const uint32_t l16 = (uint32_t)lane * 16u, l4 = (uint32_t)lane * 4u;
        const uint32_t g16 = l16 + (uint32_t)s_lo * kGStride, g12 = (uint32_t)lane * 12u + (uint32_t)s_lo * kGStride;
        const uint32_t g4 = l4 + (uint32_t)s_lo * 256u;
#define DFP4_NATIVE_RUN(LOOP)                                                                                     \
        asm volatile(LOOP                                                                                           \
                     :                                                                                              \
                     : [alo] "s"((uint32_t)ab), [ahi] "s"((uint32_t)(ab >> 32)), [blo] "s"((uint32_t)bb),        \
                       [bhi] "s"((uint32_t)(bb >> 32)), [slo] "s"((uint32_t)sb), [shi] "s"((uint32_t)(sb >> 32)), \
                       [tstride] "s"(tstride), [wv] "s"(wave), [lds] "s"(lds),                                      \
                       [ldsend] "s"(lds + (uint32_t)(kStages * kStage)), [steps] "s"((uint32_t)S),                  \
                       [l16] "v"(l16), [l4] "v"(l4), [g16] "v"(g16), [g12] "v"(g12), [g4] "v"(g4)                   \
                     : DFP4_NATIVE_VGPR_CLOBBERS, DFP4_NATIVE_ACC_CLOBBERS, DFP4_NATIVE_SGPR_CLOBBERS, "m0", "scc", \
                       "memory")
        if constexpr (kFp6 && TA == 4) DFP4_NATIVE_RUN(DFP4_NATIVE_LOOP_FP6);
        else if constexpr (kFp6) DFP4_NATIVE_RUN(DFP4_NATIVE_LOOP_FP6_H);
        else if constexpr (TA == 4) DFP4_NATIVE_RUN(DFP4_NATIVE_LOOP_FP4);
        else DFP4_NATIVE_RUN(DFP4_NATIVE_LOOP_FP4_H);
#undef DFP4_NATIVE_RUN
    }

    // epilogue: fp32 (or bf16, round to nearest even) [M, N]; accumulator tile (i, j) = 4 i + j.
    // Register x of lane (kh, c) is row 32 i + 8 (x / 4) + 4 kh + x % 4, column 32 j + c.  Row
    // addresses are wave-uniform (scalar registers); the lane adds a constant byte offset.
    const int m0 = blockIdx.y * kRowsWg + wm * kRowsWave, n0 = blockIdx.x * 256 + wn * 128;
    if (m0 >= p.M || n0 >= p.N) return;
    constexpr int kEsz = BF16 ? 2 : 4;
    // split K: the fp32 partial tile of this range goes to part[blockIdx.z] (the kernel is then the fp32 one)
    const bool partial = p.ksplit > 1;
    const int64_t ld = partial ? p.N : p.ldc;
    uint8_t* base = partial ? reinterpret_cast<uint8_t*>(p.part + (int64_t)blockIdx.z * p.M * p.N)
                            : static_cast<uint8_t*>(p.out);
    uint8_t* wave_out = base + ((int64_t)m0 * ld + n0) * kEsz;                                 // uniform
    const int64_t row_bytes = ld * kEsz;                                                       // uniform
    const bool full = m0 + kRowsWave <= p.M && n0 + 128 <= p.N;                                // uniform
    // bf16: lanes exchange values in pairs so that every lane stores two adjacent columns of one
    // row (even lanes the even row of a row pair, odd lanes the odd row)
    const bool pairs = BF16 && full && (ld & 1) == 0 && (reinterpret_cast<uintptr_t>(base) & 3) == 0;
    const uint32_t lane_off = pairs ? (uint32_t)((4 * kh + (c & 1)) * row_bytes + (c & ~1) * kEsz)
                                    : (uint32_t)(4 * kh * row_bytes + c * kEsz);
    auto store_tile = [&](auto full_c, auto pairs_c, int t, int (&v)[16]) {
        constexpr bool kFull = decltype(full_c)::value, kPairs = decltype(pairs_c)::value;
        const int i = t >> 2, j = t & 3;
        uint8_t* tile_out = wave_out + (int64_t)i * 32 * row_bytes + j * 32 * kEsz;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint8_t* rowp = tile_out + (int64_t)(8 * q) * row_bytes;                           // uniform
            if constexpr (BF16 && kPairs) {
#pragma unroll
                for (int jj = 0; jj < 4; jj += 2) {
                    const uint32_t b0 = f32_to_bf16_rne_n(__builtin_bit_cast(float, v[4 * q + jj]));
                    const uint32_t b1 = f32_to_bf16_rne_n(__builtin_bit_cast(float, v[4 * q + jj + 1]));
                    const uint32_t send = (c & 1) ? b0 : b1;
                    const uint32_t recv = (uint32_t)__builtin_amdgcn_mov_dpp((int)send, 0xB1, 0xf, 0xf, true);
                    const uint32_t word = (c & 1) ? (recv | (b1 << 16)) : (b0 | (recv << 16));
                    *reinterpret_cast<uint32_t*>(rowp + (int64_t)jj * row_bytes + lane_off) = word;
                }
            } else {
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    if (kFull || (m0 + i * 32 + 8 * q + 4 * kh + jj < p.M && n0 + j * 32 + c < p.N)) {
                        uint8_t* dst = rowp + (int64_t)jj * row_bytes + lane_off;
                        if constexpr (BF16)
                            *reinterpret_cast<uint16_t*>(dst) = f32_to_bf16_rne_n(__builtin_bit_cast(float, v[4 * q + jj]));
                        else
                            *reinterpret_cast<int*>(dst) = v[4 * q + jj];
                    }
                }
            }
        }
    };
#define DFP4_NATIVE_STORE(G)                                                                        \
    {                                                                                               \
        int v[16];                                                                                  \
        asm volatile(DFP4_NATIVE_ACC_READ_##G                                                       \
                     : "=v"(v[0]), "=v"(v[1]), "=v"(v[2]), "=v"(v[3]), "=v"(v[4]), "=v"(v[5]),      \
                       "=v"(v[6]), "=v"(v[7]), "=v"(v[8]), "=v"(v[9]), "=v"(v[10]), "=v"(v[11]),    \
                       "=v"(v[12]), "=v"(v[13]), "=v"(v[14]), "=v"(v[15]));                         \
        store_tile(kFullC, kPairsC, G, v);                                                          \
    }
#define DFP4_NATIVE_ALL                                                                             \
    DFP4_NATIVE_STORE(0) DFP4_NATIVE_STORE(1) DFP4_NATIVE_STORE(2) DFP4_NATIVE_STORE(3)             \
    DFP4_NATIVE_STORE(4) DFP4_NATIVE_STORE(5) DFP4_NATIVE_STORE(6) DFP4_NATIVE_STORE(7)             \
    if constexpr (TA == 4) {                                                                        \
        DFP4_NATIVE_STORE(8) DFP4_NATIVE_STORE(9) DFP4_NATIVE_STORE(10) DFP4_NATIVE_STORE(11)       \
        DFP4_NATIVE_STORE(12) DFP4_NATIVE_STORE(13) DFP4_NATIVE_STORE(14) DFP4_NATIVE_STORE(15)     \
    }
    if (pairs) {
        constexpr std::true_type kFullC{}, kPairsC{};
        DFP4_NATIVE_ALL
    } else if (full) {
        constexpr std::true_type kFullC{};
        constexpr std::false_type kPairsC{};
        DFP4_NATIVE_ALL
    } else {
        constexpr std::false_type kFullC{}, kPairsC{};
        DFP4_NATIVE_ALL
    }
#undef DFP4_NATIVE_ALL
#undef DFP4_NATIVE_STORE
}

// Few rows of A (decode shapes, M <= 64): 32 W rows per workgroup, its 16 waves share K (wave w
// takes a contiguous range of steps), one or two MFMAs per step; the 16 partial tiles are added in
// a fixed order through LDS.  No vector-ALU work: both operands arrive packed.
template <int FMT, bool BF16>
__global__ __launch_bounds__(1024) void gemm_native_small_kernel(NativeParams p) {
    constexpr bool kFp6 = FMT == kFmtFp6;
    constexpr int kStride = kFp6 ? kFp6ChunkBytes : 1024;
    __shared__ float s_red[8][2][16][64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kh = lane >> 5, c = lane & 31;
    const int S = p.S, t = blockIdx.x, mt = (p.M + 31) / 32;           // mt = 1 or 2 row tiles of A
    const int per = (S + 15) / 16, s_lo = wave * per, s_hi = min(S, s_lo + per);
    auto load = [&](const PackedOperand& src, int tile, int s, v8i& v, int& sc) {
        const uint8_t* q = src.bits + ((int64_t)tile * S + s) * kStride;
        const uint4 lo = *reinterpret_cast<const uint4*>(q + lane * 16);
        v = v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, 0, 0, 0, 0};
        if constexpr (kFp6) {
            const uint32_t* hi = reinterpret_cast<const uint32_t*>(q + 1024 + lane * 12);
            v[4] = (int)hi[0];
            v[5] = (int)hi[1];
        }
        sc = (int)(src.sc[((int64_t)(tile >> 2) * S + s) * 64 + lane] >> (8 * (tile & 3)));
    };
    v16f acc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int x = 0; x < 16; ++x) acc[i][x] = 0.0f;
    for (int s = s_lo; s < s_hi; ++s) {
        v8i w, a0, a1 = v8i{0, 0, 0, 0, 0, 0, 0, 0};
        int sw, s0, s1 = 0;
        load(p.w, t, s, w, sw);
        load(p.a, 0, s, a0, s0);
        if (mt > 1) load(p.a, 1, s, a1, s1);
        acc[0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a0, w, acc[0], FMT, FMT, 0, s0, 0, sw);
        if (mt > 1) acc[1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a1, w, acc[1], FMT, FMT, 0, s1, 0, sw);
    }
    // the 16 partial tiles, added in a fixed order: waves 8..15 hand theirs to waves 0..7
    if (wave >= 8) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int x = 0; x < 16; ++x) s_red[wave - 8][i][x][lane] = acc[i][x];
    }
    __syncthreads();
    if (wave < 8) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int x = 0; x < 16; ++x) s_red[wave][i][x][lane] += acc[i][x];
    }
    __syncthreads();
    const int n = t * 32 + c;
    for (int i = 0; i < mt; ++i) {
        const int x = wave;                                    // thread (x, lane) finishes one output per row tile
        float sum = 0.0f;
#pragma unroll
        for (int w8 = 0; w8 < 8; ++w8) sum += s_red[w8][i][x][lane];
        const int m = i * 32 + 8 * (x >> 2) + 4 * kh + (x & 3);
        if (m < p.M && n < p.N) {
            const int64_t o = (int64_t)m * p.ldc + n;
            if constexpr (BF16) static_cast<uint16_t*>(p.out)[o] = f32_to_bf16_rne_n(sum);
            else static_cast<float*>(p.out)[o] = sum;
        }
    }
}

// Split K: out = sum of the ranges' fp32 partial tiles, added in range order, converted once.
template <bool BF16>
__global__ __launch_bounds__(256) void native_reduce_kernel(const float* __restrict__ part, void* out, int M, int N,
                                                            int64_t ldc, int ksplit) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x, total = (int64_t)M * N;
    if (i >= total) return;
    float s = part[i];
    for (int z = 1; z < ksplit; ++z) s += part[(int64_t)z * total + i];
    const int64_t m = i / N, o = m * ldc + (i - m * N);
    if constexpr (BF16) static_cast<uint16_t*>(out)[o] = f32_to_bf16_rne_n(s);
    else static_cast<float*>(out)[o] = s;
}

inline int64_t up256(int64_t x) { return (x + 255) & ~(int64_t)255; }
// Workgroups per output tile: with at most a quarter as many tiles as compute units K is split in 2
// or 4 ranges (at half as many the partial tiles and the extra kernel cost what the split gains)
inline int native_ksplit(int64_t M, int64_t N, int64_t KB) {
    const int64_t tiles = ((M + 255) / 256) * ((N + 255) / 256), S = (KB + 1) / 2, cu = device_cu_count();
    int s = 1;
    while (s < 4 && tiles * s * 4 <= cu && S / (2 * s) >= 8) s *= 2;
    return s;
}
// One packed operand: [bits | scales], rows padded to 256, eight steps of slack behind each array.
struct OperandLayout { int64_t sc, total; };
inline OperandLayout operand_layout(int64_t rows, int64_t KB, bool fp6) {
    const int64_t S = (KB + 1) / 2, tiles = (rows + 255) / 256 * 8;
    OperandLayout l{};
    l.sc = up256((tiles * S + 8) * (fp6 ? 1792 : 1024));
    l.total = up256(l.sc + ((tiles / 4) * S + 8) * 256);
    return l;
}

}  // namespace

size_t native_packed_bytes(int64_t rows, int64_t K, bool fp6) {
    if (rows == 0 || K == 0) return 0;
    return (size_t)operand_layout(rows, K / kBlock, fp6).total;
}

size_t native_scale_offset(int64_t rows, int64_t K, bool fp6) {
    return (size_t)operand_layout(rows, K / kBlock, fp6).sc;
}

size_t native_splitk_bytes(int64_t M, int64_t N, int64_t K) {
    if (M == 0 || N == 0) return 0;
    const int s = native_ksplit(M, N, K / kBlock);
    return s > 1 ? (size_t)up256((int64_t)s * M * N * 4) : 0;
}

size_t gemm_native_workspace_bytes(int64_t M, int64_t N, int64_t K, bool fp6) {
    return native_packed_bytes(M, K, fp6) + native_packed_bytes(N, K, fp6) + native_splitk_bytes(M, N, K);
}

// Rewrite a quantized tensor in the matrix instruction's register order (see the file header).
int launch_native_pack(bool fp6, dfp4_tensor T, void* packed, size_t bytes, hipStream_t stream) {
    const int64_t KB = T.K / kBlock;
    if (T.rows == 0 || KB == 0) return DFP4_OK;
    if (T.rows >= (1 << 30) || KB >= (1 << 20)) return DFP4_ERR_SHAPE;
    const OperandLayout lay = operand_layout(T.rows, KB, fp6);
    if ((size_t)lay.total > bytes) return DFP4_ERR_WORKSPACE;
    const int S = (int)((KB + 1) / 2);
    PackParams q{};
    q.codes = T.codes; q.dial = T.dialect; q.expo = T.exponent;
    q.dst = PackedOperand{static_cast<uint8_t*>(packed), reinterpret_cast<uint32_t*>(static_cast<uint8_t*>(packed) + lay.sc)};
    q.rows = (int)T.rows; q.KB = (int)KB; q.S = S;
    dim3 gp((unsigned)((S + 3) / 4), (unsigned)((T.rows + 255) / 256 * 8));
    if (gp.y > 65535) return DFP4_ERR_SHAPE;
    if (fp6) hipLaunchKernelGGL((native_pack_kernel<kFmtFp6>), gp, dim3(256), 0, stream, q);
    else hipLaunchKernelGGL((native_pack_kernel<kFmtFp4>), gp, dim3(256), 0, stream, q);
    return check_launch();
}

// out = A * W^T from two packed operands ([M, K] and [N, K] before packing)
// `splitk` (may be null): native_splitk_bytes(M, N, K) bytes; without it K is never split
int launch_gemm_native_packed(bool fp6, const void* a_packed, const void* w_packed, int64_t M, int64_t N, int64_t K,
                              void* out, int out_dtype, int64_t ldc, void* splitk, size_t splitk_bytes,
                              hipStream_t stream) {
    const int64_t KB = K / kBlock;
    if (M == 0 || N == 0) return DFP4_OK;
    if (M >= (1 << 30) || N >= (1 << 30) || KB >= (1 << 20) || KB == 0 || ldc >= (1 << 27)) return DFP4_ERR_SHAPE;
    NativeParams p{};
    uint8_t* ap = static_cast<uint8_t*>(const_cast<void*>(a_packed));
    uint8_t* wp = static_cast<uint8_t*>(const_cast<void*>(w_packed));
    p.a = PackedOperand{ap, reinterpret_cast<uint32_t*>(ap + operand_layout(M, KB, fp6).sc)};
    p.w = PackedOperand{wp, reinterpret_cast<uint32_t*>(wp + operand_layout(N, KB, fp6).sc)};
    p.out = out; p.M = (int)M; p.N = (int)N; p.S = (int)((KB + 1) / 2); p.ldc = ldc;
    if (M <= 64) {
        // decode shapes: one workgroup per 32 W rows (A occupies the first one or two row tiles of its layout)
        p.ksplit = 1;
        dim3 gs((unsigned)((N + 31) / 32));
        const bool b16 = out_dtype == DFP4_BF16;
        if (fp6) {
            if (b16) hipLaunchKernelGGL((gemm_native_small_kernel<kFmtFp6, true>), gs, dim3(1024), 0, stream, p);
            else hipLaunchKernelGGL((gemm_native_small_kernel<kFmtFp6, false>), gs, dim3(1024), 0, stream, p);
        } else {
            if (b16) hipLaunchKernelGGL((gemm_native_small_kernel<kFmtFp4, true>), gs, dim3(1024), 0, stream, p);
            else hipLaunchKernelGGL((gemm_native_small_kernel<kFmtFp4, false>), gs, dim3(1024), 0, stream, p);
        }
        return check_launch();
    }
    p.ksplit = native_ksplit(M, N, KB);
    if (p.ksplit > 1 && (!splitk || splitk_bytes < native_splitk_bytes(M, N, K))) p.ksplit = 1;
    p.part = static_cast<float*>(splitk);
    // 256-row workgroups unless they would leave half of the compute units idle
    const int64_t tiles256 = ((M + 255) / 256) * ((N + 255) / 256);
    const bool half = tiles256 * p.ksplit * 2 <= device_cu_count() && M > 128;
    dim3 grid((unsigned)((N + 255) / 256), (unsigned)((M + (half ? 127 : 255)) / (half ? 128 : 256)), (unsigned)p.ksplit);
    if (grid.y > 65535) return DFP4_ERR_SHAPE;
    const bool bf16 = out_dtype == DFP4_BF16 && p.ksplit == 1;     // partial tiles are fp32
#define DFP4_NATIVE_LAUNCH(F, B)                                                                         \
    do {                                                                                                 \
        if (half) hipLaunchKernelGGL((gemm_native_kernel<F, B, 2>), grid, dim3(256), 0, stream, p);      \
        else hipLaunchKernelGGL((gemm_native_kernel<F, B, 4>), grid, dim3(256), 0, stream, p);           \
    } while (0)
    if (fp6) {
        if (bf16) DFP4_NATIVE_LAUNCH(kFmtFp6, true); else DFP4_NATIVE_LAUNCH(kFmtFp6, false);
    } else {
        if (bf16) DFP4_NATIVE_LAUNCH(kFmtFp4, true); else DFP4_NATIVE_LAUNCH(kFmtFp4, false);
    }
#undef DFP4_NATIVE_LAUNCH
    if (p.ksplit > 1) {
        const unsigned gr = (unsigned)((M * N + 255) / 256);
        if (out_dtype == DFP4_BF16)
            hipLaunchKernelGGL((native_reduce_kernel<true>), dim3(gr), dim3(256), 0, stream, p.part, out, p.M, p.N, ldc, p.ksplit);
        else
            hipLaunchKernelGGL((native_reduce_kernel<false>), dim3(gr), dim3(256), 0, stream, p.part, out, p.M, p.N, ldc, p.ksplit);
    }
    return check_launch();
}

}  // namespace dfp4
