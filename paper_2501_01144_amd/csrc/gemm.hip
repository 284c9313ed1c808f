// Block-scaled integer GEMM on DialectFP4 / MXFP4 operands for gfx950
// (paper Section 3.3): out = A * W^T with
//   out[m,n] = sum_kb 2^(ea[m,kb]+ew[n,kb]-2) * sum_{k in kb} (+-ua)(+-uw).
//
// The paper accumulates the products of one block pair as integers and
// applies the exponent sum once per block pair.  On gfx950 the per-block
// floating-point step would dominate (one convert + scale + add per output
// and block on the vector ALU against 32 int8 MACs per output and block on
// the matrix core), so this kernel moves the exponents into the operands:
//
//   * every row of A and of W gets a reference exponent ref = its smallest
//     block exponent; block (row, kb) has offset delta = e - ref >= 0;
//   * delta = 4 c + d.  The shift d in 0..3 is folded into the int8 operand
//     (|u| <= 15, so |u << d| <= 120); the "class" c selects a pass;
//   * passes run from the highest class down, and between classes the int32
//     accumulators are shifted left by 4 (Horner's scheme), so that all of K
//     is summed exactly in ONE int32 accumulator per output and the only
//     rounding is the final int32 -> fp32 conversion, scaled by
//     2^(refA[m] + refW[n] - 2).
//   Both operands have classes.  A block is visited once for every pair (class
//   present among the tile's 512 rows of A, class present among its 128 rows of
//   W) -- rows of other classes contribute zeros -- and the pair's class sum is
//   the number of shifts the product still receives; sums above 2 cannot be
//   taken.  With activations that have outlier channels, that is a second visit
//   for the few outlier blocks.
//
// Kernels:
//   gemm_prep_kernel     the per-operand part, once per call (dfp4_gemm) or once per
//                        tensor (dfp4_gemm_prepare).  A: per-row reference exponents,
//                        per-(512 rows, block) class masks, and A expanded to
//                        pre-shifted int8 in MFMA fragment order (A is the small
//                        operand; W stays 4-bit in HBM).  W: per-row reference
//                        exponents, per-(128 rows, block) class masks, and per class
//                        and block one dword naming the block's (dialect, shift)
//                        table, or the all-zero table for blocks of another class;
//   gemm_fast_kernel     512 x 128 outputs per workgroup, 4 waves, each wave
//                        128 x 128 with 256 accumulator registers (one wave per
//                        SIMD).  A fragments are private to a wave and come by
//                        global loads straight into registers, two steps ahead;
//                        each wave expands its own 32 rows of W from 4-bit codes
//                        (v_perm_b32 lookups) and shares the int8 result through
//                        LDS.  A lone wave issues one instruction per 4 cycles or
//                        so; the whole main loop is generated assembly that places
//                        the few non-MFMA instructions per MFMA in its shadow.
//                        With few output tiles K is split between workgroups; the
//                        last of a tile's workgroups to finish adds the others'
//                        exact int32 sums.  A tile whose exponents spread too far
//                        (or whose int32 sum could overflow) is computed by the same
//                        workgroup with one fp32 scale-and-add per block;
//   gemm_rows_kernel     the same exact scheme for at most 64 rows of A on prepared
//                        operands (decode shapes): 32 x 32 outputs per workgroup, its 16
//                        (or 8) waves share K; no list of visits, the class pairs other
//                        than (0, 0) are added with their weights afterwards;
//   gemm_small_kernel    at most 64 rows of A, nothing prepared: the exact scheme with the tile's
//                        own reference exponents found in the kernel; per-block fp32 flush
//                        for a tile whose exponents spread too far;
//   gemm_block_kernel    whole products with K > 16384: per-block fp32 flush;
//   gemm_block16_kernel  operands quantized in blocks of 16: per-block fp32 flush.
//
// The order of the elements inside an MFMA operand does not matter as long
// as A and W use the same order; both sides go through unpack8() below.
#include <type_traits>
#include "common.h"
#include "formatbook.h"
#include "quant_pass.h"
#include "gemm_step_asm.inc"

namespace dfp4 {

// [dialect][shift] -> {magnitudes lo, hi, negated magnitudes lo, hi}, bytes u << shift
struct ShiftedBook { uint32_t w[kDialects][4][4]; };
constexpr ShiftedBook make_shifted_book() {
    ShiftedBook b{};
    for (int d = 0; d < kDialects; ++d)
        for (int s = 0; s < 4; ++s)
            for (int j = 0; j < 8; ++j) {
                const uint32_t u = (uint32_t)kBook[d][j] << s;
                b.w[d][s][j / 4] |= u << (8 * (j % 4));
                b.w[d][s][2 + j / 4] |= ((256u - u) & 0xffu) << (8 * (j % 4));
            }
    return b;
}
__device__ const ShiftedBook g_shifted_book = make_shifted_book();

namespace {

// Results leave the kernel once and are not read again by it: stored with the non-temporal hint so
// that they do not push the operands other workgroups still need out of the caches.
#if defined(DFP4_TIMING_NO_OUT_STORES)   // timing experiments only: results are computed and dropped
__device__ int g_timing_store_results = 0;
#define DFP4_OUT_STORE(PTR, VAL) do { if (g_timing_store_results) *(PTR) = (VAL); } while (0)
#elif defined(DFP4_PLAIN_OUT_STORES)
#define DFP4_OUT_STORE(PTR, VAL) (*(PTR) = (VAL))
#else
#define DFP4_OUT_STORE(PTR, VAL) __builtin_nontemporal_store((VAL), (PTR))
#endif

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kTileM = 512, kTileN = 128;   // fast kernel: outputs per workgroup
constexpr int kGroups = kTileM / 32;        // 32-row groups per tile
constexpr int kMaxKB = 512;           // fast path: K <= 16384
constexpr int kMaxClass = 2;          // classes 0..2, i.e. exponent offsets 0..11
constexpr int kIntBound = 4660;       // n0 + 16 n1 + 256 n2 <= 2^31 / (32 * 120 * 120)
constexpr int kBBufBytes = 8 * 1024;  // int8 W operands of one step: 4 column tiles x 2 x 1 KiB
constexpr int kRqPitch = 136;         // bf16 per staged output row (128 + 8: rows stay 16-byte aligned)
constexpr int kVisitPad = 12;         // padding visits after the last one (the loop looks 5 steps ahead)
constexpr int kClassPairs = (kMaxClass + 1) * (kMaxClass + 2) / 2;   // (class of A, class of W) with sum <= kMaxClass
constexpr int kVisitCap = kClassPairs * kMaxKB + 2 * (kMaxClass + 1) + kVisitPad + 4;
constexpr uint32_t kZeroTab = kDialects * 4 * 16;   // byte offset of the all-zero table behind the shifted book in LDS
constexpr int kMaxSplitTiles = 2048;  // arrival counters per prepared A: K is split only below this many tiles

struct GemmParams {
    const uint8_t *a_codes, *a_dial, *a_exp, *w_codes, *w_dial, *w_exp;
    void* out;
    int M, N, KB;
    int64_t ldc, strideA_rows, strideW_rows, strideC;
    // prepared operands (per batch entry: base + batch * stride) and their regions
    uint8_t* a_prep;
    uint8_t* w_prep;
    int64_t a_prep_stride, w_prep_stride;
    int64_t off_refa, off_mask, off_cnt, off_a8;      // inside a prepared A
    int64_t off_refw, off_wmask, off_wmeta, off_wcodes;   // inside a prepared W
    uint32_t wmeta_cls_stride;                        // bytes between the table dwords of two classes
    // exact int32 partial tiles of workgroups that share an output tile (split K)
    int* part;
    int64_t part_stride;              // ints per batch entry
    int tiles_m, tiles_n;             // 512 x 128 output tiles
    int ksplit;                       // workgroups sharing one output tile (each takes a range of K)
    // requantizing epilogue: the quantized [M, N] output (blocks of 32 along N)
    uint32_t* q_codes;
    uint8_t *q_dial, *q_exp;
};

__host__ __device__ inline int64_t align256(int64_t x) { return (x + 255) & ~(int64_t)255; }

// Prepared A [M, K] (see gemm_prep_kernel): per-row reference exponents (rows padded to 512), one
// class mask per (512-row tile, block), arrival counters of the tiles whose K is split, and the
// operand expanded to pre-shifted int8 in MFMA fragment order:
// [class][tile][32-row group][block 0..KB][1 KiB]; block KB of class 0 is all zeros.
struct PrepALayout { int64_t off_refa, off_mask, off_cnt, off_a8, total; };
inline PrepALayout prep_a_layout(int64_t M, int64_t KB) {
    const int64_t tm = (M + kTileM - 1) / kTileM;
    PrepALayout l{};
    l.off_refa = 0;
    l.off_mask = align256(tm * kTileM);
    l.off_cnt = align256(l.off_mask + tm * KB);
    l.off_a8 = align256(l.off_cnt + (int64_t)(kMaxSplitTiles + 1) * 4);    // + the count of declined tiles
    l.total = align256(l.off_a8 + (kMaxClass + 1) * tm * kGroups * (KB + 1) * 1024);
    return l;
}
// Prepared W [N, K]: per-row reference exponents (rows padded to 128), one class mask per
// (128-row tile, block), per class and block one dword naming the block's (dialect, shift)
// table -- or the all-zero table where the block is of another class -- and a copy of the 4-bit
// codes.  Table dwords and codes are laid out by 32-row group and block, [group][block][row]
// (codes: 16 bytes per row and block; dwords: [class][group][block][row]), so that what a wave
// loads for one block of its 32 rows is one contiguous run of 512 (128) bytes: four (one) cache
// lines instead of 32.  Rows of the last group beyond N carry the all-zero table.
struct PrepWLayout { int64_t off_refw, off_wmask, off_wmeta, off_wcodes, total; };
inline PrepWLayout prep_w_layout(int64_t N, int64_t KB) {
    const int64_t tn = (N + kTileN - 1) / kTileN, rows = tn * kTileN;
    PrepWLayout l{};
    l.off_refw = 0;
    l.off_wmask = align256(rows);
    l.off_wmeta = align256(l.off_wmask + tn * KB);
    l.off_wcodes = align256(l.off_wmeta + (kMaxClass + 1) * rows * KB * 4);
    l.total = align256(l.off_wcodes + rows * KB * 16);
    return l;
}
// Workgroups per output tile: when there are fewer tiles than compute units, K is split
// between 2, 4 or 8 workgroups; the last of them to finish adds the others' exact int32 sums.
inline int choose_ksplit(int64_t tiles, int64_t KB) {
    const int64_t cu = device_cu_count();
    int s = 1;
    while (s < 8 && tiles * s * 2 <= cu && KB / (2 * s) >= 16) s *= 2;
    return tiles <= kMaxSplitTiles ? s : 1;
}
inline int64_t partial_bytes(int64_t M, int64_t N, int64_t KB, int64_t batch) {
    const int64_t tiles = ((M + kTileM - 1) / kTileM) * ((N + kTileN - 1) / kTileN);
    const int s = choose_ksplit(tiles * batch, KB);
    return s > 1 ? align256((int64_t)s * tiles * kTileM * kTileN * 4) : 0;
}
inline bool takes_small_kernel(int64_t M, int64_t KB) { return M <= 64 && KB > 0 && KB <= 512; }
inline bool takes_fast_kernel(int64_t M, int64_t KB) { return !takes_small_kernel(M, KB) && KB > 0 && KB <= kMaxKB; }

// 8 codes (one dword) -> 8 signed int8 through one dialect table:
// returns the even-numbered elements in one dword and the odd ones in another.
// Magnitudes and negated magnitudes are looked up with v_perm_b32 (selector =
// 3-bit index); the per-byte choice between them uses v_perm_b32's
// sign-replication selectors (8..11 = 0x00 / 0xff from bit 7 of bytes 1, 3, 5, 7
// of the source pair), which turn the code's sign bits into byte masks.
__device__ __forceinline__ void unpack8(uint32_t c, uint32_t plo, uint32_t phi, uint32_t nlo,
                                        uint32_t nhi, uint32_t& even, uint32_t& odd) {
    const uint32_t ie = c & 0x07070707u, io = (c >> 4) & 0x07070707u;
    const uint32_t pe = __builtin_amdgcn_perm(phi, plo, ie), po = __builtin_amdgcn_perm(phi, plo, io);
    const uint32_t ne = __builtin_amdgcn_perm(nhi, nlo, ie), no = __builtin_amdgcn_perm(nhi, nlo, io);
    // result byte k <- sign of byte k of x: bytes 1, 3 come from x, bytes 0, 2 from x << 8
    constexpr uint32_t kSignSel = 0x090b080au;
    const uint32_t c4 = c << 4;                                   // index sign bit 3 -> bit 7
    const uint32_t mo = __builtin_amdgcn_perm(c << 8, c, kSignSel);
    const uint32_t me = __builtin_amdgcn_perm(c4 << 8, c4, kSignSel);
    even = (ne & me) | (pe & ~me);
    odd = (no & mo) | (po & ~mo);
}

__device__ __forceinline__ v4i unpack16(uint32_t c0, uint32_t c1, uint4 tab) {
    uint32_t a, b, e, f;
    unpack8(c0, tab.x, tab.y, tab.z, tab.w, a, b);
    unpack8(c1, tab.x, tab.y, tab.z, tab.w, e, f);
    return v4i{(int)a, (int)b, (int)e, (int)f};
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// ---------------------------------------------------------------------------
// Prepass (one launch, 1024 threads per workgroup).  Workgroups [0, n_a) expand A,
// the others compute the per-row statistics of W.
//
// A workgroup = (512-row tile, chunk of 8 blocks); wave w owns the tile's 32-row
// group w.  Each wave first finds its rows' reference exponents (smallest block
// exponent of the whole row; the chunk-0 workgroup publishes them), then the
// classes present in each block of the chunk among all 512 rows (one 32-bit word
// in LDS: bit 4*block + class), then writes, for every class present, the 1 KiB
// fragment of its group: rows of other classes contribute zeros.  The 4-bit codes
// are read as whole 128-byte lines (8 lanes per row) and redistributed through LDS
// to the fragment order (lane = (t, row): elements 16t .. 16t+15 of the block).
//
// W rows: reference exponent, per class and block one table offset (dword), and the classes
// present in each block among the 128 rows of a tile.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int min_bytes(uint32_t x) {
    return min(min((int)(x & 0xffu), (int)((x >> 8) & 0xffu)), min((int)((x >> 16) & 0xffu), (int)(x >> 24)));
}
__device__ __forceinline__ int max_bytes(uint32_t x) {
    return max(max((int)(x & 0xffu), (int)((x >> 8) & 0xffu)), max((int)((x >> 16) & 0xffu), (int)(x >> 24)));
}
// up to 8 bytes starting at q (the first n are read), little-endian in a 64-bit word
__device__ __forceinline__ uint64_t load_bytes8(const uint8_t* q, int n) {
    if (n == 8) {
        uint64_t v;
        __builtin_memcpy(&v, q, 8);                   // no alignment assumed: the compiler picks the access
        return v;
    }
    uint64_t v = 0;
    for (int i = 0; i < n; ++i) v |= (uint64_t)q[i] << (8 * i);
    return v;
}

template <bool MX>
__global__ __launch_bounds__(1024) void gemm_prep_kernel(GemmParams p, int n_a, int chunks_a) {
    constexpr int kPitch = 144;                       // LDS bytes per row of staged codes (8 blocks = 128 + pad)
    __shared__ __attribute__((aligned(16))) uint8_t s_codes[16][32 * kPitch];
    __shared__ __attribute__((aligned(16))) uint32_t s_tab[kDialects * 16];
    __shared__ uint32_t s_present;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t bz = blockIdx.z;
    uint8_t* ap = p.a_prep + bz * p.a_prep_stride;    // only touched by the A workgroups
    uint8_t* wp = p.w_prep + bz * p.w_prep_stride;    // only touched by the W workgroups
    const int KB = p.KB;

    if ((int)blockIdx.x >= n_a) {
        // ---- W: a workgroup = (128-row tile, chunk of 64 blocks), 8 lanes per row (lane s takes blocks
        // s, s + 8, ...).  Every workgroup finds the rows' reference exponents from all of K.
        __shared__ uint32_t s_wmask[64];
        const int chunks_w = (KB + 63) / 64;
        const int tile = ((int)blockIdx.x - n_a) / chunks_w, chunk = ((int)blockIdx.x - n_a) % chunks_w;
        const int kc = chunk * 64, ke = min(KB, kc + 64);
        const int row = tile * kTileN + (tid >> 3), seg = tid & 7;
        const bool valid = row < p.N;
        const int64_t base = (bz * p.strideW_rows + min(row, p.N - 1)) * KB;
        const uint8_t* we = p.w_exp + base;
        const uint8_t* wd = MX ? nullptr : p.w_dial + base;
        if (tid < 64) s_wmask[tid] = 0;
        int mn = 255;
        for (int kb = seg; kb < KB; kb += 8) mn = min(mn, (int)we[kb]);
        mn = min(mn, __shfl_xor(mn, 1));
        mn = min(mn, __shfl_xor(mn, 2));
        mn = min(mn, __shfl_xor(mn, 4));
        __syncthreads();
        {
            if (valid && seg == 0 && chunk == 0) wp[p.off_refw + row] = (uint8_t)mn;
            // [group of 32 rows][block][row]: this row's slot within block 0 of its group
            const int64_t slot = (int64_t)(row >> 5) * KB * 32 + (row & 31);
            uint32_t* wmeta = reinterpret_cast<uint32_t*>(wp + p.off_wmeta) + slot;
            uint4* wct = reinterpret_cast<uint4*>(wp + p.off_wcodes) + slot;
            const uint4* wcs = reinterpret_cast<const uint4*>(p.w_codes) + base;
            const int64_t cls_stride = (int64_t)p.tiles_n * kTileN * KB;     // dwords
            for (int kb = kc + seg; kb < ke; kb += 8) {
                uint32_t cls = kMaxClass + 2, tab = kZeroTab;               // rows beyond N: the all-zero table
                if (valid) {
                    const uint32_t delta = (uint32_t)we[kb] - (uint32_t)mn;
                    const uint32_t dd = MX ? 7u : ((uint32_t)wd[kb] & 15u);
                    cls = min(delta >> 2, (uint32_t)kMaxClass + 1u);
                    tab = (dd * 4u + (delta & 3u)) * 16u;
                    wct[(int64_t)kb * 32] = wcs[kb];
                    atomicOr(&s_wmask[kb - kc], 1u << cls);
                }
#pragma unroll
                for (uint32_t c = 0; c <= (uint32_t)kMaxClass; ++c)
                    wmeta[c * cls_stride + (int64_t)kb * 32] = cls == c ? tab : kZeroTab;
            }
        }
        __syncthreads();
        if (tid < ke - kc) wp[p.off_wmask + (int64_t)tile * KB + kc + tid] = (uint8_t)s_wmask[tid];
        return;
    }

    // ---- A: tile, chunk of 8 blocks
    const int tile = (int)blockIdx.x / chunks_a, chunk = (int)blockIdx.x % chunks_a;
    const int kc = chunk * 8, nk = min(8, KB - kc);
    for (int i = tid; i < kDialects * 16; i += 1024) s_tab[i] = (&g_shifted_book.w[0][0][0])[i];
    if (tid == 0) s_present = 0;
    if (blockIdx.x == 0) {
        // arrival counters of output tiles whose K is split between workgroups: zero here; the
        // workgroup that arrives last at a tile puts its counter back to zero
        uint32_t* cnt = reinterpret_cast<uint32_t*>(ap + p.off_cnt);
        for (int i = tid; i <= kMaxSplitTiles; i += 1024) cnt[i] = 0;     // the last one counts declined tiles
    }
    __syncthreads();

    const int r = lane & 31, t = lane >> 5;
    const int row0 = tile * kTileM + wave * 32;
    const bool group_valid = row0 < p.M;              // wave-uniform
    int cls[8], sh[8];
    uint64_t d8 = 0x0707070707070707ull;
    if (group_valid) {
        // codes: lane (row q*8 + lane/8, block lane%8) reads one block; 8 lanes cover a 128-byte line
        uint4 craw[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int k8 = lane & 7;
            const int64_t rq = bz * p.strideA_rows + min(row0 + q * 8 + (lane >> 3), p.M - 1);
            craw[q] = k8 < nk ? *reinterpret_cast<const uint4*>(p.a_codes + (rq * KB + kc + k8) * 16)
                              : make_uint4(0, 0, 0, 0);
        }
        const int64_t arow = bz * p.strideA_rows + min(row0 + r, p.M - 1);
        const uint64_t e8 = load_bytes8(p.a_exp + arow * KB + kc, nk);
        if (!MX) d8 = load_bytes8(p.a_dial + arow * KB + kc, nk);
        // reference exponent of the row: lane (t, r) scans every other 16-byte piece
        int mn = 255;
        const uint8_t* erow = p.a_exp + arow * KB;
        const int n16 = KB >> 4;
        for (int i0 = 0; i0 < n16; i0 += 8) {
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                __builtin_memcpy(&v[u], erow + 16 * min(i0 + 2 * u + t, n16 - 1), 16);   // no alignment assumed
#pragma unroll
            for (int u = 0; u < 4; ++u)
                mn = min(mn, min(min(min_bytes(v[u].x), min_bytes(v[u].y)), min(min_bytes(v[u].z), min_bytes(v[u].w))));
        }
        for (int i = n16 * 16 + t; i < KB; i += 2) mn = min(mn, (int)erow[i]);
        mn = min(mn, __shfl_xor(mn, 32));
        const bool row_valid = row0 + r < p.M;
        if (chunk == 0 && t == 0) ap[p.off_refa + row0 + r] = row_valid ? (uint8_t)mn : (uint8_t)0;
        uint32_t word = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int delta = (int)((e8 >> (8 * k)) & 0xffu) - mn;
            const bool on = k < nk && row_valid;
            cls[k] = on ? min(delta >> 2, kMaxClass + 1) : -1;
            sh[k] = on ? (delta & 3) : 0;
            if (on) word |= 1u << (4 * k + cls[k]);
        }
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) word |= (uint32_t)__shfl_xor((int)word, s);
        if (lane == 0) atomicOr(&s_present, word);
#pragma unroll
        for (int q = 0; q < 4; ++q)
            *reinterpret_cast<uint4*>(&s_codes[wave][(q * 8 + (lane >> 3)) * kPitch + (lane & 7) * 16]) = craw[q];
    } else if (chunk == 0 && t == 0) {
        ap[p.off_refa + row0 + r] = 0;                // padding rows of the last tile
    }
    __syncthreads();
    const uint32_t present = s_present;
    if (wave == 0 && lane < nk) ap[p.off_mask + (int64_t)tile * KB + kc + lane] = (uint8_t)((present >> (4 * lane)) & 15u);
    const int64_t grp = (int64_t)tile * kGroups + wave;
    if (chunk == 0)                                   // the all-zero block (index KB) of this group, class 0
        *reinterpret_cast<uint4*>(ap + p.off_a8 + (grp * (KB + 1) + KB) * 1024 + lane * 16) = make_uint4(0, 0, 0, 0);
    if (!group_valid) return;
    const int64_t cls_stride = (int64_t)p.tiles_m * kGroups * (KB + 1) * 1024;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        if (k >= nk) break;
        const uint2 c = *reinterpret_cast<const uint2*>(&s_codes[wave][r * kPitch + k * 16 + t * 8]);
        const uint32_t dial = (uint32_t)(d8 >> (8 * k)) & 15u;
        const uint4 tab = *reinterpret_cast<const uint4*>(&s_tab[(dial * 4 + sh[k]) * 4]);
        const v4i data = unpack16(c.x, c.y, tab);
        uint8_t* dst = ap + p.off_a8 + (grp * (KB + 1) + kc + k) * 1024 + t * 512 + r * 16;
#pragma unroll
        for (int cc = 0; cc <= kMaxClass; ++cc)
            if ((present >> (4 * k + cc)) & 1u)
                *reinterpret_cast<v4i*>(dst + cc * cls_stride) = cls[k] == cc ? data : v4i{0, 0, 0, 0};
    }
}

// ---------------------------------------------------------------------------
// Per-block flush (always correct): 128 x 128 outputs per workgroup of 256 threads,
// operands straight from global memory, one fp32 scale-and-add per block as in the
// paper's MAC (Section 3.3).  Used by gemm_block_kernel for products the single-
// accumulator kernel does not take, and by that kernel itself for tiles it declines.
// ---------------------------------------------------------------------------
template <bool MX, bool BF16>
__device__ __forceinline__ void block_flush_tile(const GemmParams& p, int64_t bz, int by, int bx,
                                                 uint8_t (&s_exp)[2][256]) {
    const int KB = p.KB;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = by * 128, n0 = bx * 128;
    const int64_t a_row0 = bz * p.strideA_rows, w_row0 = bz * p.strideW_rows;
    const int half = lane >> 5, l32 = lane & 31;

    int64_t a_row[2], w_row[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        a_row[i] = a_row0 + min(m0 + wm * 64 + i * 32 + l32, p.M - 1);
        w_row[i] = w_row0 + min(n0 + wn * 64 + i * 32 + l32, p.N - 1);
    }
    const int t = threadIdx.x;
    const int64_t e_row = t < 128 ? a_row0 + min(m0 + t, p.M - 1) : w_row0 + min(n0 + t - 128, p.N - 1);
    const uint8_t* e_src = (t < 128 ? p.a_exp : p.w_exp) + e_row * KB;

    float acc[2][2][16];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int x = 0; x < 16; ++x) acc[i][j][x] = 0.0f;

    // operands of one block, loaded one iteration ahead so that the memory latency of block kb + 1
    // passes behind the arithmetic of block kb
    struct BlockOperands { uint2 ca[2], cw[2]; uint32_t da[2], dw[2], e; };
    auto load_block = [&](int kb) {
        BlockOperands o;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            o.ca[i] = *reinterpret_cast<const uint2*>(p.a_codes + (a_row[i] * KB + kb) * 16 + half * 8);
            o.cw[i] = *reinterpret_cast<const uint2*>(p.w_codes + (w_row[i] * KB + kb) * 16 + half * 8);
            o.da[i] = MX ? 7u : ((uint32_t)p.a_dial[a_row[i] * KB + kb] & 15u);
            o.dw[i] = MX ? 7u : ((uint32_t)p.w_dial[w_row[i] * KB + kb] & 15u);
        }
        o.e = e_src[kb];
        return o;
    };
    BlockOperands nxt{};
    if (KB > 0) nxt = load_block(0);              // K = 0: nothing to read, the outputs are zeros
    for (int kb = 0; kb < KB; ++kb) {
        const BlockOperands cur = nxt;
        if (kb + 1 < KB) nxt = load_block(kb + 1);
        uint8_t* se = s_exp[kb & 1];
        se[t] = (uint8_t)cur.e;
        v4i a[2], b[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            a[i] = unpack16(cur.ca[i].x, cur.ca[i].y, *reinterpret_cast<const uint4*>(g_shifted_book.w[cur.da[i]][0]));
            b[i] = unpack16(cur.cw[i].x, cur.cw[i].y, *reinterpret_cast<const uint4*>(g_shifted_book.w[cur.dw[i]][0]));
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                v16i pr = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                pr = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], pr, 0, 0, 0);
                const int ew = se[128 + wn * 64 + j * 32 + l32];
#pragma unroll
                for (int x = 0; x < 16; ++x) {
                    const int row = 8 * (x >> 2) + 4 * half + (x & 3);
                    const int ea = se[wm * 64 + i * 32 + row];
                    acc[i][j][x] += ldexpf((float)pr[x], ea + ew - 256);
                }
            }
    }

#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + wn * 64 + j * 32 + l32;
#pragma unroll
            for (int x = 0; x < 16; ++x) {
                const int m = m0 + wm * 64 + i * 32 + 8 * (x >> 2) + 4 * half + (x & 3);
                if (m < p.M && n < p.N) {
                    const int64_t o = bz * p.strideC + (int64_t)m * p.ldc + n;
                    if constexpr (BF16)
                        static_cast<uint16_t*>(p.out)[o] = f32_to_bf16_rne(acc[i][j][x]);
                    else
                        static_cast<float*>(p.out)[o] = acc[i][j][x];
                }
            }
        }
}

// Requantizing GEMM, tiles that went through the per-block flush: quantize the 128 x 128 bf16
// results the workgroup has just written to the temporary `p.out` (16 rows x 4 blocks per sweep,
// 4 lanes per block).  lds_s / lds_q: the quantizer's tables.
template <bool MX>
__device__ __forceinline__ void quantize_flushed_piece(const GemmParams& p, int64_t bz, int by, int bx,
                                                       const uint8_t* lds_s, const uint8_t* lds_q) {
    __threadfence_block();
    __syncthreads();
    const int tid = threadIdx.x;
    const int nb_row = p.N / kBlock;
    const uint16_t* src = static_cast<const uint16_t*>(p.out) + bz * p.strideC;
    for (int sweep = 0; sweep < 8; ++sweep) {
        const int q = tid >> 2, sub = tid & 3;
        const int m = by * 128 + sweep * 16 + (q >> 2), nb = bx * 4 + (q & 3);
        const bool valid = m < p.M && nb < nb_row;      // the same for the 4 lanes of a block
        uint4 wv = make_uint4(0, 0, 0, 0);
        if (valid) wv = *reinterpret_cast<const uint4*>(src + (int64_t)m * p.ldc + nb * kBlock + sub * 8);
        uint32_t code, eb, dl = 0;
        if constexpr (MX) mxfp4_pass(wv, lds_q, code, eb);
        else dfp4_pass(wv, lds_s, lds_q, code, eb, dl);
        if (valid) {
            const size_t blk = (size_t)(bz * p.M + m) * nb_row + nb;
            p.q_codes[blk * 4 + sub] = code;
            if (sub == 0) {
                p.q_exp[blk] = (uint8_t)eb;
                if constexpr (!MX) p.q_dial[blk] = (uint8_t)dl;
            }
        }
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------
// Operands quantized in blocks of 16 (Section 4.2, Table 3: smaller blocks for the sublayers most
// sensitive to quantization, possibly mixed with blocks of 32 on the other operand): the paper's
// MAC with one exponent pair per pair of 16-element blocks.  A 32 x 32 x 32 matrix instruction adds
// up both halves of a 32-element stretch, so each stretch takes two of them, one per half with the
// other half's lanes zeroed, each followed by its own fp32 scale-and-add.  128 x 128 outputs per
// workgroup, operands straight from global memory one stretch ahead.  a16 / w16: that operand's
// dialect and exponent arrays hold one entry per 16 elements (otherwise per 32).
// ---------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(256) void gemm_block16_kernel(GemmParams p, int a16, int w16) {
    __shared__ uint8_t s_exp[2][512];                  // [buffer][A rows x 2 halves | W rows x 2 halves]
    const int KB = p.KB;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * 128, n0 = blockIdx.x * 128;
    const int half = lane >> 5, l32 = lane & 31;
    int64_t a_row[2], w_row[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        a_row[i] = min(m0 + wm * 64 + i * 32 + l32, p.M - 1);
        w_row[i] = min(n0 + wn * 64 + i * 32 + l32, p.N - 1);
    }
    // metadata index of (row, stretch kb, half h): per 16 elements (row * KB + kb) * 2 + h, per 32 row * KB + kb
    auto meta_a = [&](int64_t row, int kb, int h) { return a16 ? (row * KB + kb) * 2 + h : row * KB + kb; };
    auto meta_w = [&](int64_t row, int kb, int h) { return w16 ? (row * KB + kb) * 2 + h : row * KB + kb; };
    const int t = threadIdx.x;
    const bool t_is_a = t < 128;
    const int64_t e_row = t_is_a ? min(m0 + t, p.M - 1) : min(n0 + t - 128, p.N - 1);

    float acc[2][2][16];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int x = 0; x < 16; ++x) acc[i][j][x] = 0.0f;

    struct Stretch { uint2 ca[2], cw[2]; uint32_t da[2], dw[2], e0, e1; };
    auto load_stretch = [&](int kb) {
        Stretch o;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            o.ca[i] = *reinterpret_cast<const uint2*>(p.a_codes + (a_row[i] * KB + kb) * 16 + half * 8);
            o.cw[i] = *reinterpret_cast<const uint2*>(p.w_codes + (w_row[i] * KB + kb) * 16 + half * 8);
            o.da[i] = (uint32_t)p.a_dial[meta_a(a_row[i], kb, half)] & 15u;
            o.dw[i] = (uint32_t)p.w_dial[meta_w(w_row[i], kb, half)] & 15u;
        }
        o.e0 = t_is_a ? p.a_exp[meta_a(e_row, kb, 0)] : p.w_exp[meta_w(e_row, kb, 0)];
        o.e1 = t_is_a ? p.a_exp[meta_a(e_row, kb, 1)] : p.w_exp[meta_w(e_row, kb, 1)];
        return o;
    };
    Stretch nxt{};
    if (KB > 0) nxt = load_stretch(0);
    for (int kb = 0; kb < KB; ++kb) {
        const Stretch cur = nxt;
        if (kb + 1 < KB) nxt = load_stretch(kb + 1);
        uint8_t* se = s_exp[kb & 1];
        se[2 * t] = (uint8_t)cur.e0;
        se[2 * t + 1] = (uint8_t)cur.e1;
        v4i a[2], b[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            a[i] = unpack16(cur.ca[i].x, cur.ca[i].y, *reinterpret_cast<const uint4*>(g_shifted_book.w[cur.da[i]][0]));
            b[i] = unpack16(cur.cw[i].x, cur.cw[i].y, *reinterpret_cast<const uint4*>(g_shifted_book.w[cur.dw[i]][0]));
        }
        __syncthreads();
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                // this half's 16 elements only: the lanes that hold the other half multiply zeros
                const v4i ah = half == hh ? a[i] : v4i{0, 0, 0, 0};
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    v16i pr = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                    pr = __builtin_amdgcn_mfma_i32_32x32x32_i8(ah, b[j], pr, 0, 0, 0);
                    const int ew = se[2 * (128 + wn * 64 + j * 32 + l32) + hh];
#pragma unroll
                    for (int x = 0; x < 16; ++x) {
                        const int row = 8 * (x >> 2) + 4 * half + (x & 3);
                        const int ea = se[2 * (wm * 64 + i * 32 + row) + hh];
                        acc[i][j][x] += ldexpf((float)pr[x], ea + ew - 256);
                    }
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + wn * 64 + j * 32 + l32;
#pragma unroll
            for (int x = 0; x < 16; ++x) {
                const int m = m0 + wm * 64 + i * 32 + 8 * (x >> 2) + 4 * half + (x & 3);
                if (m < p.M && n < p.N) {
                    const int64_t o = (int64_t)m * p.ldc + n;
                    if constexpr (BF16)
                        static_cast<uint16_t*>(p.out)[o] = f32_to_bf16_rne(acc[i][j][x]);
                    else
                        static_cast<float*>(p.out)[o] = acc[i][j][x];
                }
            }
        }
}

// ---------------------------------------------------------------------------
// Fast kernel: 512 x 128 outputs per workgroup, one int32 accumulator per output.
// Wave w owns rows 128w .. 128w+127 and all 128 columns (16 accumulator tiles of
// 32 x 32: tile i = 4 * gi + n is rows 32 gi .., columns 32 n ..).
// ---------------------------------------------------------------------------
template <bool MX, bool BF16, bool RQ>
__global__ __launch_bounds__(256, 1) void gemm_fast_kernel(GemmParams p) {
    // int8 W operands of a pair of blocks: [column tile n][t][lane][16 bytes]; three buffers in rotation
    __shared__ __attribute__((aligned(16))) uint8_t s_b[3][kBBufBytes];
    // requantizing epilogue only: quantizer tables and, per wave, 64 rows x 128 columns of bf16 results
    __shared__ __attribute__((aligned(16))) uint8_t s_rq_q[RQ ? (MX ? 64 : kDialects * 1024) : 16];
    __shared__ __attribute__((aligned(16))) uint8_t s_rq_s[RQ ? (MX ? 16 : kPairs * 1024) : 16];
    __shared__ __attribute__((aligned(16))) uint16_t s_rq[RQ ? 4 * 64 * kRqPitch : 8];
    __shared__ __attribute__((aligned(16))) uint32_t s_tab[kDialects * 4 * 4 + 4];   // + the all-zero table
    // visits: block | class of A << 10 | class of W << 12, from the highest class sum to the lowest
    __shared__ uint16_t s_vl[kVisitCap];
    __shared__ __attribute__((aligned(4))) uint8_t s_refa[kTileM];
    __shared__ uint8_t s_refw[kTileN];
    __shared__ int s_ctl[8];                 // segment ends (entries), feasibility

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#ifdef DFP4_TIMING_STAMPS   // timing experiments only: 100 MHz timestamps of the kernel's phases, into the workspace
#ifndef DFP4_STAMP_ROW      // which row of tiles (blockIdx.y) writes them
#define DFP4_STAMP_ROW 0
#endif
#define DFP4_STAMP(I)                                                                                   \
    if (tid == 0 && p.ksplit == 1 && p.part && blockIdx.y == (DFP4_STAMP_ROW) && blockIdx.z == 0 && blockIdx.x < 64)   \
        reinterpret_cast<unsigned long long*>(p.part)[blockIdx.x * 8 + (I)] = wall_clock64();
#else
#define DFP4_STAMP(I)
#endif
    DFP4_STAMP(0)
    const int KB = p.KB;
    // Which output tile: the plain order (columns first).  Measured and found no faster: the workgroups of
    // one XCD (each has its own L2) walking the row tiles of a column tile before the next (W then fetched
    // once: 3 % slower), and one row tile of A per XCD (the same).
    const int tx = blockIdx.x, ty = blockIdx.y;
    const int m0 = ty * kTileM, n0 = tx * kTileN;
    const int S = p.ksplit, sidx = (int)(blockIdx.z % (unsigned)S);
    const int64_t bz = blockIdx.z / (unsigned)S;
    const uint8_t* ap = p.a_prep + bz * p.a_prep_stride;
    const uint8_t* wp = p.w_prep + bz * p.w_prep_stride;
    const int tile_id = ty * p.tiles_n + tx;
    // this workgroup's range of blocks
    const int kb_per = (KB + S - 1) / S;
    const int kb_lo = sidx * kb_per, kb_hi = min(KB, kb_lo + kb_per);

    // ---- prologue: tables, references, list of (block, class of A, class of W) visits
    // every global load of the prologue is issued before the first value is used: one memory round trip, not four
    const uint8_t* mask_a = ap + p.off_mask + (int64_t)ty * KB;
    const uint8_t* mask_w = wp + p.off_wmask + (int64_t)tx * KB;
    uint32_t ma[kMaxKB / 64], mw[kMaxKB / 64];
    if (wave == 0) {
#pragma unroll
        for (int j = 0; j < kMaxKB / 64; ++j) {
            const int kb = j * 64 + lane;
            ma[j] = kb < KB ? mask_a[kb] : 0u;
            mw[j] = kb < KB ? mask_w[kb] : 0u;
        }
    }
    static_assert(kDialects * 16 == 256 && kTileM == 512, "one table word and two reference bytes per thread");
    const uint32_t tab_word = (&g_shifted_book.w[0][0][0])[tid];
    const uint8_t refa0 = ap[p.off_refa + m0 + tid], refa1 = ap[p.off_refa + m0 + 256 + tid];   // rows padded to 512
    const uint8_t refw0 = tid < kTileN && n0 + tid < p.N ? wp[p.off_refw + n0 + tid] : (uint8_t)0;
    s_tab[tid] = tab_word;
    if (tid < 4) s_tab[kDialects * 16 + tid] = 0u;
    s_refa[tid] = refa0;
    s_refa[256 + tid] = refa1;
    if (tid < kTileN) s_refw[tid] = refw0;
    if (tid < 8) s_ctl[tid] = 0;
    if (wave == 0) {
        // A block is visited once for every pair (class present among the tile's 512 rows of A, class
        // present among its 128 rows of W); rows of other classes contribute zeros.  Visits are
        // ordered by the class sum, which is the number of 4-bit shifts the accumulators still
        // receive.  The list holds the visits of this workgroup's range of blocks; whether the tile
        // can be taken at all is decided from ALL blocks, so that every workgroup sharing the tile
        // decides the same.
        bool bad = false;
#pragma unroll
        for (int j = 0; j < kMaxKB / 64; ++j) {
            // highest classes present: their sum must not exceed the classes kept
            const int ha = 31 - __builtin_clz(ma[j] | 1u), hw = 31 - __builtin_clz(mw[j] | 1u);
            bad |= ha + hw > kMaxClass;
        }
        int pos = 0, weight = 0;                                      // weight: sum of 16^(class sum) over all of K
        for (int ct = kMaxClass; ct >= 0; --ct) {
            for (int ca = 0; ca <= ct; ++ca) {
                const int cw = ct - ca;
#pragma unroll
                for (int j = 0; j < kMaxKB / 64; ++j) {
                    if (j * 64 >= KB) break;                          // uniform
                    const int kb = j * 64 + lane;
                    const bool f = ((ma[j] >> ca) & 1u) && ((mw[j] >> cw) & 1u);
                    weight += __popcll(__ballot(f)) << (4 * ct);
                    const bool mine = f && kb >= kb_lo && kb < kb_hi;
                    const unsigned long long bal = __ballot(mine);
                    if (mine) s_vl[pos + __popcll(bal & ((1ull << lane) - 1ull))] = (uint16_t)(kb | (ca << 10) | (cw << 12));
                    pos += __popcll(bal);
                }
            }
            if (pos & 1) {                                            // a step takes two visits
                if (lane == 0) s_vl[pos] = (uint16_t)KB;              // padding: the all-zero block of class 0
                pos += 1;
            }
            if (lane == 0) s_ctl[kMaxClass - ct] = pos;               // s_ctl[0..2]: end of class sum 2, 1, 0
        }
        if (lane < kVisitPad) s_vl[pos + lane] = (uint16_t)KB;        // the loop looks five steps ahead
        // exponent offsets beyond the classes kept, or an int32 accumulator that could overflow
        if (__ballot(bad) != 0ull || weight > kIntBound) {
            if (lane == 0) s_ctl[4] = 1;
        }
    }
    __syncthreads();
    DFP4_STAMP(1)
    // segment ends in steps (uniform: they go to the loop in scalar registers)
    const int end2 = __builtin_amdgcn_readfirstlane(s_ctl[0] / 2), end1 = __builtin_amdgcn_readfirstlane(s_ctl[1] / 2),
              total = __builtin_amdgcn_readfirstlane(s_ctl[2] / 2);
    if (s_ctl[4] != 0) {
        // The tile cannot be taken (every workgroup sharing it sees the same): the first of them
        // computes it with one fp32 scale-and-add per block, 128 rows at a time; the others leave.
        if (sidx != 0) return;
        if (tid == 0)
            atomicAdd(reinterpret_cast<uint32_t*>(const_cast<uint8_t*>(ap) + p.off_cnt) + kMaxSplitTiles, 1u);
        if constexpr (RQ) {
            if constexpr (MX) {
                if (tid < 64) s_rq_q[tid] = g_quant_tables.mx[tid];
            } else {
                const uint4* gq = reinterpret_cast<const uint4*>(g_quant_tables.q);
                const uint4* gs = reinterpret_cast<const uint4*>(g_quant_tables.s);
                for (int i = tid; i < 1024; i += 256) reinterpret_cast<uint4*>(s_rq_q)[i] = gq[i];
                for (int i = tid; i < 512; i += 256) reinterpret_cast<uint4*>(s_rq_s)[i] = gs[i];
            }
        }
        uint8_t (&s_exp)[2][256] = *reinterpret_cast<uint8_t (*)[2][256]>(&s_b[0][0]);
        for (int piece = 0; piece < 4; ++piece) {
            const int by = ty * 4 + piece;
            if (by * 128 >= p.M) break;
            __syncthreads();
            block_flush_tile<MX, BF16>(p, bz, by, tx, s_exp);
            if constexpr (RQ) quantize_flushed_piece<MX>(p, bz, by, tx, s_rq_s, s_rq_q);
        }
        return;
    }

    const int h = lane >> 5, r = lane & 31;            // MFMA operand: lanes 32.. hold the pair's second block
    const uint32_t wave_u = (uint32_t)__builtin_amdgcn_readfirstlane(wave);
    const uint32_t lds_tab = (uint32_t)__builtin_amdgcn_readfirstlane(
        (int)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)&s_tab[0]);
    const uint32_t lds_vl = (uint32_t)__builtin_amdgcn_readfirstlane(
        (int)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)&s_vl[0]);
    const uint32_t lds_b = (uint32_t)__builtin_amdgcn_readfirstlane(
        (int)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)&s_b[0][0]);
    const uint32_t grp_stride = (uint32_t)(KB + 1) * 1024u;
    const uint32_t cls_stride = (uint32_t)p.tiles_m * kGroups * grp_stride;
    const uint32_t tile_off = (uint32_t)ty * kGroups * grp_stride;
#ifdef DFP4_TIMING_SAME_A   // timing experiments only: every wave reads the fragments of wave 0 (wrong results)
    const uint8_t* a8w = ap + p.off_a8;
#else
    const uint8_t* a8w = ap + p.off_a8 + (uint64_t)wave_u * 4u * grp_stride;   // uniform per wave
#endif
    const uint8_t* wcodes = wp + p.off_wcodes;                                // uniform; [group][block][row]
    const uint8_t* wmeta = wp + p.off_wmeta;                                  // uniform; [class][group][block][row]
    const int ncol = n0 + wave * 32 + r;                // this lane's W row (rows beyond N exist: all-zero tables)
    // this lane's row of W: slot (row % 32) of block 0 of its 32-row group; a block further is 32 slots further
    const uint32_t w_slot = (uint32_t)(ncol >> 5) * (uint32_t)KB * 32u + (uint32_t)(ncol & 31);
    const uint32_t w_row_codes = w_slot * 16u, w_row_meta = w_slot * 4u;

    // W operands of the first two steps (the loop expands those of step s + 2 during step s)
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const uint32_t entry = s_vl[2 * s + h];
        const uint32_t kb = min(entry & 1023u, (uint32_t)KB - 1u);
        const uint4 c = *reinterpret_cast<const uint4*>(wcodes + w_row_codes + kb * 512u);
        const uint32_t meta = *reinterpret_cast<const uint32_t*>(wmeta + ((entry >> 12) & 3u) * p.wmeta_cls_stride +
                                                                 w_row_meta + kb * 128u);
        const uint4 tab = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint8_t*>(s_tab) + meta);
        *reinterpret_cast<v4i*>(&s_b[s][(wave * 2 + 0) * 1024 + lane * 16]) = unpack16(c.x, c.y, tab);
        *reinterpret_cast<v4i*>(&s_b[s][(wave * 2 + 1) * 1024 + lane * 16]) = unpack16(c.z, c.w, tab);
    }
    __syncthreads();
    DFP4_STAMP(2)

    // ---- main loop (gemm_step_asm.inc): accumulators in a[0:255]
    {
        const uint64_t a8u = reinterpret_cast<uint64_t>(a8w), wcu = reinterpret_cast<uint64_t>(wcodes),
                       wmu = reinterpret_cast<uint64_t>(wmeta);
        const uint32_t a_lane = (uint32_t)r * 16u, l16 = (uint32_t)lane * 16u, h2 = (uint32_t)h * 2u;
        const uint32_t sign_sel = 0x090b080au, kbm = (uint32_t)KB - 1u;
        asm volatile(DFP4_MAINLOOP_ASM
                     :
                     : [a8lo] "s"((uint32_t)a8u), [a8hi] "s"((uint32_t)(a8u >> 32)), [gstr] "s"(grp_stride),
                       [wclo] "s"((uint32_t)wcu), [wchi] "s"((uint32_t)(wcu >> 32)),
                       [wmlo] "s"((uint32_t)wmu), [wmhi] "s"((uint32_t)(wmu >> 32)),
                       [cstr] "s"(cls_stride), [toff] "s"(tile_off), [kbm] "s"(kbm), [tabb] "s"(lds_tab),
                       [vlb] "s"(lds_vl), [bb] "s"(lds_b), [sel] "s"(sign_sel),
                       [e2] "s"((uint32_t)end2), [e1] "s"((uint32_t)end1), [e0] "s"((uint32_t)total),
                       [wcs] "s"(p.wmeta_cls_stride),
                       [wv] "s"(wave_u), [alane] "v"(a_lane), [l16] "v"(l16), [wrc] "v"(w_row_codes),
                       [wrm] "v"(w_row_meta), [h2] "v"(h2)
                     : DFP4_LOOP_VGPR_CLOBBERS, DFP4_ACC_CLOBBERS, DFP4_LOOP_SGPR_CLOBBERS, "scc", "memory");
    }

    DFP4_STAMP(3)
    // ---- epilogue (nothing to store or publish for a wave whose 128 rows lie beyond M)
    if constexpr (RQ) {
        if constexpr (MX) {
            if (tid < 64) s_rq_q[tid] = g_quant_tables.mx[tid];
        } else {
            const uint4* gq = reinterpret_cast<const uint4*>(g_quant_tables.q);
            const uint4* gs = reinterpret_cast<const uint4*>(g_quant_tables.s);
            for (int i = tid; i < 1024; i += 256) reinterpret_cast<uint4*>(s_rq_q)[i] = gq[i];
            for (int i = tid; i < 512; i += 256) reinterpret_cast<uint4*>(s_rq_s)[i] = gs[i];
        }
        __syncthreads();
    }
    const bool active = m0 + (int)wave_u * 128 < p.M;      // wave-uniform
#define DFP4_READ_ACC(G, V)                                                                         \
    asm volatile(DFP4_ACC_READ_ASM_##G                                                              \
                 : "=v"(V[0]), "=v"(V[1]), "=v"(V[2]), "=v"(V[3]), "=v"(V[4]), "=v"(V[5]),          \
                   "=v"(V[6]), "=v"(V[7]), "=v"(V[8]), "=v"(V[9]), "=v"(V[10]), "=v"(V[11]),        \
                   "=v"(V[12]), "=v"(V[13]), "=v"(V[14]), "=v"(V[15]))
#define DFP4_FOR_TILES(F)                                                                           \
    F(0) F(1) F(2) F(3) F(4) F(5) F(6) F(7) F(8) F(9) F(10) F(11) F(12) F(13) F(14) F(15)
    // partial tiles of the workgroups that share this output tile: [range][(16 tile + x) * 256 + thread]
    const int* part = S > 1 ? p.part + bz * p.part_stride + (int64_t)tile_id * S * (kTileM * kTileN) : nullptr;
    if (S > 1) {
        // K is shared with other workgroups.  Every one publishes its exact int32 sums and then
        // counts itself in; the one that arrives last adds the others' sums to its own (the total
        // is exact and does not depend on the order) and goes on to the conversion and the stores.
        // The sums travel as device-scope relaxed atomic stores and loads (they pass the per-XCD
        // L2 instead of being written back and invalidated wholesale by a fence); "all my stores
        // have completed" is the wait on the memory counter before the barrier.
        if (active) {
            int* mine = const_cast<int*>(part) + (int64_t)sidx * (kTileM * kTileN);
#define DFP4_PUBLISH(G)                                                                             \
            {                                                                                       \
                int v[16];                                                                          \
                DFP4_READ_ACC(G, v);                                                                \
                _Pragma("unroll") for (int x = 0; x < 16; ++x)                                      \
                    __hip_atomic_store(&mine[(G * 16 + x) * 256 + tid], v[x], __ATOMIC_RELAXED,     \
                                       __HIP_MEMORY_SCOPE_AGENT);                                   \
            }
            DFP4_FOR_TILES(DFP4_PUBLISH)
#undef DFP4_PUBLISH
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) {
            uint32_t* cnt = reinterpret_cast<uint32_t*>(const_cast<uint8_t*>(ap) + p.off_cnt) + tile_id;
            const uint32_t arrived = atomicAdd(cnt, 1u);
            if (arrived == (uint32_t)S - 1u) atomicExch(cnt, 0u);       // ready for the next product
            s_ctl[5] = (int)arrived;
        }
        __syncthreads();
        if (s_ctl[5] != S - 1) return;
    }
    if (!active) return;                                   // nothing to store for rows beyond M
#define DFP4_READ_TILE(G, V)                                                                        \
    DFP4_READ_ACC(G, V);                                                                            \
    if (S > 1) {                                                                                    \
        for (int s_ = 0; s_ < S; ++s_) {                                                            \
            if (s_ == sidx) continue;                                                               \
            const int* other_ = part + (int64_t)s_ * (kTileM * kTileN);                             \
            _Pragma("unroll") for (int x = 0; x < 16; ++x)                                          \
                V[x] += __hip_atomic_load(&other_[(G * 16 + x) * 256 + tid], __ATOMIC_RELAXED,      \
                                          __HIP_MEMORY_SCOPE_AGENT);                                \
        }                                                                                           \
    }
    if constexpr (RQ) {
        // Requantizing epilogue (Section 3.3: results are quantized again for the next
        // multiplication).  Each value is converted and rounded to bf16 exactly as the bf16
        // output would be; the wave stages 64 rows x 128 columns in LDS and re-reads them in
        // the quantizer's layout (4 lanes per block of 32 consecutive columns), then stores
        // codes, dialect ids and exponent bytes of the [M, N] result blocked along N.
        const int row0 = m0 + (int)wave_u * 128;
        uint16_t* st = &s_rq[wave * 64 * kRqPitch];
        const int nb_row = p.N / kBlock;
        int ew[4];
#pragma unroll
        for (int n = 0; n < 4; ++n) ew[n] = (int)s_refw[n * 32 + r] - 256;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
#define DFP4_STAGE(G)                                                                               \
            if ((G >> 3) == half) {                                                                 \
                int v[16];                                                                          \
                DFP4_READ_TILE(G, v);                                                               \
                const int gi = G >> 2, n = G & 3;                                                   \
                _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                     \
                    const uint32_t e4 = *reinterpret_cast<const uint32_t*>(                         \
                        &s_refa[wave * 128 + gi * 32 + 8 * q + 4 * h]);                             \
                    _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                 \
                        const float f = ldexpf((float)v[4 * q + j], (int)((e4 >> (8 * j)) & 0xffu) + ew[n]); \
                        st[((gi & 1) * 32 + 8 * q + 4 * h + j) * kRqPitch + n * 32 + r] = f32_to_bf16_rne(f); \
                    }                                                                               \
                }                                                                                   \
            }
            DFP4_FOR_TILES(DFP4_STAGE)
#undef DFP4_STAGE
            for (int pass = 0; pass < 16; ++pass) {
                const int b = pass * 16 + (lane >> 2), row = b >> 2, cb = b & 3, sub = lane & 3;
                const uint4 wv = *reinterpret_cast<const uint4*>(&st[row * kRqPitch + cb * 32 + sub * 8]);
                uint32_t code, eb, dl = 0;
                if constexpr (MX) mxfp4_pass(wv, s_rq_q, code, eb);
                else dfp4_pass(wv, s_rq_s, s_rq_q, code, eb, dl);
                const int m = row0 + half * 64 + row, nb = (n0 >> 5) + cb;
                if (m < p.M && nb < nb_row) {
                    const size_t blk = (size_t)(bz * p.M + m) * nb_row + nb;
                    p.q_codes[blk * 4 + sub] = code;
                    if (sub == 0) {
                        p.q_exp[blk] = (uint8_t)eb;
                        if constexpr (!MX) p.q_dial[blk] = (uint8_t)dl;
                    }
                }
            }
        }
        return;
    }
    {
        // The one rounding of the whole product: int32 -> fp32, scaled by 2^(refA + refW - 2).
        // Accumulator x of lane (h, r) of tile (gi, n) is output row 128*wave + 32*gi +
        // 8*(x>>2) + 4*h + (x&3), column 32*n + r.  Row addresses are wave-uniform (scalar
        // registers); the lane adds a constant byte offset, so a store costs a handful of
        // instructions.
        constexpr int kEsz = BF16 ? 2 : 4;
        const int row0 = m0 + (int)wave_u * 128;
        uint8_t* wave_out = static_cast<uint8_t*>(p.out) +
                            (bz * p.strideC + (int64_t)row0 * p.ldc + n0) * kEsz;            // uniform
        const int64_t row_bytes = p.ldc * kEsz;                                              // uniform
        const bool full = row0 + 128 <= p.M && n0 + kTileN <= p.N;                           // uniform
        // bf16: lanes exchange values in pairs so that every lane stores two adjacent columns of
        // one row (even lanes the even row of a row pair, odd lanes the odd row)
        const bool pairs = BF16 && full && (p.ldc & 1) == 0 && ((p.strideC * kEsz) & 3) == 0 &&
                           (reinterpret_cast<uintptr_t>(p.out) & 3) == 0;                    // uniform
        const uint32_t lane_off = pairs ? (uint32_t)((4 * h + (r & 1)) * row_bytes + (r & ~1) * kEsz)
                                        : (uint32_t)(4 * h * row_bytes + r * kEsz);
        int ew[4];
#pragma unroll
        for (int n = 0; n < 4; ++n) ew[n] = (int)s_refw[n * 32 + r] - 256;
        auto store_tile = [&](auto full_c, auto pairs_c, int i, int (&v)[16]) {
            constexpr bool kFull = decltype(full_c)::value, kPairs = decltype(pairs_c)::value;
            const int gi = i >> 2, n = i & 3;
            uint8_t* tile_out = wave_out + (int64_t)gi * 32 * row_bytes + n * 32 * kEsz;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t e4 = *reinterpret_cast<const uint32_t*>(&s_refa[wave * 128 + gi * 32 + 8 * q + 4 * h]);
                float f[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    f[j] = ldexpf((float)v[4 * q + j], (int)((e4 >> (8 * j)) & 0xffu) + ew[n]);
                uint8_t* rowp = tile_out + (int64_t)(8 * q) * row_bytes;                    // uniform
                if constexpr (BF16 && kPairs) {
#pragma unroll
                    for (int j = 0; j < 4; j += 2) {
                        const uint32_t b0 = f32_to_bf16_rne(f[j]), b1 = f32_to_bf16_rne(f[j + 1]);
                        const uint32_t send = (r & 1) ? b0 : b1;
                        const uint32_t recv = (uint32_t)__builtin_amdgcn_mov_dpp((int)send, 0xB1, 0xf, 0xf, true);
                        const uint32_t word = (r & 1) ? (recv | (b1 << 16)) : (b0 | (recv << 16));
                        DFP4_OUT_STORE(reinterpret_cast<uint32_t*>(rowp + (int64_t)j * row_bytes + lane_off), word);
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        if (kFull || (row0 + gi * 32 + 8 * q + 4 * h + j < p.M && n0 + n * 32 + r < p.N)) {
                            uint8_t* dst = rowp + (int64_t)j * row_bytes + lane_off;
                            if constexpr (BF16)
                                DFP4_OUT_STORE(reinterpret_cast<uint16_t*>(dst), f32_to_bf16_rne(f[j]));
                            else
                                DFP4_OUT_STORE(reinterpret_cast<float*>(dst), f[j]);
                        }
                    }
                }
            }
        };
#define DFP4_FINISH(G)                                                                              \
        {                                                                                           \
            int v[16];                                                                              \
            DFP4_READ_TILE(G, v);                                                                   \
            store_tile(kFullC, kPairsC, G, v);                                                      \
        }
        if (pairs) {
            constexpr std::true_type kFullC{}, kPairsC{};
            DFP4_FOR_TILES(DFP4_FINISH)
        } else if (full) {
            constexpr std::true_type kFullC{};
            constexpr std::false_type kPairsC{};
            DFP4_FOR_TILES(DFP4_FINISH)
        } else {
            constexpr std::false_type kFullC{}, kPairsC{};
            DFP4_FOR_TILES(DFP4_FINISH)
        }
#undef DFP4_FINISH
    }
    DFP4_STAMP(4)
#undef DFP4_STAMP
#undef DFP4_FOR_TILES
#undef DFP4_READ_TILE
#undef DFP4_READ_ACC
}

// ---------------------------------------------------------------------------
// Few rows of A (decode shapes, M <= 64): W is streamed once per 32 rows of A and
// the time goes into expanding W, so the tile is 32 (A rows) x 32 (W rows) per
// workgroup and the workgroup's 16 (or 8) waves share K: wave w takes a contiguous
// range of blocks and multiplies block by block (one MFMA each); the partial tiles
// are added in a fixed order through LDS.  No prepass and no workspace.
// small_tile() applies the exponent pair per block in fp32 as the paper does;
// small_exact_tile() (tried first) folds the exponents into the operands instead.
// ---------------------------------------------------------------------------
constexpr int kSmallWaves = 16;     // waves of a workgroup, at most (LDS is laid out for this many)
constexpr int kSmallMaxKB = 512;      // LDS holds the 32 rows' exponent bytes of all blocks
constexpr int kSmallMaxM = 64;
static_assert(kSmallMaxM == 64 && kSmallMaxKB == 512, "takes_small_kernel() states these limits");

struct SmallTileLds {
    __attribute__((aligned(16))) uint32_t tab[kDialects * 4];   // shift-0 tables
    __attribute__((aligned(4))) uint8_t ea[kSmallMaxKB * 32];   // [block][row] exponent bytes of A
    float red[kSmallWaves / 2][16][64];
};

// One 32 x 32 output tile by a workgroup of 16 waves, one fp32 scale-and-add per block.
template <bool MX, bool BF16, int NW>
__device__ __forceinline__ void small_tile(const GemmParams& p, int64_t bz, int m0, int n0, SmallTileLds& lds) {
    uint32_t (&s_tab)[kDialects * 4] = lds.tab;
    uint8_t (&s_ea)[kSmallMaxKB * 32] = lds.ea;
    float (&s_red)[kSmallWaves / 2][16][64] = lds.red;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, r = lane & 31;
    const int KB = p.KB;
    const int64_t a_row0 = bz * p.strideA_rows, w_row0 = bz * p.strideW_rows;

    const int64_t arow = a_row0 + min(m0 + r, p.M - 1), wrow = w_row0 + min(n0 + r, p.N - 1);
    const uint8_t* ac = p.a_codes + arow * KB * 16 + h * 8;
    const uint8_t* wc = p.w_codes + wrow * KB * 16 + h * 8;
    const uint8_t* ad = MX ? nullptr : p.a_dial + arow * KB;
    const uint8_t* wd = MX ? nullptr : p.w_dial + wrow * KB;
    const uint8_t* we = p.w_exp + wrow * KB;
    const int per = (KB + NW - 1) / NW;
    const int kb_lo = wave * per, kb_hi = min(KB, kb_lo + per);

    for (int i = tid; i < kDialects * 4; i += NW * 64) s_tab[i] = g_shifted_book.w[i >> 2][0][i & 3];
    for (int i = tid; i < 32 * KB; i += NW * 64) {
        const int row = i / KB, kb = i - row * KB;
        s_ea[kb * 32 + row] = p.a_exp[(a_row0 + min(m0 + row, p.M - 1)) * KB + kb];
    }
    __syncthreads();

    float acc[16];
#pragma unroll
    for (int x = 0; x < 16; ++x) acc[x] = 0.0f;
    constexpr int kU = 4;              // blocks whose loads are issued together
    for (int kb0 = kb_lo; kb0 < kb_hi; kb0 += kU) {
        uint2 ca[kU], cw[kU];
        uint32_t da[kU], dw[kU], ew[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int kb = min(kb0 + u, kb_hi - 1);            // the tail repeats the last block (not used)
            ca[u] = *reinterpret_cast<const uint2*>(ac + (int64_t)kb * 16);
            cw[u] = *reinterpret_cast<const uint2*>(wc + (int64_t)kb * 16);
            da[u] = MX ? 7u : ((uint32_t)ad[kb] & 15u);
            dw[u] = MX ? 7u : ((uint32_t)wd[kb] & 15u);
            ew[u] = we[kb];
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int kb = kb0 + u;
            if (kb >= kb_hi) break;                            // wave-uniform
            const v4i a = unpack16(ca[u].x, ca[u].y, *reinterpret_cast<const uint4*>(&s_tab[da[u] * 4]));
            const v4i b = unpack16(cw[u].x, cw[u].y, *reinterpret_cast<const uint4*>(&s_tab[dw[u] * 4]));
            v16i pr = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
            pr = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, pr, 0, 0, 0);
            const int ewc = (int)ew[u] - 256;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t e4 = *reinterpret_cast<const uint32_t*>(&s_ea[kb * 32 + 8 * q + 4 * h]);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[4 * q + j] += ldexpf((float)pr[4 * q + j], (int)((e4 >> (8 * j)) & 0xffu) + ewc);
            }
        }
    }
    // the NW partial tiles, added in a fixed order: the upper half of the waves hands theirs to the lower
    if (wave >= NW / 2) {
#pragma unroll
        for (int x = 0; x < 16; ++x) s_red[wave - NW / 2][x][lane] = acc[x];
    }
    __syncthreads();
    if (wave < NW / 2) {
#pragma unroll
        for (int x = 0; x < 16; ++x) s_red[wave][x][lane] += acc[x];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16 / NW; ++i) {
        const int x = wave + i * NW;                           // thread (x, lane) finishes one output
        float sum = 0.0f;
#pragma unroll
        for (int w = 0; w < NW / 2; ++w) sum += s_red[w][x][lane];
        const int m = m0 + 8 * (x >> 2) + 4 * h + (x & 3), n = n0 + r;
        if (m < p.M && n < p.N) {
            const int64_t o = bz * p.strideC + (int64_t)m * p.ldc + n;
            if constexpr (BF16)
                static_cast<uint16_t*>(p.out)[o] = f32_to_bf16_rne(sum);
            else
                static_cast<float*>(p.out)[o] = sum;
        }
    }
}

// The same tile with the exact scheme of the large kernel, nothing prepared: the workgroup finds the
// reference exponents of its 32 rows of A and 32 rows of W itself (both tiles' exponent bytes go to
// LDS), folds each block's offset into the int8 operands (shift) and a class (weight 16^class sum),
// and sums all of K in int32 -- no floating-point work per block, which is what bounds small_tile().
// Blocks whose rows are all of class 0 on both sides (the common case) take one MFMA; others take one
// per pair of classes present, rows of other classes zeroed, added with the pair's weight.  Returns
// false, having stored nothing, when the exponents spread beyond what an int32 sum can hold (decided
// from the largest offsets of the two tiles, the same for every thread): small_tile() computes the tile.
struct SmallExactLds {
    __attribute__((aligned(16))) uint32_t tab[kDialects * 16 + 4];     // [dialect][shift] tables
    __attribute__((aligned(16))) uint8_t ea[kSmallMaxKB * 32];         // [block][row] exponent bytes of A
    __attribute__((aligned(16))) uint8_t ew[kSmallMaxKB * 32];         // and of W; later the partial tiles
    int mn[64], mx[64];                                                // per row of A (0..31) and of W (32..63)
};
static_assert(sizeof(int) * (kSmallWaves / 2) * 16 * 64 <= 2 * kSmallMaxKB * 32, "partial tiles reuse ea and ew");

template <bool MX, bool BF16, int NW>
__device__ __forceinline__ bool small_exact_tile(const GemmParams& p, int64_t bz, int m0, int n0, SmallExactLds& lds) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, r = lane & 31;
    const int KB = p.KB;
    const int64_t a_row0 = bz * p.strideA_rows, w_row0 = bz * p.strideW_rows;
    const int64_t arow = a_row0 + min(m0 + r, p.M - 1), wrow = w_row0 + min(n0 + r, p.N - 1);
    const uint8_t* ac = p.a_codes + arow * KB * 16 + h * 8;
    const uint8_t* wc = p.w_codes + wrow * KB * 16 + h * 8;
    const uint8_t* ad = MX ? nullptr : p.a_dial + arow * KB;
    const uint8_t* wd = MX ? nullptr : p.w_dial + wrow * KB;
    const int per = (KB + NW - 1) / NW;
    const int kb_lo = wave * per, kb_hi = min(KB, kb_lo + per);

    for (int i = tid; i < kDialects * 16 + 4; i += NW * 64) lds.tab[i] = i < kDialects * 16 ? (&g_shifted_book.w[0][0][0])[i] : 0u;
    for (int i = tid; i < 32 * KB; i += NW * 64) {
        const int row = i / KB, kb = i - row * KB;
        lds.ea[kb * 32 + row] = p.a_exp[(a_row0 + min(m0 + row, p.M - 1)) * KB + kb];
        lds.ew[kb * 32 + row] = p.w_exp[(w_row0 + min(n0 + row, p.N - 1)) * KB + kb];
    }
    if (tid < 64) {
        lds.mn[tid] = 255;
        lds.mx[tid] = 0;
    }
    __syncthreads();
    {
        // smallest and largest exponent byte of every row: thread (row, part) scans every (2 NW)-th block
        const int row = tid & 31, part = tid >> 5;
        int amn = 255, amx = 0, wmn = 255, wmx = 0;
        for (int kb = part; kb < KB; kb += 2 * NW) {
            const int a = lds.ea[kb * 32 + row], w = lds.ew[kb * 32 + row];
            amn = min(amn, a); amx = max(amx, a);
            wmn = min(wmn, w); wmx = max(wmx, w);
        }
        if (part < KB) {
            atomicMin(&lds.mn[row], amn); atomicMax(&lds.mx[row], amx);
            atomicMin(&lds.mn[32 + row], wmn); atomicMax(&lds.mx[32 + row], wmx);
        }
    }
    __syncthreads();
    {
        // Can every class pair that may occur be taken, and the worst-case sum be held?  From the largest
        // offsets only: classes up to ca_max and cw_max may meet in any block.
        int da = 0, dw = 0;
        for (int i = 0; i < 32; ++i) {
            da = max(da, lds.mx[i] - lds.mn[i]);
            dw = max(dw, lds.mx[32 + i] - lds.mn[32 + i]);
        }
        const int ca_max = da >> 2, cw_max = dw >> 2;
        if (ca_max + cw_max > kMaxClass) return false;
        int per_block = 0;
        for (int ca = 0; ca <= ca_max; ++ca)
            for (int cw = 0; cw <= cw_max; ++cw) per_block += 1 << (4 * (ca + cw));
        if (per_block * KB > kIntBound) return false;
    }
    const int refa = lds.mn[r], refw = lds.mn[32 + r];

    v16i acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    const v4i zero4 = {0, 0, 0, 0};
    constexpr int kU = 4;              // blocks whose loads are issued together
    for (int kb0 = kb_lo; kb0 < kb_hi; kb0 += kU) {
        uint2 ca[kU], cw[kU];
        uint32_t da[kU], dw[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int kb = min(kb0 + u, kb_hi - 1);            // the tail repeats the last block (not used)
            ca[u] = *reinterpret_cast<const uint2*>(ac + (int64_t)kb * 16);
            cw[u] = *reinterpret_cast<const uint2*>(wc + (int64_t)kb * 16);
            da[u] = MX ? 7u : ((uint32_t)ad[kb] & 15u);
            dw[u] = MX ? 7u : ((uint32_t)wd[kb] & 15u);
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int kb = kb0 + u;
            if (kb >= kb_hi) break;                            // wave-uniform
            const int oa = (int)lds.ea[kb * 32 + r] - refa, ow = (int)lds.ew[kb * 32 + r] - refw;   // offsets >= 0
            const int cla = oa >> 2, clw = ow >> 2;
            const uint4 ta = *reinterpret_cast<const uint4*>(&lds.tab[(da[u] * 4 + (oa & 3)) * 4]);
            const uint4 tw = *reinterpret_cast<const uint4*>(&lds.tab[(dw[u] * 4 + (ow & 3)) * 4]);
            const v4i a = unpack16(ca[u].x, ca[u].y, ta), b = unpack16(cw[u].x, cw[u].y, tw);
            if (__ballot((cla | clw) != 0) == 0ull) {
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc, 0, 0, 0);
            } else {
                for (int ct = 0; ct <= kMaxClass; ++ct) {
                    for (int c1 = 0; c1 <= ct; ++c1) {
                        const int c2 = ct - c1;
                        if (__ballot(cla == c1) == 0ull || __ballot(clw == c2) == 0ull) continue;
                        const v4i pa = cla == c1 ? a : zero4, pb = clw == c2 ? b : zero4;
                        v16i t16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                        t16 = __builtin_amdgcn_mfma_i32_32x32x32_i8(pa, pb, t16, 0, 0, 0);
#pragma unroll
                        for (int x = 0; x < 16; ++x) acc[x] += t16[x] << (4 * ct);
                    }
                }
            }
        }
    }
    // the NW exact partial tiles, added through LDS (over the exponent bytes, which are no longer needed)
    __syncthreads();
    int (*red)[16][64] = reinterpret_cast<int (*)[16][64]>(lds.ea);
    if (wave >= NW / 2) {
#pragma unroll
        for (int x = 0; x < 16; ++x) red[wave - NW / 2][x][lane] = acc[x];
    }
    __syncthreads();
    if (wave < NW / 2) {
#pragma unroll
        for (int x = 0; x < 16; ++x) red[wave][x][lane] += acc[x];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16 / NW; ++i) {
        const int x = wave + i * NW;                           // thread (x, lane) finishes one output
        int sum = 0;
#pragma unroll
        for (int w = 0; w < NW / 2; ++w) sum += red[w][x][lane];
        const int lr = 8 * (x >> 2) + 4 * h + (x & 3), m = m0 + lr, n = n0 + r;
        if (m < p.M && n < p.N) {
            const float f = ldexpf((float)sum, lds.mn[lr] + lds.mn[32 + r] - 256);
            const int64_t o = bz * p.strideC + (int64_t)m * p.ldc + n;
            if constexpr (BF16)
                static_cast<uint16_t*>(p.out)[o] = f32_to_bf16_rne(f);
            else
                static_cast<float*>(p.out)[o] = f;
        }
    }
    return true;
}

template <bool MX, bool BF16, int NW>
__global__ __launch_bounds__(NW * 64) void gemm_small_kernel(GemmParams p) {
    __shared__ union {
        SmallExactLds exact;
        SmallTileLds flush;
    } lds;
    const int m0 = (int)blockIdx.y * 32, n0 = (int)blockIdx.x * 32;
    if (small_exact_tile<MX, BF16, NW>(p, blockIdx.z, m0, n0, lds.exact)) return;
    __syncthreads();
    small_tile<MX, BF16, NW>(p, blockIdx.z, m0, n0, lds.flush);
}

// ---------------------------------------------------------------------------
// Few rows of A on PREPARED operands (decode shapes with weights prepared offline): the exact
// scheme of the large kernel -- exponent offsets folded into the int8 operands, classes weighted
// by 16^(class of A + class of W), one conversion at the end -- in the shape of the few-rows
// kernel: a workgroup of NW waves owns 32 rows of A x 32 rows of W and the waves share K in
// contiguous ranges of block pairs.  The kernel is bound by latency, so it keeps the chain of
// dependent memory accesses short: there is no list of visits.  A wave issues, before anything
// else, the loads of its first pairs for the common case (class 0 of both operands): class masks,
// codes and table offsets of W, expanded fragments of A.  The masks come back first; a block that
// has other classes as well (rare: outlier channels) gets extra products, each computed into a
// temporary tile and added with its weight 16^(class sum), which is exact in int32 under the same
// bound the large kernel checks.  Whether the tile can be taken at all is decided by every wave
// from the masks of all of K (same data, same decision).  The NW exact partial tiles are added
// through LDS.  A tile the scheme cannot take is computed by small_tile().
// ---------------------------------------------------------------------------
template <bool MX, bool BF16, int NW>
__global__ __launch_bounds__(NW * 64) void gemm_rows_kernel(GemmParams p) {
    __shared__ __attribute__((aligned(16))) uint32_t s_tab[kDialects * 16 + 4];
    __shared__ union {
        int red[kSmallWaves / 2][16][64];
        SmallTileLds small;
    } u;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, r = lane & 31;
    const int KB = p.KB;
    const int m0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
    const uint8_t* ap = p.a_prep;
    const uint8_t* wp = p.w_prep;
    const uint8_t* mask_a = ap + p.off_mask + (int64_t)(m0 / kTileM) * KB;      // classes of the 512-row tile of A
    const uint8_t* mask_w = wp + p.off_wmask + (int64_t)(n0 / kTileN) * KB;     // and of the 128-row tile of W

    const uint32_t grp_stride = (uint32_t)(KB + 1) * 1024u;
    const uint64_t cls_stride = (uint64_t)p.tiles_m * kGroups * grp_stride;
    const uint8_t* a8 = ap + p.off_a8 + (uint64_t)(m0 / 32) * grp_stride + (uint32_t)r * 16u;
    const int ncol = n0 + r;                            // rows beyond N exist in the prepared W: all-zero tables
    const uint64_t w_slot = (uint64_t)(ncol >> 5) * KB * 32u + (uint32_t)(ncol & 31);      // [group][block][row]
    const uint8_t* wcodes = wp + p.off_wcodes + w_slot * 16u;
    const uint8_t* wmeta = wp + p.off_wmeta + w_slot * 4u;

    // this wave's range of block pairs (lane half h takes block 2 * pair + h)
    const int P = (KB + 1) / 2, per = (P + NW - 1) / NW;
    const int p_lo = min(P, wave * per), p_hi = min(P, p_lo + per);
    constexpr int kU = 4;                              // pairs whose loads are issued together
    uint32_t mA[kU], mW[kU], meta[kU];
    uint4 wc[kU];
    v4i af[kU][2];
    auto issue = [&](int g0) {
#pragma unroll
        for (int q = 0; q < kU; ++q) {                 // the masks first: they are needed first
            const int kb = 2 * min(g0 + q, p_hi - 1) + h;
            mA[q] = kb < KB ? mask_a[kb] : 0u;
            mW[q] = kb < KB ? mask_w[kb] : 0u;
        }
#pragma unroll
        for (int q = 0; q < kU; ++q) {
            const int kb = 2 * min(g0 + q, p_hi - 1) + h, kbw = min(kb, KB - 1);
            wc[q] = *reinterpret_cast<const uint4*>(wcodes + (uint32_t)kbw * 512u);
            meta[q] = *reinterpret_cast<const uint32_t*>(wmeta + (uint32_t)kbw * 128u);        // class 0 of W
            const uint8_t* src = a8 + (uint32_t)min(kb, KB) * 1024u;                          // class 0 of A; KB = zeros
            af[q][0] = *reinterpret_cast<const v4i*>(src);
            af[q][1] = *reinterpret_cast<const v4i*>(src + 512);
        }
    };
    // loads in the order their values are needed: the masks of all of K (the decision below), the
    // table, then the first pairs' operands
    uint32_t da[kMaxKB / 64], dw[kMaxKB / 64];
#pragma unroll
    for (int j = 0; j < kMaxKB / 64; ++j) {
        const int kb = j * 64 + lane;
        da[j] = kb < KB ? mask_a[kb] : 0u;
        dw[j] = kb < KB ? mask_w[kb] : 0u;
    }
    const uint32_t tab_word = tid < kDialects * 16 ? (&g_shifted_book.w[0][0][0])[tid] : 0u;
    if (p_lo < p_hi) issue(p_lo);

    // reference exponents of the outputs this thread finishes (x = wave, wave + NW, ..): loaded now, used last
    int ref_sum[16 / NW];
#pragma unroll
    for (int i = 0; i < 16 / NW; ++i) {
        const int x = wave + i * NW;
        const int m = min(m0 + 8 * (x >> 2) + 4 * h + (x & 3), p.M - 1);
        ref_sum[i] = (int)ap[p.off_refa + m] + (int)wp[p.off_refw + ncol] - 256;
    }
    // Can the tile be taken?  Classes beyond those kept, or a sum of weights an int32 accumulator
    // could not hold.  Every wave decides from the masks of all of K.
    bool declined;
    {
        bool bad = false;
        int weight = 0;
#pragma unroll
        for (int j = 0; j < kMaxKB / 64; ++j) {
            if (j * 64 >= KB) break;                   // uniform
            const uint32_t a = da[j], w = dw[j];
            const int ha = 31 - __builtin_clz(a | 1u), hw = 31 - __builtin_clz(w | 1u);
            bad |= ha + hw > kMaxClass;
#pragma unroll
            for (int ct = 0; ct <= kMaxClass; ++ct)
#pragma unroll
                for (int ca = 0; ca <= ct; ++ca)
                    weight += __popcll(__ballot(((a >> ca) & 1u) && ((w >> (ct - ca)) & 1u))) << (4 * ct);
        }
        declined = __ballot(bad) != 0ull || weight > kIntBound;
    }
    if (tid < kDialects * 16 + 4) s_tab[tid] = tab_word;        // NW * 64 >= 512 > 260 entries
    __syncthreads();
    if (declined) {
        if (tid == 0 && blockIdx.x % (kTileN / 32) == 0)   // counted once per 512 x 128 tile, like the large kernel
            atomicAdd(reinterpret_cast<uint32_t*>(const_cast<uint8_t*>(ap) + p.off_cnt) + kMaxSplitTiles, 1u);
        small_tile<MX, BF16, NW>(p, 0, m0, n0, u.small);
        return;
    }

    v16i acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    const v4i zero4 = {0, 0, 0, 0};
    bool any_odd = false;                              // some block of this wave's range has other classes too
    for (int g0 = p_lo; g0 < p_hi; g0 += kU) {
        if (g0 != p_lo) issue(g0);
        bool odd = false;
#pragma unroll
        for (int q = 0; q < kU; ++q) odd |= g0 + q < p_hi && 2 * (g0 + q) + h < KB && (mA[q] != 1u || mW[q] != 1u);
        const bool mixed = __ballot(odd) != 0ull;      // uniform
        any_odd |= mixed;
#pragma unroll
        for (int q = 0; q < kU; ++q) {
            if (g0 + q >= p_hi) break;                 // wave-uniform
            const uint4 tab = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint8_t*>(s_tab) + meta[q]);
            const v4i b0 = unpack16(wc[q].x, wc[q].y, tab), b1 = unpack16(wc[q].z, wc[q].w, tab);
            v4i a0 = af[q][0], a1 = af[q][1];
            if (mixed) {                               // a class-0 fragment exists only where the tile has class 0
                const bool have = (mA[q] & 1u) != 0u && 2 * (g0 + q) + h < KB;
                a0 = have ? a0 : zero4;
                a1 = have ? a1 : zero4;
            }
            acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b0, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b1, acc, 0, 0, 0);
        }
    }
    // The other class pairs (rare: blocks with outliers), pair by pair: lanes whose block has the
    // class pair bring its operands, the others zeros; the product goes to a temporary tile and is
    // added with its weight.
    if (any_odd) {
        for (int pr = p_lo; pr < p_hi; ++pr) {
            const int kb = 2 * pr + h;
            const uint32_t kbw = (uint32_t)min(kb, KB - 1);
            const uint32_t ma = kb < KB ? mask_a[kb] : 0u, mw = kb < KB ? mask_w[kb] : 0u;
            if (__ballot((ma | mw) > 1u) == 0ull) continue;
            const uint4 codes = *reinterpret_cast<const uint4*>(wcodes + kbw * 512u);
            for (int ct = 1; ct <= kMaxClass; ++ct) {
                for (int ca = 0; ca <= ct; ++ca) {
                    const int cw = ct - ca;
                    const bool part = ((ma >> ca) & 1u) && ((mw >> cw) & 1u);
                    if (__ballot(part) == 0ull) continue;
                    const uint8_t* src = a8 + (uint64_t)ca * cls_stride + kbw * 1024u;
                    const v4i x0 = part ? *reinterpret_cast<const v4i*>(src) : zero4;
                    const v4i x1 = part ? *reinterpret_cast<const v4i*>(src + 512) : zero4;
                    const uint32_t mt = *reinterpret_cast<const uint32_t*>(
                        wmeta + (uint64_t)cw * p.wmeta_cls_stride + kbw * 128u);
                    const uint4 tab = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint8_t*>(s_tab) + mt);
                    const v4i b0 = unpack16(codes.x, codes.y, tab), b1 = unpack16(codes.z, codes.w, tab);
                    v16i t16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                    t16 = __builtin_amdgcn_mfma_i32_32x32x32_i8(x0, b0, t16, 0, 0, 0);
                    t16 = __builtin_amdgcn_mfma_i32_32x32x32_i8(x1, b1, t16, 0, 0, 0);
#pragma unroll
                    for (int x = 0; x < 16; ++x) acc[x] += t16[x] << (4 * ct);
                }
            }
        }
    }
    // the NW exact partial tiles: the upper half of the waves hands theirs to the lower, then thread
    // (x, lane) finishes one output
    if (wave >= NW / 2) {
#pragma unroll
        for (int x = 0; x < 16; ++x) u.red[wave - NW / 2][x][lane] = acc[x];
    }
    __syncthreads();
    if (wave < NW / 2) {
#pragma unroll
        for (int x = 0; x < 16; ++x) u.red[wave][x][lane] += acc[x];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16 / NW; ++i) {
        const int x = wave + i * NW;
        int sum = 0;
#pragma unroll
        for (int w = 0; w < NW / 2; ++w) sum += u.red[w][x][lane];
        const int m = m0 + 8 * (x >> 2) + 4 * h + (x & 3), n = n0 + r;
        if (m < p.M && n < p.N) {
            const float f = ldexpf((float)sum, ref_sum[i]);
            const int64_t o = (int64_t)m * p.ldc + n;
            if constexpr (BF16)
                static_cast<uint16_t*>(p.out)[o] = f32_to_bf16_rne(f);
            else
                static_cast<float*>(p.out)[o] = f;
        }
    }
}

// Whole product through the per-block flush (K beyond the single-accumulator kernel's limit).
template <bool MX, bool BF16>
__global__ __launch_bounds__(256) void gemm_block_kernel(GemmParams p) {
    __shared__ uint8_t s_exp[2][256];
    block_flush_tile<MX, BF16>(p, blockIdx.z, (int)blockIdx.y, (int)blockIdx.x, s_exp);
}

}  // namespace

// Largest operands the single-accumulator kernel addresses with its 32-bit offsets: the expanded
// A (all classes) and the 4-bit codes of W each stay below 2 GiB.  Larger products are cut into
// pieces of at most this many rows on the host.
static int64_t max_rows_a(int64_t KB) {
    const int64_t tiles = (((int64_t)1 << 31) - 1) / ((int64_t)(kMaxClass + 1) * kGroups * (KB + 1) * 1024);
    return (tiles < 65535 ? tiles : 65535) * kTileM;
}
static int64_t max_rows_w(int64_t KB) { return ((((int64_t)1 << 31) - 1) / (KB * 16)) / kTileN * kTileN; }

size_t gemm_prepared_bytes(int64_t rows, int64_t K, bool weight) {
    const int64_t KB = K / kBlock;
    if (rows <= 0 || KB <= 0 || KB > kMaxKB) return 0;
    return (size_t)(weight ? prep_w_layout(rows, KB).total : prep_a_layout(rows, KB).total);
}

// byte offset, inside a prepared A, of the dword that counts tiles declined since it was prepared
size_t gemm_prepared_declined_offset(int64_t M, int64_t K) {
    return (size_t)prep_a_layout(M, K / kBlock).off_cnt + (size_t)kMaxSplitTiles * 4;
}

size_t gemm_prepared_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    const int64_t KB = K / kBlock;
    if (M <= 0 || N <= 0 || !takes_fast_kernel(M, KB)) return 0;
    return (size_t)partial_bytes(M, N, KB, 1);
}

size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    const int64_t KB = K / kBlock;
    if (M <= 0 || N <= 0 || !takes_fast_kernel(M, KB)) return 0;
    const int64_t Mc = M < max_rows_a(KB) ? M : max_rows_a(KB), Nc = N < max_rows_w(KB) ? N : max_rows_w(KB);
    return (size_t)(prep_a_layout(Mc, KB).total + prep_w_layout(Nc, KB).total + partial_bytes(Mc, Nc, KB, 1));
}

size_t gemm_requant_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    if (M <= 0 || N <= 0) return 0;
    return (size_t)align256((int64_t)gemm_workspace_bytes(M, N, K)) + (size_t)align256(M * N * 2);
}

namespace {

template <typename F>
void dispatch_mx_bf16(bool mx, bool bf16, F&& f) {
    if (mx) {
        if (bf16) f(std::true_type{}, std::true_type{}); else f(std::true_type{}, std::false_type{});
    } else {
        if (bf16) f(std::false_type{}, std::true_type{}); else f(std::false_type{}, std::false_type{});
    }
}

void fill_params(GemmParams& p, const dfp4_tensor& A, const dfp4_tensor& W, void* out, int64_t ldc,
                 int64_t strideA_rows, int64_t strideW_rows, int64_t strideC, const dfp4_tensor* rq) {
    p.a_codes = A.codes; p.a_dial = A.dialect; p.a_exp = A.exponent;
    p.w_codes = W.codes; p.w_dial = W.dialect; p.w_exp = W.exponent;
    p.out = out; p.M = (int)A.rows; p.N = (int)W.rows; p.KB = (int)(A.K / kBlock);
    p.ldc = ldc; p.strideA_rows = strideA_rows; p.strideW_rows = strideW_rows; p.strideC = strideC;
    p.tiles_m = (int)((A.rows + kTileM - 1) / kTileM); p.tiles_n = (int)((W.rows + kTileN - 1) / kTileN);
    p.ksplit = 1;
    if (rq) {
        p.q_codes = reinterpret_cast<uint32_t*>(rq->codes); p.q_dial = rq->dialect; p.q_exp = rq->exponent;
    }
}

void set_prepared(GemmParams& p, uint8_t* a_prep, int64_t a_stride, uint8_t* w_prep, int64_t w_stride) {
    const PrepALayout la = prep_a_layout(p.M, p.KB);
    const PrepWLayout lw = prep_w_layout(p.N, p.KB);
    p.a_prep = a_prep; p.a_prep_stride = a_stride;
    p.w_prep = w_prep; p.w_prep_stride = w_stride;
    p.off_refa = la.off_refa; p.off_mask = la.off_mask; p.off_cnt = la.off_cnt; p.off_a8 = la.off_a8;
    p.off_refw = lw.off_refw; p.off_wmask = lw.off_wmask; p.off_wmeta = lw.off_wmeta; p.off_wcodes = lw.off_wcodes;
    p.wmeta_cls_stride = (uint32_t)((int64_t)p.tiles_n * kTileN * p.KB * 4);
}

// prepass: A workgroups (when do_a) and W workgroups (when do_w) in one launch
int launch_prep(bool mx, const GemmParams& p, bool do_a, bool do_w, int64_t batch, hipStream_t stream) {
    const int64_t KB = p.KB;
    const int chunks_a = (int)((KB + 7) / 8);
    const int64_t n_a = do_a ? (int64_t)p.tiles_m * chunks_a : 0;
    const int64_t n_w = do_w ? (int64_t)p.tiles_n * ((KB + 63) / 64) : 0;
    if (n_a + n_w == 0) return DFP4_OK;
    if (n_a + n_w > 0x7fffffff || batch > 65535) return DFP4_ERR_SHAPE;
    dim3 gp((unsigned)(n_a + n_w), 1, (unsigned)batch);
    if (mx)
        hipLaunchKernelGGL((gemm_prep_kernel<true>), gp, dim3(1024), 0, stream, p, (int)n_a, chunks_a);
    else
        hipLaunchKernelGGL((gemm_prep_kernel<false>), gp, dim3(1024), 0, stream, p, (int)n_a, chunks_a);
    return check_launch();
}

// single-accumulator kernel on prepared operands; `part`: room for the partial tiles where K is split
int launch_fast(bool mx, bool bf16, GemmParams& p, int64_t batch, int* part, size_t part_bytes, bool rq,
                hipStream_t stream) {
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    p.ksplit = choose_ksplit(tiles * batch, p.KB);
    const size_t per_batch = (size_t)p.ksplit * tiles * kTileM * kTileN * 4;
    if (p.ksplit > 1 && (!part || per_batch * (size_t)batch > part_bytes)) p.ksplit = 1;   // no room: no split
    p.part = part;
    p.part_stride = (int64_t)(per_batch / 4);
    if (batch * p.ksplit > 65535 || p.tiles_m > 65535) return DFP4_ERR_SHAPE;
    dim3 gf((unsigned)p.tiles_n, (unsigned)p.tiles_m, (unsigned)(batch * p.ksplit));
    if (rq) {
        if (mx) hipLaunchKernelGGL((gemm_fast_kernel<true, true, true>), gf, dim3(256), 0, stream, p);
        else hipLaunchKernelGGL((gemm_fast_kernel<false, true, true>), gf, dim3(256), 0, stream, p);
    } else {
        dispatch_mx_bf16(mx, bf16, [&](auto mxc, auto bc) {
            hipLaunchKernelGGL((gemm_fast_kernel<decltype(mxc)::value, decltype(bc)::value, false>), gf, dim3(256), 0,
                               stream, p);
        });
    }
    return check_launch();
}

// products the single-accumulator kernel does not take: few rows, or K beyond its limit
int launch_other(bool mx, bool bf16, GemmParams& p, int64_t batch, const dfp4_tensor* rq, hipStream_t stream) {
    if (batch > 65535) return DFP4_ERR_SHAPE;
    if (takes_small_kernel(p.M, p.KB)) {
        dim3 gs((unsigned)((p.N + 31) / 32), (unsigned)((p.M + 31) / 32), (unsigned)batch);
        // 16 waves per tile while every tile finds a compute unit of its own; 8 beyond that, so that two
        // workgroups share a unit (registers allow 16 waves per unit) instead of waiting for a second round
        const bool narrow = (int64_t)gs.x * gs.y * gs.z > device_cu_count();
        dispatch_mx_bf16(mx, bf16, [&](auto mxc, auto bc) {
            if (narrow)
                hipLaunchKernelGGL((gemm_small_kernel<decltype(mxc)::value, decltype(bc)::value, 8>), gs,
                                   dim3(8 * 64), 0, stream, p);
            else
                hipLaunchKernelGGL((gemm_small_kernel<decltype(mxc)::value, decltype(bc)::value, kSmallWaves>), gs,
                                   dim3(kSmallWaves * 64), 0, stream, p);
        });
    } else {
        dim3 gb((unsigned)((p.N + 127) / 128), (unsigned)((p.M + 127) / 128), (unsigned)batch);
        if (gb.y > 65535) return DFP4_ERR_SHAPE;
        dispatch_mx_bf16(mx, bf16, [&](auto mxc, auto bc) {
            hipLaunchKernelGGL((gemm_block_kernel<decltype(mxc)::value, decltype(bc)::value>), gb, dim3(256), 0,
                               stream, p);
        });
    }
    const int rc = check_launch();
    if (rc != DFP4_OK || !rq) return rc;
    // the bf16 temporary holds [batch * M, N]
    return launch_quantize(mx, p.out, (int64_t)p.M * batch, p.N, p.ldc, *rq, stream);
}

bool shape_in_range(int64_t M, int64_t N, int64_t KB, int64_t batch, int64_t ldc) {
    return M < (1 << 30) && N < (1 << 30) && KB < (1 << 26) && batch <= 65535 && ldc < (1 << 27);
}

}  // namespace

// Shape limits of launch_gemm, so that callers can refuse a product before they enqueue anything.
int gemm_shape_check(dfp4_tensor A, dfp4_tensor W, int64_t ldc, int64_t batch, bool rq) {
    const int64_t M = A.rows, N = W.rows, KB = A.K / kBlock;
    if (M == 0 || N == 0 || batch == 0) return DFP4_OK;
    if (!shape_in_range(M, N, KB, batch, ldc)) return DFP4_ERR_SHAPE;
    if (takes_fast_kernel(M, KB) && (rq || batch > 1) && (M > max_rows_a(KB) || N > max_rows_w(KB)))
        return DFP4_ERR_SHAPE;         // only the plain single product is cut into pieces
    if (!takes_fast_kernel(M, KB) && !takes_small_kernel(M, KB) && (M + 127) / 128 > 65535) return DFP4_ERR_SHAPE;
    return DFP4_OK;
}

// `rq` (optional): quantize the result along N into *rq.  `out` must then be a bf16 [batch * M, N]
// temporary (ldc = N): it receives the results of every path that does not quantize in its epilogue.
int launch_gemm(bool mx, dfp4_tensor A, dfp4_tensor W, void* out, int out_dtype, int64_t ldc,
                int64_t batch, int64_t strideA_rows, int64_t strideW_rows, int64_t strideC,
                void* workspace, size_t workspace_bytes, hipStream_t stream, const dfp4_tensor* rq) {
    const int64_t M = A.rows, N = W.rows, KB = A.K / kBlock;
    if (M == 0 || N == 0 || batch == 0) return DFP4_OK;
    int rc = gemm_shape_check(A, W, ldc, batch, rq != nullptr);
    if (rc != DFP4_OK) return rc;
    const bool bf16 = out_dtype == DFP4_BF16;
    if (!takes_fast_kernel(M, KB)) {
        GemmParams p{};
        fill_params(p, A, W, out, ldc, strideA_rows, strideW_rows, strideC, rq);
        return launch_other(mx, bf16, p, batch, rq, stream);
    }
    // pieces of at most mc x nc outputs (one piece for every product of ordinary size)
    const int64_t mc = M < max_rows_a(KB) ? M : max_rows_a(KB), nc = N < max_rows_w(KB) ? N : max_rows_w(KB);
    const PrepALayout la = prep_a_layout(mc, KB);
    const PrepWLayout lw = prep_w_layout(nc, KB);
    const size_t prep_bytes = (size_t)(la.total + lw.total) * (size_t)batch;
    if (!workspace || prep_bytes > workspace_bytes) return DFP4_ERR_WORKSPACE;
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    const size_t esz = bf16 ? 2 : 4;
    for (int64_t m0 = 0; m0 < M; m0 += mc) {
        for (int64_t n0 = 0; n0 < N; n0 += nc) {
            dfp4_tensor a = A, w = W;
            a.rows = M - m0 < mc ? M - m0 : mc;
            w.rows = N - n0 < nc ? N - n0 : nc;
            a.codes += m0 * KB * 16; a.exponent += m0 * KB; if (a.dialect) a.dialect += m0 * KB;
            w.codes += n0 * KB * 16; w.exponent += n0 * KB; if (w.dialect) w.dialect += n0 * KB;
            GemmParams p{};
            fill_params(p, a, w, static_cast<uint8_t*>(out) + (size_t)(m0 * ldc + n0) * esz, ldc, strideA_rows,
                        strideW_rows, strideC, rq);
            // the piece's own layouts (a last piece may be smaller), always within the room of a full one
            const PrepALayout pa = prep_a_layout(a.rows, KB);
            const PrepWLayout pw = prep_w_layout(w.rows, KB);
            set_prepared(p, ws, pa.total, ws + (size_t)la.total * batch, pw.total);
            rc = launch_prep(mx, p, n0 == 0, true, batch, stream);
            if (rc != DFP4_OK) return rc;
            rc = launch_fast(mx, bf16, p, batch, reinterpret_cast<int*>(ws + prep_bytes), workspace_bytes - prep_bytes,
                             rq != nullptr, stream);
            if (rc != DFP4_OK) return rc;
        }
    }
    return DFP4_OK;
}

// One operand prepared ahead of the product (weights: once; an activation: once for all the
// products that consume it).
int launch_gemm_prepare(bool mx, dfp4_tensor T, bool weight, void* prepared, hipStream_t stream) {
    const int64_t KB = T.K / kBlock;
    GemmParams p{};
    dfp4_tensor none{};
    none.K = T.K;
    if (weight) {
        if (T.rows > max_rows_w(KB)) return DFP4_ERR_SHAPE;
        fill_params(p, none, T, nullptr, 0, 0, 0, 0, nullptr);
    } else {
        if (T.rows > max_rows_a(KB)) return DFP4_ERR_SHAPE;
        fill_params(p, T, none, nullptr, 0, 0, 0, 0, nullptr);
    }
    set_prepared(p, static_cast<uint8_t*>(prepared), 0, static_cast<uint8_t*>(prepared), 0);
    return launch_prep(mx, p, !weight, weight, 1, stream);
}

int launch_gemm_block16(dfp4_tensor A, bool a16, dfp4_tensor W, bool w16, void* out, int out_dtype, int64_t ldc,
                        hipStream_t stream) {
    const int64_t M = A.rows, N = W.rows, KB = A.K / kBlock;
    if (M == 0 || N == 0) return DFP4_OK;
    if (!shape_in_range(M, N, KB, 1, ldc) || (M + 127) / 128 > 65535) return DFP4_ERR_SHAPE;
    GemmParams p{};
    fill_params(p, A, W, out, ldc, 0, 0, 0, nullptr);
    dim3 gb((unsigned)((N + 127) / 128), (unsigned)((M + 127) / 128), 1);
    if (out_dtype == DFP4_BF16)
        hipLaunchKernelGGL((gemm_block16_kernel<true>), gb, dim3(256), 0, stream, p, a16 ? 1 : 0, w16 ? 1 : 0);
    else
        hipLaunchKernelGGL((gemm_block16_kernel<false>), gb, dim3(256), 0, stream, p, a16 ? 1 : 0, w16 ? 1 : 0);
    return check_launch();
}

int launch_gemm_prepared(bool mx, dfp4_tensor A, void* a_prepared, dfp4_tensor W, const void* w_prepared, void* out,
                         int out_dtype, int64_t ldc, void* workspace, size_t workspace_bytes, hipStream_t stream) {
    const int64_t M = A.rows, N = W.rows, KB = A.K / kBlock;
    if (M == 0 || N == 0) return DFP4_OK;
    if (!shape_in_range(M, N, KB, 1, ldc)) return DFP4_ERR_SHAPE;
    const bool bf16 = out_dtype == DFP4_BF16;
    GemmParams p{};
    fill_params(p, A, W, out, ldc, 0, 0, 0, nullptr);
    if (KB == 0 || KB > kMaxKB) return launch_other(mx, bf16, p, 1, nullptr, stream);
    if (M > max_rows_a(KB) || N > max_rows_w(KB)) return DFP4_ERR_SHAPE;
    set_prepared(p, static_cast<uint8_t*>(a_prepared), 0, static_cast<uint8_t*>(const_cast<void*>(w_prepared)), 0);
    if (takes_small_kernel(M, KB)) {
        // few rows: the exact scheme in the shape of the few-rows kernel
        dim3 gs((unsigned)((N + 31) / 32), (unsigned)((M + 31) / 32), 1);
        const bool narrow = (int64_t)gs.x * gs.y > device_cu_count();     // as for gemm_small_kernel
        dispatch_mx_bf16(mx, bf16, [&](auto mxc, auto bc) {
            if (narrow)
                hipLaunchKernelGGL((gemm_rows_kernel<decltype(mxc)::value, decltype(bc)::value, 8>), gs,
                                   dim3(8 * 64), 0, stream, p);
            else
                hipLaunchKernelGGL((gemm_rows_kernel<decltype(mxc)::value, decltype(bc)::value, kSmallWaves>), gs,
                                   dim3(kSmallWaves * 64), 0, stream, p);
        });
        return check_launch();
    }
    return launch_fast(mx, bf16, p, 1, static_cast<int*>(workspace), workspace_bytes, false, stream);
}

}  // namespace dfp4
