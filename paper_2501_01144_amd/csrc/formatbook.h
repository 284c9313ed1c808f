// DialectFP4 formatbook and the lookup tables the kernels derive from it.
//
// The book (Section 3.1 of the paper, 16-dialect DialectFP4 example) is data:
// 16 dialects x 8 magnitudes in half-units (value = 0.5 * u, u in 0..15),
// ascending, position = 3-bit index.  Dialects 2p and 2p+1 form pair p and
// share the largest magnitude 7.5 - 0.5 p.  Rows 4 and 5 are the ones the
// paper prints (Sections 3.2 and 3.3); the remaining rows follow the three
// formatbook criteria of Section 3.1.  Everything else in this header is
// computed from the book at compile time, so replacing a row changes no code.
#pragma once
#include <stdint.h>

namespace dfp4 {

constexpr int kBlock = 32;
constexpr int kDialects = 16;
constexpr int kPairs = 8;

constexpr uint8_t kBook[kDialects][8] = {
    {0, 1, 2, 3, 4, 6, 12, 15}, {0, 1, 2, 3, 4, 6, 10, 15},   // 7.5
    {0, 1, 2, 3, 4, 6, 11, 14}, {0, 1, 2, 3, 4, 6,  9, 14},   // 7.0
    {0, 1, 2, 3, 4, 6, 10, 13}, {0, 1, 2, 3, 4, 6,  8, 13},   // 6.5
    {0, 1, 2, 3, 4, 6,  9, 12}, {0, 1, 2, 3, 4, 6,  8, 12},   // 6.0 (odd one is FP4 E2M1)
    {0, 1, 2, 3, 4, 6,  9, 11}, {0, 1, 2, 3, 4, 6,  8, 11},   // 5.5
    {0, 1, 2, 3, 4, 6,  8, 10}, {0, 1, 2, 3, 4, 6,  7, 10},   // 5.0
    {0, 1, 2, 3, 4, 6,  8,  9}, {0, 1, 2, 3, 4, 6,  7,  9},   // 4.5
    {0, 1, 2, 3, 4, 6,  7,  8}, {0, 1, 2, 3, 4, 5,  6,  8},   // 4.0
};

// FP4 E2M1 magnitudes in half-units (the MXFP4 element format).
constexpr uint8_t kE2M1[8] = {0, 1, 2, 3, 4, 6, 8, 12};

// Index of the nearest magnitude of dialect d for a 5-bit magnitude t
// (quarter-units, t = floor(4 s)).  The midpoint of two neighbouring
// half-unit values a < b is (a + b) quarter-units; a magnitude on the
// midpoint goes up (Section 3.3: [4.0, 5.75) -> 5.0 in dialect 4).
constexpr int nearest_index(int d, int t) {
    int idx = 0;
    for (int j = 1; j < 8; ++j)
        if (t >= kBook[d][j - 1] + kBook[d][j]) idx = j;
    return idx;
}

constexpr bool book_has(int d, int u) {
    for (int j = 0; j < 8; ++j)
        if (kBook[d][j] == u) return true;
    return false;
}

// Beneficial range of dialect d (Section 3.2, second stage) in quarter-units,
// [lo, hi): the cell of d's own differing value among all values of its pair.
struct Range { int lo, hi; };
constexpr Range beneficial_range(int d) {
    int mine = -1;
    for (int j = 0; j < 8; ++j)
        if (!book_has(d ^ 1, kBook[d][j])) mine = kBook[d][j];
    int below = -1, above = 99;
    for (int dd = d & ~1; dd <= (d | 1); ++dd)
        for (int j = 0; j < 8; ++j) {
            int u = kBook[dd][j];
            if (u < mine && u > below) below = u;
            if (u > mine && u < above) above = u;
        }
    return Range{below + mine, mine + above};
}

constexpr bool in_range(int d, int t) {
    Range r = beneficial_range(d);
    return t >= r.lo && t < r.hi;
}

// E2M1 index for key = 2 t + sticky (sticky: the magnitude has bits below the
// quarter-unit): round to nearest, ties to the even index, saturating.
constexpr int e2m1_index(int key) {
    int t = key >> 1, sticky = key & 1, idx = 0;
    for (int j = 1; j < 8; ++j) {
        int mid = kE2M1[j - 1] + kE2M1[j];
        if (t > mid || (t == mid && (sticky || (j % 2 == 0)))) idx = j;
    }
    return idx;
}

// Lookup tables over a PAIR of 5-bit magnitudes, key = t0 | t1 << 5.
//   q[d][key]  = index(t0) | index(t1) << 4 under dialect d   (two code nibbles, no sign)
//   s[p][key]  = (votes for the even dialect of pair p) - (votes for the odd one), int8 in -2..2
//   mx[key64]  = E2M1 index for one element with key = 2 t + sticky
//   near_i[d][t], near_u[d][t] = index / half-unit value of dialect d nearest to a single magnitude t
struct QuantTables {
    uint8_t q[kDialects * 1024];
    uint8_t s[kPairs * 1024];
    uint8_t mx[64];
    uint8_t near_i[kDialects * 32];
    uint8_t near_u[kDialects * 32];
    uint8_t vote1[kPairs * 32];          // vote of a single magnitude in pair p: +1 even dialect, -1 odd (int8)
};

constexpr QuantTables make_quant_tables() {
    QuantTables T{};
    for (int d = 0; d < kDialects; ++d) {
        uint8_t one[32] = {};
        for (int t = 0; t < 32; ++t) one[t] = (uint8_t)nearest_index(d, t);
        for (int k = 0; k < 1024; ++k)
            T.q[d * 1024 + k] = (uint8_t)(one[k & 31] | (one[k >> 5] << 4));
    }
    for (int p = 0; p < kPairs; ++p) {
        // votes of the two magnitudes of a key: +1 for the even dialect's range, -1 for the odd one's
        int one[32] = {};
        for (int t = 0; t < 32; ++t)
            one[t] = (in_range(2 * p, t) ? 1 : 0) - (in_range(2 * p + 1, t) ? 1 : 0);
        for (int k = 0; k < 1024; ++k)
            T.s[p * 1024 + k] = (uint8_t)(one[k & 31] + one[k >> 5]);      // int8, two's complement
    }
    for (int k = 0; k < 64; ++k) T.mx[k] = (uint8_t)e2m1_index(k);
    for (int d = 0; d < kDialects; ++d)
        for (int t = 0; t < 32; ++t) {
            T.near_i[d * 32 + t] = (uint8_t)nearest_index(d, t);
            T.near_u[d * 32 + t] = kBook[d][nearest_index(d, t)];
        }
    for (int p = 0; p < kPairs; ++p)
        for (int t = 0; t < 32; ++t)
            T.vote1[p * 32 + t] = (uint8_t)((in_range(2 * p, t) ? 1 : 0) - (in_range(2 * p + 1, t) ? 1 : 0));
    return T;
}

}  // namespace dfp4
