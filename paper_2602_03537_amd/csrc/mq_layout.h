// Packed weight layout shared by the pack/unpack kernels and the linear kernels.
//
// W [N,K] is cut into tiles of 64 rows x 128 columns (one quantisation group).
// Tile (rb, g) lives at uint4 index ((rb*G + g)*R + i)*64 + lane, i = 0..R-1:
// a wavefront fetches it with R coalesced 16-byte loads and lane l then holds
// the whole group of row rb*64+l in 4R dwords ("lane dwords").
//
// Lane dwords are split into units of UD dwords.  Each 16-bit half of a dword
// is an independent container: the low half carries even columns, the high
// half the following odd column, so that one masked dword is an fp16 pair that
// meets the activation pair (x[2p], x[2p+1]).  A unit carries PPU such pairs.
// A code is stored as one or more bit-fields ("ops").  Every field sits, after
// an optional right shift of the whole dword, inside mantissa bits 0..9 of its
// half, so  (dword >> sh) & (mask * 0x10001)  is a pair of fp16 SUBNORMALS with
// value  digit * 2^(p-24)  where p = ctz(mask) and digit are `bits` bits of the
// code starting at bit d.  gfx950's v_dot2_f32_f16 and f16 MFMA take fp16
// subnormals at full rate and exactly, so no int->float conversion is issued.
// Fields with equal (p - d) share one fp32 accumulator ("key"); the group total
// is  sum_key acc[key] * 2^(24 - (p-d))  in units of the r-bit code.
//
// Section 4 of the paper splits 2..4-bit codes over three buffers (2+1+1 bits)
// so that widths share storage; here every width has its own dense layout and
// exactly r bits per weight are streamed.
#pragma once
#include <stdint.h>

namespace mq {

constexpr int kRowBlock = 64;   // rows per tile == lanes per wavefront
constexpr int kGroup = 128;     // columns per tile == quantisation group
constexpr int kC = 8;           // master bit-width of the parent

struct Op {
    int dw;    // dword inside the unit
    int sh;    // right shift applied to the dword before masking (0 = none)
    int mask;  // 16-bit mask after the shift (replicated to both halves)
    int d;     // first bit of the code this field carries
    int pair;  // activation pair inside the unit
};

constexpr int ctz16(int m) { int p = 0; while (!((m >> p) & 1)) ++p; return p; }
constexpr int popc16(int m) { int c = 0; for (int i = 0; i < 16; ++i) c += (m >> i) & 1; return c; }

template <int R> struct Layout;

// r = 2: eight codes per half.  Bits 0..9 hold five, bits 10..15 three more (one shift).
template <> struct Layout<2> {
    static constexpr int UD = 1, PPU = 8, NOPS = 8, NKEYS = 5;
    static constexpr Op op(int i) {
        constexpr Op t[NOPS] = {{0, 0, 0x0003, 0, 0},  {0, 0, 0x000C, 0, 1},  {0, 0, 0x0030, 0, 2},
                                {0, 0, 0x00C0, 0, 3},  {0, 0, 0x0300, 0, 4},  {0, 10, 0x0003, 0, 5},
                                {0, 10, 0x000C, 0, 6}, {0, 10, 0x0030, 0, 7}};
        return t[i];
    }
    static constexpr int key(int k) { constexpr int t[NKEYS] = {0, 2, 4, 6, 8}; return t[k]; }
};

// r = 3: a unit of three dwords holds 16 pairs.  Each half: five codes (15 bits)
// plus one bit of the 16th code (bit 15 of halves A, B, C = bits 0, 1, 2).
template <> struct Layout<3> {
    static constexpr int UD = 3, PPU = 16, NOPS = 18, NKEYS = 5;
    static constexpr Op op(int i) {
        constexpr Op t[NOPS] = {
            {0, 0, 0x0007, 0, 0},  {0, 0, 0x0038, 0, 1},  {0, 0, 0x01C0, 0, 2},  {0, 9, 0x0007, 0, 3},  {0, 9, 0x0038, 0, 4},
            {1, 0, 0x0007, 0, 5},  {1, 0, 0x0038, 0, 6},  {1, 0, 0x01C0, 0, 7},  {1, 9, 0x0007, 0, 8},  {1, 9, 0x0038, 0, 9},
            {2, 0, 0x0007, 0, 10}, {2, 0, 0x0038, 0, 11}, {2, 0, 0x01C0, 0, 12}, {2, 9, 0x0007, 0, 13}, {2, 9, 0x0038, 0, 14},
            {0, 9, 0x0040, 0, 15}, {1, 9, 0x0040, 1, 15}, {2, 9, 0x0040, 2, 15}};
        return t[i];
    }
    static constexpr int key(int k) { constexpr int t[NKEYS] = {0, 3, 6, 5, 4}; return t[k]; }
};

// r = 4: four codes per half; the upper two after a shift by 8.
template <> struct Layout<4> {
    static constexpr int UD = 1, PPU = 4, NOPS = 4, NKEYS = 2;
    static constexpr Op op(int i) {
        constexpr Op t[NOPS] = {{0, 0, 0x000F, 0, 0}, {0, 0, 0x00F0, 0, 1}, {0, 8, 0x000F, 0, 2}, {0, 8, 0x00F0, 0, 3}};
        return t[i];
    }
    static constexpr int key(int k) { constexpr int t[NKEYS] = {0, 4}; return t[k]; }
};

// r = 6: a unit of three dwords holds 8 pairs.  Each half: two whole codes
// (bits 0..5 and 6..11) and four spare bits; pair 6 = B[12:13] + 4*A[12:15],
// pair 7 = C[12:15] + 16*B[14:15], chosen so that only three keys occur.
template <> struct Layout<6> {
    static constexpr int UD = 3, PPU = 8, NOPS = 10, NKEYS = 3;
    static constexpr Op op(int i) {
        constexpr Op t[NOPS] = {{0, 0, 0x003F, 0, 0}, {0, 6, 0x003F, 0, 1}, {1, 0, 0x003F, 0, 2}, {1, 6, 0x003F, 0, 3},
                                {2, 0, 0x003F, 0, 4}, {2, 6, 0x003F, 0, 5}, {1, 6, 0x00C0, 0, 6}, {0, 6, 0x03C0, 2, 6},
                                {2, 6, 0x03C0, 0, 7}, {1, 6, 0x0300, 4, 7}};
        return t[i];
    }
    static constexpr int key(int k) { constexpr int t[NKEYS] = {0, 6, 4}; return t[k]; }
};

// r = 8: two codes per half, the upper after a shift by 8.
template <> struct Layout<8> {
    static constexpr int UD = 1, PPU = 2, NOPS = 2, NKEYS = 1;
    static constexpr Op op(int i) {
        constexpr Op t[NOPS] = {{0, 0, 0x00FF, 0, 0}, {0, 8, 0x00FF, 0, 1}};
        return t[i];
    }
    static constexpr int key(int k) { constexpr int t[NKEYS] = {0}; return t[k]; }
};

// accumulator index of an op: position of (p - d) in the key list
template <int R> constexpr int key_index(int i) {
    const Op o = Layout<R>::op(i);
    const int kd = ctz16(o.mask) - o.d;
    for (int k = 0; k < Layout<R>::NKEYS; ++k)
        if (Layout<R>::key(k) == kd) return k;
    return -1;
}

// Compile-time self-check of a layout: every op maps to a key, the fields of a
// unit tile its UD*32 bits exactly once, and each pair's fields cover bits 0..R-1 once.
template <int R> constexpr bool layout_ok() {
    using T = Layout<R>;
    if ((4 * R) % T::UD) return false;
    if (T::PPU * 2 * R != T::UD * 32) return false;
    unsigned used[4] = {0, 0, 0, 0};
    for (int i = 0; i < T::NOPS; ++i) {
        const Op o = T::op(i);
        if (key_index<R>(i) < 0) return false;
        if (o.mask & ~0x03FF) return false;  // must stay inside the fp16 mantissa
        const unsigned field = ((unsigned)o.mask << o.sh) & 0xFFFFu;
        if (popc16((int)field) != popc16(o.mask)) return false;  // shifted out of the half
        if (used[o.dw] & field) return false;
        used[o.dw] |= field;
    }
    for (int dw = 0; dw < T::UD; ++dw)
        if (used[dw] != 0xFFFFu) return false;
    for (int p = 0; p < T::PPU; ++p) {
        unsigned bits = 0;
        for (int i = 0; i < T::NOPS; ++i) {
            const Op o = T::op(i);
            if (o.pair != p) continue;
            const unsigned f = (unsigned)(o.mask >> ctz16(o.mask)) << o.d;
            if (bits & f) return false;
            bits |= f;
        }
        if (bits != (1u << R) - 1u) return false;
    }
    return true;
}
static_assert(layout_ok<2>() && layout_ok<3>() && layout_ok<4>() && layout_ok<6>() && layout_ok<8>(),
              "inconsistent packed layout table");

}  // namespace mq
