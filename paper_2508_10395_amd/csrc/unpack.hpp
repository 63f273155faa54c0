// Code-unit unpacking shared by the weight preparation (host, to learn the slot
// order) and the rematerialisation kernel (device).
//
// A "unit" is 32 consecutive b-bit codes of one token row = b aligned dwords of the
// row's little-endian bit string.  unpack_unit<b> turns it into 16 dwords, each a
// pair of bf16 values of the form 1 + code * 2^(o-7): the code's bits are dropped
// straight into the bf16 mantissa at bit offset o under the exponent of 1.0
// (0x3F80), so no integer->float conversion is needed.  Dword 4*ks+v feeds
// k-step ks of the unit, elements 2v (low half) and 2v+1 (high half) of the MFMA
// operand.  Which code lands in which slot, and at which offset o, is a fixed
// permutation chosen to minimise shifts; the weight preparation discovers it by
// running this very function on probe inputs (build_unpack_table), so the two
// sides cannot disagree.  The factor 2^(o-7) and the "+1" are undone by scaling
// the matching weight row by 2^(7-o-b) and by a column-sum correction.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define XQ_HD __host__ __device__ __forceinline__
#else
#define XQ_HD inline
#endif

namespace xq {

constexpr uint32_t BF16_ONE_PAIR = 0x3F803F80u;

XQ_HD uint32_t and_or(uint32_t a, uint32_t m, uint32_t o) { return (a & m) | o; }
XQ_HD uint32_t funnel_r(uint32_t hi, uint32_t lo, int s)
{
    return (uint32_t)((((uint64_t)hi << 32) | lo) >> s);
}

template <int BITS>
struct UnpackUnit;

// 4 bits: dword ks holds the 8 codes of k-step ks; pairs (v, v+4) sit 16 bits apart.
template <>
struct UnpackUnit<4> {
    static XQ_HD void run(const uint32_t* w, uint32_t* out)
    {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const uint32_t d = w[ks];
            out[4 * ks + 0] = and_or(d << 3, 0x00780078u, BF16_ONE_PAIR);
            out[4 * ks + 1] = and_or(d >> 1, 0x00780078u, BF16_ONE_PAIR);
            out[4 * ks + 2] = and_or(d >> 5, 0x00780078u, BF16_ONE_PAIR);
            out[4 * ks + 3] = and_or(d >> 9, 0x00780078u, BF16_ONE_PAIR);
        }
    }
};

// 2 bits: one dword = 16 codes = two k-steps; pairs (v, v+8) sit 16 bits apart.
// Fields sit at mantissa offsets 3 or 5, so four shifted copies serve all 8 pairs.
template <>
struct UnpackUnit<2> {
    static XQ_HD void run(const uint32_t* w, uint32_t* out)
    {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t d = w[h];
            const uint32_t a = d << 3;    // codes 0,1 at offsets 3,5
            const uint32_t b = d >> 1;    // codes 2,3
            const uint32_t c = d >> 5;    // codes 4,5
            const uint32_t e = d >> 9;    // codes 6,7
            out[8 * h + 0] = and_or(a, 0x00180018u, BF16_ONE_PAIR);
            out[8 * h + 1] = and_or(a, 0x00600060u, BF16_ONE_PAIR);
            out[8 * h + 2] = and_or(b, 0x00180018u, BF16_ONE_PAIR);
            out[8 * h + 3] = and_or(b, 0x00600060u, BF16_ONE_PAIR);
            out[8 * h + 4] = and_or(c, 0x00180018u, BF16_ONE_PAIR);
            out[8 * h + 5] = and_or(c, 0x00600060u, BF16_ONE_PAIR);
            out[8 * h + 6] = and_or(e, 0x00180018u, BF16_ONE_PAIR);
            out[8 * h + 7] = and_or(e, 0x00600060u, BF16_ONE_PAIR);
        }
    }
};

// 3 bits: 96 bits in three dwords.  Codes p and p+16 are 48 bits apart, i.e. 16 bits
// apart once the right halves of two dwords are merged; fields go to offsets 1 or 4.
// Codes 5, 10, 21, 26 straddle a 16-bit boundary and are fetched with funnel shifts.
template <>
struct UnpackUnit<3> {
    static XQ_HD void run(const uint32_t* w, uint32_t* out)
    {
        const uint32_t d0 = w[0], d1 = w[1], d2 = w[2];
        const uint32_t ea = (d0 & 0x0000FFFFu) | (d1 & 0xFFFF0000u);   // codes 0-4 | 16-20 at 0,3,6,9,12
        const uint32_t eb = (d2 & 0x0000FFFFu) | (d0 & 0xFFFF0000u);   // codes 22-25 | 6-9 at 2,5,8,11
        const uint32_t ec = (d1 & 0x0000FFFFu) | (d2 & 0xFFFF0000u);   // codes 11-15 | 27-31 at 1,4,7,10,13
        const uint32_t M1 = 0x000E000Eu, M4 = 0x00700070u;
        const uint32_t a0 = ea << 1, a1 = ea >> 5, a2 = ea >> 11;
        out[0] = and_or(a0, M1, BF16_ONE_PAIR);
        out[1] = and_or(a0, M4, BF16_ONE_PAIR);
        out[2] = and_or(a1, M1, BF16_ONE_PAIR);
        out[3] = and_or(a1, M4, BF16_ONE_PAIR);
        out[4] = and_or(a2, M1, BF16_ONE_PAIR);
        const uint32_t b0 = eb >> 1, b1 = eb >> 7;
        out[5] = and_or(b0, M1, BF16_ONE_PAIR);
        out[6] = and_or(b0, M4, BF16_ONE_PAIR);
        out[7] = and_or(b1, M1, BF16_ONE_PAIR);
        out[8] = and_or(b1, M4, BF16_ONE_PAIR);
        const uint32_t c1 = ec >> 6, c2 = ec >> 12;
        out[9] = and_or(ec, M1, BF16_ONE_PAIR);
        out[10] = and_or(ec, M4, BF16_ONE_PAIR);
        out[11] = and_or(c1, M1, BF16_ONE_PAIR);
        out[12] = and_or(c1, M4, BF16_ONE_PAIR);
        out[13] = and_or(c2, M1, BF16_ONE_PAIR);
        // code 5 (bits 15-17 of d0) with code 26 (bits 14-16 of d2)
        const uint32_t x5 = d0 >> 14, y26 = d2 << 3;
        out[14] = and_or((x5 & 0x0000FFFFu) | (y26 & 0xFFFF0000u), M1, BF16_ONE_PAIR);
        // code 10 (bits 30-32 of the unit) with code 21 (bits 63-65)
        const uint32_t x10 = funnel_r(d1, d0, 29), y21 = funnel_r(d2, d1, 14);
        out[15] = and_or((x10 & 0x0000FFFFu) | (y21 & 0xFFFF0000u), M1, BF16_ONE_PAIR);
    }
};

// Slot order and mantissa offsets of UnpackUnit<BITS>, found by probing it.
struct UnpackTable {
    int8_t code_of_slot[4][8];   // [k-step in unit][operand element] -> code index 0..31
    int8_t wexp_of_code[32];     // weight-row exponent 7 - o - BITS for that code
    int8_t valid;
};

template <int BITS>
inline UnpackTable build_unpack_table()
{
    UnpackTable t{};
    uint32_t zero_in[4] = {0, 0, 0, 0}, base[16], out[16];
    UnpackUnit<BITS>::run(zero_in, base);
    bool ok = true;
    bool seen_slot[4][8] = {};
    for (int i = 0; i < 16; ++i) ok = ok && base[i] == BF16_ONE_PAIR;
    for (int p = 0; p < 32 && ok; ++p) {
        uint32_t in[4] = {0, 0, 0, 0};
        for (int k = 0; k < BITS; ++k) {
            const int bit = p * BITS + k;
            in[bit >> 5] |= 1u << (bit & 31);
        }
        UnpackUnit<BITS>::run(in, out);
        int hits = 0;
        for (int i = 0; i < 16; ++i) {
            const uint32_t diff = out[i] ^ base[i];
            if (!diff) continue;
            ++hits;
            const int hi = (diff >> 16) ? 1 : 0;
            const uint32_t field = hi ? (diff >> 16) : diff;
            if (hi && (diff & 0xFFFFu)) ok = false;
            int o = 0;
            while (o < 16 && !((field >> o) & 1u)) ++o;
            if (field != (((1u << BITS) - 1u) << o) || o + BITS > 7) ok = false;
            const int ks = i >> 2, el = 2 * (i & 3) + hi;
            if (seen_slot[ks][el]) ok = false;
            seen_slot[ks][el] = true;
            t.code_of_slot[ks][el] = (int8_t)p;
            t.wexp_of_code[p] = (int8_t)(7 - o - BITS);
        }
        if (hits != 1) ok = false;
    }
    // every code value must arrive unchanged: probe a second pattern (alternating values)
    if (ok) {
        uint32_t in[4] = {0, 0, 0, 0};
        for (int p = 0; p < 32; ++p) {
            const uint32_t val = (uint32_t)((p * 5 + 3) & ((1 << BITS) - 1));
            for (int k = 0; k < BITS; ++k)
                if ((val >> k) & 1u) {
                    const int bit = p * BITS + k;
                    in[bit >> 5] |= 1u << (bit & 31);
                }
        }
        UnpackUnit<BITS>::run(in, out);
        for (int ks = 0; ks < 4; ++ks)
            for (int el = 0; el < 8; ++el) {
                const int p = t.code_of_slot[ks][el];
                const uint32_t half = (out[4 * ks + el / 2] >> ((el & 1) * 16)) & 0xFFFFu;
                const int o = 7 - BITS - t.wexp_of_code[p];
                const uint32_t val = (uint32_t)((p * 5 + 3) & ((1 << BITS) - 1));
                if (half != (0x3F80u | (val << o))) ok = false;
            }
    }
    t.valid = ok ? 1 : 0;
    return t;
}

}  // namespace xq
