// Code-unit unpacking shared by the weight preparation (host, to learn the slot
// order) and the rematerialisation kernel (device).
//
// A "unit" is 32 consecutive b-bit codes of one token row = b aligned dwords of the
// row's little-endian bit string.  UnpackUnit<b> turns it into 16 dwords, each a
// pair of fp16 SUBNORMALS: the code's bits are masked into the fp16 mantissa at bit
// offset o with a zero exponent field, which is the number code * 2^(o-24) exactly
// -- no integer->float conversion, no implicit leading one to remove (the fp16 MFMA
// takes subnormal operands at face value).  Dword 4*ks+v feeds k-step ks of the
// unit, elements 2v (low half) and 2v+1 (high half) of the MFMA operand.  Which
// code lands in which slot, and at which offset o, is a fixed permutation chosen to
// minimise shifts; the weight preparation discovers it by running this very
// function on probe inputs (build_unpack_table), so the two sides cannot disagree.
// The weight row of a code at offset o is scaled by 2^(10-o-b), so every product is
// code * W * 2^(-14-b); the kernel's pre-pass folds the constant into the per-group
// scale (effective scale e = scale * 2^(b+14)).
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define XQ_HD __host__ __device__ __forceinline__
#else
#define XQ_HD inline
#endif

namespace xq {

constexpr int F16_MANT_BITS = 10;
constexpr int F16_SUBNORMAL_EXP = 24;     // a subnormal with mantissa m is m * 2^-24

XQ_HD uint32_t field(uint32_t a, uint32_t m) { return a & m; }
XQ_HD uint32_t merge16(uint32_t lo_src, uint32_t hi_src)   // low half of lo_src, high half of hi_src
{
    return (lo_src & 0x0000FFFFu) | (hi_src & 0xFFFF0000u);
}
XQ_HD uint32_t funnel_r(uint32_t hi, uint32_t lo, int s)
{
    return (uint32_t)((((uint64_t)hi << 32) | lo) >> s);
}

// UnpackKStep<BITS, J>::run(w, out): the 4 operand dwords of k-step J (0..3) of a unit.
// `w` points at the unit's BITS dwords.
template <int BITS, int J>
struct UnpackKStep;

// Fields are placed as high in the 10-bit mantissa as the shared shifts allow: the MFMA aligns
// its products by their exponent fields, so every leading zero of a subnormal operand is a bit
// of accumulation precision given away.
//
// 4 bits: dword J holds the 8 codes of k-step J; pairs (v, v+4) sit 16 bits apart; offset 6.
template <int J>
struct UnpackKStep<4, J> {
    static XQ_HD void run(const uint32_t* w, uint32_t* out)
    {
        const uint32_t d = w[J];
        out[0] = field(d << 6, 0x03C003C0u);
        out[1] = field(d << 2, 0x03C003C0u);
        out[2] = field(d >> 2, 0x03C003C0u);
        out[3] = field(d >> 6, 0x03C003C0u);
    }
};

// 2 bits: one dword = 16 codes = two k-steps; pairs (v, v+8) sit 16 bits apart.
// Fields sit at mantissa offsets 6 or 8, so two shifted copies serve the 4 pairs of a k-step.
template <int J>
struct UnpackKStep<2, J> {
    static XQ_HD void run(const uint32_t* w, uint32_t* out)
    {
        const uint32_t d = w[J >> 1];
        const uint32_t a = (J & 1) ? d >> 2 : d << 6;    // codes 0,1 (4,5) at offsets 6,8
        const uint32_t b = (J & 1) ? d >> 6 : d << 2;    // codes 2,3 (6,7)
        out[0] = field(a, 0x00C000C0u);
        out[1] = field(a, 0x03000300u);
        out[2] = field(b, 0x00C000C0u);
        out[3] = field(b, 0x03000300u);
    }
};

// 3 bits: 96 bits in three dwords.  Codes p and p+16 are 48 bits apart, i.e. 16 bits
// apart once the right halves of two dwords are merged; fields go to offsets 4 or 7.
// Codes 5, 10, 21, 26 straddle a 16-bit boundary and are fetched with funnel shifts.
//   ea = lo16(d0)|hi16(d1): codes 0-4 | 16-20 at bit 0,3,6,9,12 of each half
//   eb = lo16(d2)|hi16(d0): codes 22-25 | 6-9  at bit 2,5,8,11
//   ec = lo16(d1)|hi16(d2): codes 11-15 | 27-31 at bit 1,4,7,10,13
template <int J>
struct UnpackKStep<3, J> {
    static XQ_HD void run(const uint32_t* w, uint32_t* out)
    {
        const uint32_t d0 = w[0], d1 = w[1], d2 = w[2];
        const uint32_t M4 = 0x00700070u, M7 = 0x03800380u;
        if (J == 0) {
            const uint32_t ea = merge16(d0, d1);
            const uint32_t a0 = ea << 4, a1 = ea >> 2;
            out[0] = field(a0, M4);                      // codes 0 | 16
            out[1] = field(a0, M7);                      //       1 | 17
            out[2] = field(a1, M4);                      //       2 | 18
            out[3] = field(a1, M7);                      //       3 | 19
        } else if (J == 1) {
            const uint32_t ea = merge16(d0, d1), eb = merge16(d2, d0);
            const uint32_t b0 = eb << 2;
            out[0] = field(ea >> 8, M4);                 //       4 | 20
            out[1] = field(b0, M4);                      //      22 | 6
            out[2] = field(b0, M7);                      //      23 | 7
            out[3] = field(eb >> 4, M4);                 //      24 | 8
        } else if (J == 2) {
            const uint32_t eb = merge16(d2, d0), ec = merge16(d1, d2);
            out[0] = field(eb >> 4, M7);                 //      25 | 9
            out[1] = field(ec, M4);                      //      12 | 28
            out[2] = field(ec, M7);                      //      13 | 29
            out[3] = field(ec << 3, M4);                 //      11 | 27
        } else {
            const uint32_t ec = merge16(d1, d2);
            const uint32_t c1 = ec >> 6;
            out[0] = field(c1, M4);                      //      14 | 30
            out[1] = field(c1, M7);                      //      15 | 31
            // code 5 (bits 15-17 of d0) with code 26 (bits 14-16 of d2)
            out[2] = field(merge16(d0 >> 11, d2 << 6), M4);
            // code 10 (bits 30-32 of the unit) with code 21 (bits 63-65)
            out[3] = field(merge16(funnel_r(d1, d0, 26), funnel_r(d2, d1, 11)), M4);
        }
    }
};

template <int BITS>
struct UnpackUnit {
    static XQ_HD void run(const uint32_t* w, uint32_t* out)
    {
        UnpackKStep<BITS, 0>::run(w, out);
        UnpackKStep<BITS, 1>::run(w, out + 4);
        UnpackKStep<BITS, 2>::run(w, out + 8);
        UnpackKStep<BITS, 3>::run(w, out + 12);
    }
};

// Slot order and mantissa offsets of UnpackUnit<BITS>, found by probing it.
struct UnpackTable {
    int8_t code_of_slot[4][8];   // [k-step in unit][operand element] -> code index 0..31
    int8_t wexp_of_code[32];     // weight-row exponent 10 - o - BITS for that code
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
    for (int i = 0; i < 16; ++i) ok = ok && base[i] == 0u;
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
            if (field != (((1u << BITS) - 1u) << o) || o + BITS > F16_MANT_BITS) ok = false;
            const int ks = i >> 2, el = 2 * (i & 3) + hi;
            if (seen_slot[ks][el]) ok = false;
            seen_slot[ks][el] = true;
            t.code_of_slot[ks][el] = (int8_t)p;
            t.wexp_of_code[p] = (int8_t)(F16_MANT_BITS - o - BITS);
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
                const int o = F16_MANT_BITS - BITS - t.wexp_of_code[p];
                const uint32_t val = (uint32_t)((p * 5 + 3) & ((1 << BITS) - 1));
                if (half != (val << o)) ok = false;
            }
    }
    t.valid = ok ? 1 : 0;
    return t;
}

}  // namespace xq
