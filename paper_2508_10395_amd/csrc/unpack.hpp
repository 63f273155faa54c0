// Code-unit unpacking shared by the weight preparation (host, to learn the slot
// order) and the rematerialisation kernel (device).
//
// A "unit" is 32 consecutive b-bit codes of one token row = b aligned dwords of the
// row's little-endian bit string.  UnpackUnit<b> turns it into 16 dwords, each a
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

// (a & m) | BF16_ONE_PAIR.  On the device this is one v_and_or_b32: gfx9 VOP3 takes at
// most one scalar/literal operand, so the mask goes in an SGPR and the constant in a VGPR.
XQ_HD uint32_t and_or_one(uint32_t a, uint32_t m, uint32_t one_vgpr)
{
#if defined(__HIP_DEVICE_COMPILE__)
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "s"(m), "v"(one_vgpr));
    return r;
#else
    return (a & m) | one_vgpr;
#endif
}
XQ_HD uint32_t merge16(uint32_t lo_src, uint32_t hi_src)   // low half of lo_src, high half of hi_src
{
    return (lo_src & 0x0000FFFFu) | (hi_src & 0xFFFF0000u);
}
XQ_HD uint32_t funnel_r(uint32_t hi, uint32_t lo, int s)
{
    return (uint32_t)((((uint64_t)hi << 32) | lo) >> s);
}

// UnpackKStep<BITS, J>::run(w, one, out): the 4 operand dwords of k-step J (0..3) of a unit.
// `w` points at the unit's BITS dwords; `one` must hold BF16_ONE_PAIR.
template <int BITS, int J>
struct UnpackKStep;

// 4 bits: dword J holds the 8 codes of k-step J; pairs (v, v+4) sit 16 bits apart.
template <int J>
struct UnpackKStep<4, J> {
    static XQ_HD void run(const uint32_t* w, uint32_t one, uint32_t* out)
    {
        const uint32_t d = w[J];
        out[0] = and_or_one(d << 3, 0x00780078u, one);
        out[1] = and_or_one(d >> 1, 0x00780078u, one);
        out[2] = and_or_one(d >> 5, 0x00780078u, one);
        out[3] = and_or_one(d >> 9, 0x00780078u, one);
    }
};

// 2 bits: one dword = 16 codes = two k-steps; pairs (v, v+8) sit 16 bits apart.
// Fields sit at mantissa offsets 3 or 5, so two shifted copies serve the 4 pairs of a k-step.
template <int J>
struct UnpackKStep<2, J> {
    static XQ_HD void run(const uint32_t* w, uint32_t one, uint32_t* out)
    {
        const uint32_t d = w[J >> 1];
        const uint32_t a = (J & 1) ? d >> 5 : d << 3;    // codes 0,1 (4,5) at offsets 3,5
        const uint32_t b = (J & 1) ? d >> 9 : d >> 1;    // codes 2,3 (6,7)
        out[0] = and_or_one(a, 0x00180018u, one);
        out[1] = and_or_one(a, 0x00600060u, one);
        out[2] = and_or_one(b, 0x00180018u, one);
        out[3] = and_or_one(b, 0x00600060u, one);
    }
};

// 3 bits: 96 bits in three dwords.  Codes p and p+16 are 48 bits apart, i.e. 16 bits
// apart once the right halves of two dwords are merged; fields go to offsets 1 or 4.
// Codes 5, 10, 21, 26 straddle a 16-bit boundary and are fetched with funnel shifts.
//   ea = lo16(d0)|hi16(d1): codes 0-4 | 16-20 at bit 0,3,6,9,12 of each half
//   eb = lo16(d2)|hi16(d0): codes 22-25 | 6-9  at bit 2,5,8,11
//   ec = lo16(d1)|hi16(d2): codes 11-15 | 27-31 at bit 1,4,7,10,13
template <int J>
struct UnpackKStep<3, J> {
    static XQ_HD void run(const uint32_t* w, uint32_t one, uint32_t* out)
    {
        const uint32_t d0 = w[0], d1 = w[1], d2 = w[2];
        const uint32_t M1 = 0x000E000Eu, M4 = 0x00700070u;
        if (J == 0) {
            const uint32_t ea = merge16(d0, d1);
            const uint32_t a0 = ea << 1, a1 = ea >> 5;
            out[0] = and_or_one(a0, M1, one);
            out[1] = and_or_one(a0, M4, one);
            out[2] = and_or_one(a1, M1, one);
            out[3] = and_or_one(a1, M4, one);
        } else if (J == 1) {
            const uint32_t ea = merge16(d0, d1), eb = merge16(d2, d0);
            const uint32_t b0 = eb >> 1, b1 = eb >> 7;
            out[0] = and_or_one(ea >> 11, M1, one);
            out[1] = and_or_one(b0, M1, one);
            out[2] = and_or_one(b0, M4, one);
            out[3] = and_or_one(b1, M1, one);
        } else if (J == 2) {
            const uint32_t eb = merge16(d2, d0), ec = merge16(d1, d2);
            const uint32_t c1 = ec >> 6;
            out[0] = and_or_one(eb >> 7, M4, one);
            out[1] = and_or_one(ec, M1, one);
            out[2] = and_or_one(ec, M4, one);
            out[3] = and_or_one(c1, M1, one);
        } else {
            const uint32_t ec = merge16(d1, d2);
            out[0] = and_or_one(ec >> 6, M4, one);
            out[1] = and_or_one(ec >> 12, M1, one);
            // code 5 (bits 15-17 of d0) with code 26 (bits 14-16 of d2)
            out[2] = and_or_one(merge16(d0 >> 14, d2 << 3), M1, one);
            // code 10 (bits 30-32 of the unit) with code 21 (bits 63-65)
            out[3] = and_or_one(merge16(funnel_r(d1, d0, 29), funnel_r(d2, d1, 14)), M1, one);
        }
    }
};

template <int BITS>
struct UnpackUnit {
    static XQ_HD void run(const uint32_t* w, uint32_t* out)
    {
        UnpackKStep<BITS, 0>::run(w, BF16_ONE_PAIR, out);
        UnpackKStep<BITS, 1>::run(w, BF16_ONE_PAIR, out + 4);
        UnpackKStep<BITS, 2>::run(w, BF16_ONE_PAIR, out + 8);
        UnpackKStep<BITS, 3>::run(w, BF16_ONE_PAIR, out + 12);
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
