// Quantise-and-append kernels: X cache rows (Sec. 3.1) and cross-layer delta rows
// (Sec. 3.2) of arxiv 2508.10395.  HBM-streaming: one workgroup per token row, every
// lane loads 16 consecutive bf16 channels (32 B), a group of G channels lives in G/16
// adjacent lanes of one DPP row, min/max are reduced with DPP, the b-bit codes are
// packed in registers and written as the row's little-endian bit string.  The grid
// is (token, sequence), so no index arithmetic beyond a few multiplies is needed.
#include "common.hpp"

namespace xq {

// Exactly rounded codes without a per-element IEEE divide.
//
// The definition is code = rint(fl32((x - zero)/scale)).  scale has an 8-bit
// significand (bf16), so fl32(n/scale) lands on k+0.5 only when n equals the fp32
// number (k+0.5)*scale exactly, and lies on the same side of k+0.5 as the real
// quotient otherwise.  Hence any y = RN(q*(1+e)) with |e| << 2^-33 gives
// rint(y) == rint(fl32(n/scale)).  y is formed from a two-term reciprocal
// rh + rl = 1/scale * (1 + O(2^-44)):  y = fma(n, rh, n*rl).
struct GroupRecip {
    float rh, rl;
};
__device__ __forceinline__ GroupRecip make_recip(float sf)
{
    GroupRecip r;
    float rh = __builtin_amdgcn_rcpf(sf);
    float e = __builtin_fmaf(-sf, rh, 1.0f);   // exact residual
    float rl = e * rh;
    bool ok = sf != 0.0f;
    r.rh = ok ? rh : 0.0f;
    r.rl = ok ? rl : 0.0f;
    return r;
}

template <int LANES>
__device__ __forceinline__ void group_minmax(float& mn, float& mx)
{
    mn = fminf(mn, dpp_f32<DPP_QUAD_XOR1>(mn));
    mx = fmaxf(mx, dpp_f32<DPP_QUAD_XOR1>(mx));
    mn = fminf(mn, dpp_f32<DPP_QUAD_XOR2>(mn));
    mx = fmaxf(mx, dpp_f32<DPP_QUAD_XOR2>(mx));
    if constexpr (LANES == 8) {
        mn = fminf(mn, dpp_f32<DPP_ROW_HALF_MIRROR>(mn));
        mx = fmaxf(mx, dpp_f32<DPP_ROW_HALF_MIRROR>(mx));
    }
}

// Rounding and packing without a convert per element: for 0 <= y < 2^22, y + 2^23 (one fp32 add,
// round-to-nearest-even) is the float whose bit pattern is 0x4B000000 + rint(y); clamping that
// float to [2^23, 2^23 + qmax] clamps the code (the bounds are integers, so rounding first and
// clamping second gives the same code).  The packed word is then a sum of shifted bit patterns,
// and the shifted constants are taken out once per word (arithmetic modulo 2^32).
constexpr float ROUND_MAGIC = 8388608.0f;
constexpr uint32_t ROUND_MAGIC_BITS = 0x4B000000u;
constexpr uint32_t magic_sum(int n, int bits)
{
    uint32_t c = 0;
    for (int k = 0; k < n; ++k) c += ROUND_MAGIC_BITS << (bits * k);
    return c;
}

struct __attribute__((packed, aligned(4))) Dword2 {
    uint32_t a, b;
};

__device__ __forceinline__ void unpack8(const uint4& raw, float* v)
{
    v[0] = bf16_lo_to_f32(raw.x); v[1] = bf16_hi_to_f32(raw.x);
    v[2] = bf16_lo_to_f32(raw.y); v[3] = bf16_hi_to_f32(raw.y);
    v[4] = bf16_lo_to_f32(raw.z); v[5] = bf16_hi_to_f32(raw.z);
    v[6] = bf16_lo_to_f32(raw.w); v[7] = bf16_hi_to_f32(raw.w);
}

// Packs the 16 codes of one lane (bit patterns 0x4B000000 + code) into the row's little-endian bit
// string and stores them: lane `pi` owns bits [16 pi BITS, 16 (pi + 1) BITS) of the row at rowp.
template <int BITS>
__device__ __forceinline__ void pack_store16(const uint32_t (&q)[16], uint8_t* rowp, int pi, bool live)
{
    if constexpr (BITS == 8) {
        constexpr uint32_t C = magic_sum(4, 8);
        uint4 w;
        w.x = q[0] + (q[1] << 8) + (q[2] << 16) + (q[3] << 24) - C;
        w.y = q[4] + (q[5] << 8) + (q[6] << 16) + (q[7] << 24) - C;
        w.z = q[8] + (q[9] << 8) + (q[10] << 16) + (q[11] << 24) - C;
        w.w = q[12] + (q[13] << 8) + (q[14] << 16) + (q[15] << 24) - C;
        if (live) reinterpret_cast<uint4*>(rowp)[pi] = w;
    } else if constexpr (BITS == 4) {
        constexpr uint32_t C = magic_sum(8, 4);
        uint2 w = {0u - C, 0u - C};
#pragma unroll
        for (int k = 0; k < 8; ++k) { w.x += q[k] << (4 * k); w.y += q[8 + k] << (4 * k); }
        if (live) reinterpret_cast<uint2*>(rowp)[pi] = w;
    } else if constexpr (BITS == 2) {
        uint32_t w = 0u - magic_sum(16, 2);
#pragma unroll
        for (int k = 0; k < 16; ++k) w += q[k] << (2 * k);
        if (live) reinterpret_cast<uint32_t*>(rowp)[pi] = w;
    } else {   // 3 bits: 48 bits per lane, two lanes make three dwords
        constexpr uint32_t C = magic_sum(8, 3);
        uint32_t w0 = 0u - C, w1 = 0u - C;                           // 24 bits of codes each
#pragma unroll
        for (int k = 0; k < 8; ++k) { w0 += q[k] << (3 * k); w1 += q[8 + k] << (3 * k); }
        const uint32_t lo = w0 | (w1 << 24), hi = w1 >> 8;          // bits 0-31, 32-47
        const uint32_t lo_other = dpp_u32<DPP_QUAD_XOR1>(lo);
        uint8_t* pair = rowp + 12 * (pi >> 1);
        if (live) {
            if ((pi & 1) == 0) {
                Dword2 w; w.a = lo; w.b = hi | (lo_other << 16);
                *reinterpret_cast<Dword2*>(pair) = w;
            } else {
                reinterpret_cast<uint32_t*>(pair)[2] = (lo >> 16) | (hi << 16);
            }
        }
    }
}

// Workgroup (t, b) quantises input row b*T + t into cache row b*cap + start[b] + t; a thread
// takes 16 consecutive channels at a time.  In DELTA mode the value quantised is
// x - acc[b][start[b]+t] (fp32).  d/16 is a multiple of G/16, so a group's lanes are either all
// inside the row or all past it (those recompute the row's last piece and store nothing).
template <int BITS, int G, bool DELTA>
__global__ __launch_bounds__(256) void quantize_append_kernel(
    const uint4* __restrict__ x, const uint4* __restrict__ acc, uint8_t* __restrict__ codes,
    uint16_t* __restrict__ scale, uint16_t* __restrict__ zero, int T, int cap, int d, BatchI32 start)
{
    constexpr int LANES = G / 16;
    constexpr float QMAX = (float)((1 << BITS) - 1);
    const int t = blockIdx.x, b = blockIdx.y;
    const long long row_in = (long long)b * T + t;
    const long long row_out = (long long)b * cap + start.v[b] + t;
    const int ppr = d >> 4;                               // 16-channel pieces per row
    const uint4* xr = x + row_in * (d >> 3);
    const uint4* ar = DELTA ? acc + row_out * (d >> 3) : nullptr;
    uint8_t* rowp = codes + row_out * ((long long)d * BITS / 8);
    uint16_t* srow = scale + row_out * (d / G);
    uint16_t* zrow = zero + row_out * (d / G);

    for (int p0 = 0; p0 < ppr; p0 += blockDim.x) {
        const int pi = p0 + (int)threadIdx.x;
        const bool live = pi < ppr;
        const int pc = live ? pi : ppr - 1;
        uint4 raw0, raw1;
        if constexpr (DELTA && BITS != 3) {
            // the new rows are read once: non-temporal loads keep them from displacing the accumulator rows in the
            // last-level cache (measured on [8][4096][4096]: 2- and 4-bit deltas 69 -> 72 % of HBM peak; the 3-bit
            // kernel, whose stores are 12-byte pairs, loses 2 % with them and keeps plain loads)
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            const u32x4* xv = reinterpret_cast<const u32x4*>(xr);
            const u32x4 n0 = __builtin_nontemporal_load(&xv[2 * pc]), n1 = __builtin_nontemporal_load(&xv[2 * pc + 1]);
            raw0 = make_uint4(n0.x, n0.y, n0.z, n0.w); raw1 = make_uint4(n1.x, n1.y, n1.z, n1.w);
        } else {
            raw0 = xr[2 * pc]; raw1 = xr[2 * pc + 1];
        }
        float v[16];
        unpack8(raw0, v);
        unpack8(raw1, v + 8);
        if constexpr (DELTA) {
            const uint4 a0 = ar[2 * pc], a1 = ar[2 * pc + 1];
            float av[16];
            unpack8(a0, av);
            unpack8(a1, av + 8);
#pragma unroll
            for (int k = 0; k < 16; ++k) v[k] -= av[k];
        }
        float mn = v[0], mx = v[0];
#pragma unroll
        for (int k = 1; k < 16; k += 2) {                 // v_min3_f32 / v_max3_f32
            const float lo = k + 1 < 16 ? v[k + 1] : v[k];
            mn = fminf(fminf(mn, v[k]), lo);
            mx = fmaxf(fmaxf(mx, v[k]), lo);
        }
        group_minmax<LANES>(mn, mx);

        uint32_t zb = f32_to_bf16_rne(mn);
        zb = (zb & 0x7FFFu) ? zb : 0u;                    // -0 -> +0
        const float range = mx - mn;
        const float step = range / QMAX;                  // IEEE divide
        const uint32_t sb = f32_to_bf16_rne(step);
        const float zf = bf16_bits_to_f32(zb);
        const float sf = bf16_bits_to_f32(sb);
        const GroupRecip r = make_recip(sf);

        uint32_t q[16];                                   // 0x4B000000 + code
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const float n = v[k] - zf;
            const float y = __builtin_fmaf(n, r.rh, n * r.rl);
            q[k] = __float_as_uint(__builtin_amdgcn_fmed3f(y + ROUND_MAGIC, ROUND_MAGIC, ROUND_MAGIC + QMAX));
        }
        if (live && (pi % LANES) == 0) {
            srow[pi / LANES] = (uint16_t)sb;
            zrow[pi / LANES] = (uint16_t)zb;
        }

        pack_store16<BITS>(q, rowp, pi, live);
    }
}

template <int BITS, int G, bool DELTA>
static hipError_t launch(const uint16_t* x, const uint16_t* acc, const xq_cache_t* c, int T,
                         const BatchI32& start, hipStream_t s)
{
    const int ppr = c->fmt.d / 16;
    const int block = ppr >= 256 ? 256 : (ppr + 63) / 64 * 64;
    quantize_append_kernel<BITS, G, DELTA><<<dim3((unsigned)T, (unsigned)c->B), dim3(block), 0, s>>>(
        reinterpret_cast<const uint4*>(x), reinterpret_cast<const uint4*>(acc), c->codes, c->scale,
        c->zero, T, c->cap, c->fmt.d, start);
    return hipGetLastError();
}

template <bool DELTA>
static hipError_t dispatch(const uint16_t* x, const uint16_t* acc, const xq_cache_t* c, int T,
                           const BatchI32& start, hipStream_t s)
{
    const int key = c->fmt.bits * 1000 + c->fmt.group;
    switch (key) {
        case 2064: return launch<2, 64, DELTA>(x, acc, c, T, start, s);
        case 2128: return launch<2, 128, DELTA>(x, acc, c, T, start, s);
        case 3064: return launch<3, 64, DELTA>(x, acc, c, T, start, s);
        case 3128: return launch<3, 128, DELTA>(x, acc, c, T, start, s);
        case 4064: return launch<4, 64, DELTA>(x, acc, c, T, start, s);
        case 4128: return launch<4, 128, DELTA>(x, acc, c, T, start, s);
        case 8064: return launch<8, 64, DELTA>(x, acc, c, T, start, s);
        case 8128: return launch<8, 128, DELTA>(x, acc, c, T, start, s);
    }
    return hipErrorInvalidValue;
}

hipError_t run_quantize_append(const xq_cache_t* c, const uint16_t* x, const uint16_t* acc, int T,
                               const BatchI32& start, hipStream_t s)
{
    return acc ? dispatch<true>(x, acc, c, T, start, s) : dispatch<false>(x, nullptr, c, T, start, s);
}

// ---- per-channel groups (Sec. 3.3.1): a group is one channel over a block of G consecutive tokens.
// One pass over HBM: a wave owns 64 rows x 128 channels of a block, a lane two adjacent channels,
// and keeps its column of the piece -- one dword per row -- in 64 registers.  Min/max need no
// exchange inside the wave; for G = 128 the two waves that share a piece swap theirs through LDS
// (one barrier).  Zero-point, scale and the codes are then computed per lane; only the packing
// needs 16 consecutive channels per lane, so the codes go through the wave's own 8 KiB of LDS as
// bytes ([row][128]) and come back as 8 rows x 8 units of 16 codes per instruction, packed and
// stored exactly as in the per-token kernel.
template <int BITS, int G>
__global__ __launch_bounds__(256) void quantize_blocks_per_channel_kernel(
    const uint32_t* __restrict__ x, uint8_t* __restrict__ codes, uint16_t* __restrict__ scale,
    uint16_t* __restrict__ zero, int nblk, int cap, int d, BatchI32 block0)
{
    constexpr int RW = 64;                       // rows per wave
    constexpr int RSPLIT = G / RW;               // waves per piece (1 or 2)
    static_assert(G == 64 || G == 128, "block size");
    __shared__ __attribute__((aligned(16))) uint8_t stage[4][RW * 128];
    __shared__ float xch[4][4][64];
    constexpr float QMAX = (float)((1 << BITS) - 1);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int piece = blockIdx.x * (4 / RSPLIT) + wave / RSPLIT;              // 128-channel piece of the row
    const int rhalf = wave % RSPLIT;                                          // which 64 rows of the block
    const bool active = piece * 128 < d;
    const int pc = active ? piece : 0;
    const int blk = blockIdx.y, b = blockIdx.z;
    const long long row_in0 = ((long long)b * nblk + blk) * G + rhalf * RW;
    const long long blk_out = (long long)b * (cap / G) + block0.v[b] + blk;
    const long long row_out0 = (long long)b * cap + (long long)(block0.v[b] + blk) * G + rhalf * RW;
    const long long row_bytes = (long long)d * BITS / 8;
    const int dw_per_row = d >> 1;

    uint32_t raw[RW];
    const uint32_t* src = x + row_in0 * dw_per_row + pc * 64 + lane;
#pragma unroll
    for (int r = 0; r < RW; ++r) raw[r] = src[(long long)r * dw_per_row];
    float mn0 = bf16_lo_to_f32(raw[0]), mx0 = mn0, mn1 = bf16_hi_to_f32(raw[0]), mx1 = mn1;
#pragma unroll
    for (int r = 1; r < RW; r += 2) {
        const float a0 = bf16_lo_to_f32(raw[r]), a1 = bf16_hi_to_f32(raw[r]);
        const float b0 = r + 1 < RW ? bf16_lo_to_f32(raw[r + 1]) : a0, b1 = r + 1 < RW ? bf16_hi_to_f32(raw[r + 1]) : a1;
        mn0 = fminf(fminf(mn0, a0), b0); mx0 = fmaxf(fmaxf(mx0, a0), b0);
        mn1 = fminf(fminf(mn1, a1), b1); mx1 = fmaxf(fmaxf(mx1, a1), b1);
    }
    if constexpr (RSPLIT == 2) {
        xch[wave][0][lane] = mn0; xch[wave][1][lane] = mx0; xch[wave][2][lane] = mn1; xch[wave][3][lane] = mx1;
        __syncthreads();
        mn0 = fminf(mn0, xch[wave ^ 1][0][lane]); mx0 = fmaxf(mx0, xch[wave ^ 1][1][lane]);
        mn1 = fminf(mn1, xch[wave ^ 1][2][lane]); mx1 = fmaxf(mx1, xch[wave ^ 1][3][lane]);
    }
    if (!active) return;                                                      // (after the only barrier)
    uint32_t z0 = f32_to_bf16_rne(mn0), z1 = f32_to_bf16_rne(mn1);
    z0 = (z0 & 0x7FFFu) ? z0 : 0u;                                            // -0 -> +0
    z1 = (z1 & 0x7FFFu) ? z1 : 0u;
    const uint32_t s0 = f32_to_bf16_rne((mx0 - mn0) / QMAX), s1 = f32_to_bf16_rne((mx1 - mn1) / QMAX);   // IEEE divides
    const float zf0 = bf16_bits_to_f32(z0), zf1 = bf16_bits_to_f32(z1);
    const GroupRecip r0 = make_recip(bf16_bits_to_f32(s0)), r1 = make_recip(bf16_bits_to_f32(s1));
    if (rhalf == 0) {
        reinterpret_cast<uint32_t*>(scale + blk_out * d)[piece * 64 + lane] = s0 | (s1 << 16);
        reinterpret_cast<uint32_t*>(zero + blk_out * d)[piece * 64 + lane] = z0 | (z1 << 16);
    }

    uint8_t* mine = stage[wave];
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        const float n0 = bf16_lo_to_f32(raw[r]) - zf0, n1 = bf16_hi_to_f32(raw[r]) - zf1;
        const float y0 = __builtin_fmaf(n0, r0.rh, n0 * r0.rl), y1 = __builtin_fmaf(n1, r1.rh, n1 * r1.rl);
        const uint32_t q0 = __float_as_uint(__builtin_amdgcn_fmed3f(y0 + ROUND_MAGIC, ROUND_MAGIC, ROUND_MAGIC + QMAX));
        const uint32_t q1 = __float_as_uint(__builtin_amdgcn_fmed3f(y1 + ROUND_MAGIC, ROUND_MAGIC, ROUND_MAGIC + QMAX));
        reinterpret_cast<uint16_t*>(mine + r * 128)[lane] = (uint16_t)((q0 & 0xFFu) | (q1 << 8));
    }
    __builtin_amdgcn_wave_barrier();
    // packing: lane = (row r8 + lane / 8, unit lane % 8 of 16 codes)
    const int unit = lane & 7, sub = lane >> 3;
#pragma unroll 2
    for (int r8 = 0; r8 < RW; r8 += 8) {
        const int r = r8 + sub;
        const uint4 cw = *reinterpret_cast<const uint4*>(mine + r * 128 + unit * 16);
        const uint32_t w4[4] = {cw.x, cw.y, cw.z, cw.w};
        uint32_t q[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) q[k] = ((w4[k >> 2] >> (8 * (k & 3))) & 0xFFu) | ROUND_MAGIC_BITS;
        pack_store16<BITS>(q, codes + (row_out0 + r) * row_bytes, piece * 8 + unit, true);
    }
}

template <int BITS>
static hipError_t launch_blocks_pc(const xq_cache_t* c, const uint16_t* x, int nblk, const BatchI32& block0, hipStream_t s)
{
    const int d = c->fmt.d;
    const int ppw = c->fmt.group == 64 ? 4 : 2;                       // 128-channel pieces per workgroup
    const dim3 grid((unsigned)((d / 128 + ppw - 1) / ppw), (unsigned)nblk, (unsigned)c->B);
    const uint32_t* xp = reinterpret_cast<const uint32_t*>(x);
    if (c->fmt.group == 64)
        quantize_blocks_per_channel_kernel<BITS, 64><<<grid, dim3(256), 0, s>>>(xp, c->codes, c->scale, c->zero, nblk, c->cap, d, block0);
    else
        quantize_blocks_per_channel_kernel<BITS, 128><<<grid, dim3(256), 0, s>>>(xp, c->codes, c->scale, c->zero, nblk, c->cap, d, block0);
    return hipGetLastError();
}

hipError_t run_quantize_blocks_per_channel(const xq_cache_t* c, const uint16_t* x, int nblk, const BatchI32& block0,
                                           hipStream_t s)
{
    switch (c->fmt.bits) {
        case 2: return launch_blocks_pc<2>(c, x, nblk, block0, s);
        case 3: return launch_blocks_pc<3>(c, x, nblk, block0, s);
        case 4: return launch_blocks_pc<4>(c, x, nblk, block0, s);
        case 8: return launch_blocks_pc<8>(c, x, nblk, block0, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace xq
