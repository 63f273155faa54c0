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
        const uint4 raw0 = xr[2 * pc], raw1 = xr[2 * pc + 1];
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
// Workgroup = (1024-channel slab, block, sequence), 4 waves; a lane owns 16 consecutive channels,
// the waves split the block's rows.  Pass 1 reduces min/max per channel (rows in registers, waves
// through LDS); pass 2 re-reads the rows (1 MB per block: L2) and encodes them with the per-channel
// scale and zero-point, packing each row exactly as the per-token kernel does.
template <int BITS>
__global__ __launch_bounds__(256) void quantize_blocks_per_channel_kernel(
    const uint4* __restrict__ x, uint8_t* __restrict__ codes, uint16_t* __restrict__ scale,
    uint16_t* __restrict__ zero, int nblk, int G, int cap, int d, BatchI32 block0)
{
    __shared__ float smn[4][64][17], smx[4][64][17];
    constexpr float QMAX = (float)((1 << BITS) - 1);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int blk = blockIdx.y, b = blockIdx.z;
    const int ppr = d >> 4;
    const int pi = blockIdx.x * 64 + lane;
    const bool live = pi < ppr;
    const int pc = live ? pi : ppr - 1;
    const long long row_in0 = ((long long)b * nblk + blk) * G;              // first input row of the block
    const long long blk_out = (long long)b * (cap / G) + block0.v[b] + blk;    // block index in the cache
    const long long row_out0 = (long long)b * cap + (long long)(block0.v[b] + blk) * G;
    const long long row_bytes = (long long)d * BITS / 8;

    float mn[16], mx[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) { mn[k] = INFINITY; mx[k] = -INFINITY; }
    // (G / 4 rows per wave, G a multiple of 16: four rows' loads are in flight at a time)
    for (int r0 = wave; r0 < G; r0 += 16) {
        uint4 raw[4][2];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint4* xr = x + (row_in0 + r0 + 4 * u) * (d >> 3);
            raw[u][0] = xr[2 * pc];
            raw[u][1] = xr[2 * pc + 1];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float v[16];
            unpack8(raw[u][0], v);
            unpack8(raw[u][1], v + 8);
#pragma unroll
            for (int k = 0; k < 16; ++k) { mn[k] = fminf(mn[k], v[k]); mx[k] = fmaxf(mx[k], v[k]); }
        }
    }
#pragma unroll
    for (int k = 0; k < 16; ++k) { smn[wave][lane][k] = mn[k]; smx[wave][lane][k] = mx[k]; }
    __syncthreads();
    float zf[16], rh[16], rl[16];
    uint32_t zb[16], sb[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        float a = smn[0][lane][k], c = smx[0][lane][k];
#pragma unroll
        for (int w = 1; w < 4; ++w) { a = fminf(a, smn[w][lane][k]); c = fmaxf(c, smx[w][lane][k]); }
        uint32_t z = f32_to_bf16_rne(a);
        z = (z & 0x7FFFu) ? z : 0u;                       // -0 -> +0
        const float step = (c - a) / QMAX;                // IEEE divide
        const uint32_t sbits = f32_to_bf16_rne(step);
        const GroupRecip rr = make_recip(bf16_bits_to_f32(sbits));
        zb[k] = z; sb[k] = sbits;
        zf[k] = bf16_bits_to_f32(z); rh[k] = rr.rh; rl[k] = rr.rl;
    }
    if (wave == 0 && live) {
        uint4 s0, s1, z0, z1;
        s0.x = sb[0] | (sb[1] << 16); s0.y = sb[2] | (sb[3] << 16); s0.z = sb[4] | (sb[5] << 16); s0.w = sb[6] | (sb[7] << 16);
        s1.x = sb[8] | (sb[9] << 16); s1.y = sb[10] | (sb[11] << 16); s1.z = sb[12] | (sb[13] << 16); s1.w = sb[14] | (sb[15] << 16);
        z0.x = zb[0] | (zb[1] << 16); z0.y = zb[2] | (zb[3] << 16); z0.z = zb[4] | (zb[5] << 16); z0.w = zb[6] | (zb[7] << 16);
        z1.x = zb[8] | (zb[9] << 16); z1.y = zb[10] | (zb[11] << 16); z1.z = zb[12] | (zb[13] << 16); z1.w = zb[14] | (zb[15] << 16);
        uint4* sp = reinterpret_cast<uint4*>(scale + blk_out * d) + 2 * pi;
        uint4* zp = reinterpret_cast<uint4*>(zero + blk_out * d) + 2 * pi;
        sp[0] = s0; sp[1] = s1; zp[0] = z0; zp[1] = z1;
    }
    for (int r0 = wave; r0 < G; r0 += 16) {
        uint4 raw[4][2];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint4* xr = x + (row_in0 + r0 + 4 * u) * (d >> 3);
            raw[u][0] = xr[2 * pc];
            raw[u][1] = xr[2 * pc + 1];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float v[16];
            unpack8(raw[u][0], v);
            unpack8(raw[u][1], v + 8);
            uint32_t q[16];
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const float n = v[k] - zf[k];
                const float y = __builtin_fmaf(n, rh[k], n * rl[k]);
                q[k] = __float_as_uint(__builtin_amdgcn_fmed3f(y + ROUND_MAGIC, ROUND_MAGIC, ROUND_MAGIC + QMAX));
            }
            pack_store16<BITS>(q, codes + (row_out0 + r0 + 4 * u) * row_bytes, pi, live);
        }
    }
}

hipError_t run_quantize_blocks_per_channel(const xq_cache_t* c, const uint16_t* x, int nblk, const BatchI32& block0,
                                           hipStream_t s)
{
    const int d = c->fmt.d, G = c->fmt.group;
    const dim3 grid((unsigned)((d / 16 + 63) / 64), (unsigned)nblk, (unsigned)c->B);
    const uint4* xp = reinterpret_cast<const uint4*>(x);
    switch (c->fmt.bits) {
        case 2: quantize_blocks_per_channel_kernel<2><<<grid, dim3(256), 0, s>>>(xp, c->codes, c->scale, c->zero, nblk, G, c->cap, d, block0); break;
        case 3: quantize_blocks_per_channel_kernel<3><<<grid, dim3(256), 0, s>>>(xp, c->codes, c->scale, c->zero, nblk, G, c->cap, d, block0); break;
        case 4: quantize_blocks_per_channel_kernel<4><<<grid, dim3(256), 0, s>>>(xp, c->codes, c->scale, c->zero, nblk, G, c->cap, d, block0); break;
        case 8: quantize_blocks_per_channel_kernel<8><<<grid, dim3(256), 0, s>>>(xp, c->codes, c->scale, c->zero, nblk, G, c->cap, d, block0); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace xq
