// Quantise-and-append kernels: X cache rows (Sec. 3.1) and cross-layer delta rows
// (Sec. 3.2) of arxiv 2508.10395.  HBM-streaming: every lane loads 8 consecutive
// bf16 channels (16 B), a group of G channels lives in G/8 adjacent lanes of one
// 16-lane DPP row, min/max are reduced with DPP, the b-bit codes are packed in
// registers and written as the row's little-endian bit string.
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
    mn = fminf(mn, dpp_f32<DPP_ROW_HALF_MIRROR>(mn));
    mx = fmaxf(mx, dpp_f32<DPP_ROW_HALF_MIRROR>(mx));
    if constexpr (LANES == 16) {
        mn = fminf(mn, dpp_f32<DPP_ROW_MIRROR>(mn));
        mx = fmaxf(mx, dpp_f32<DPP_ROW_MIRROR>(mx));
    }
}

// One thread = one chunk of 8 channels.  x is [B][T][d]; in DELTA mode the value
// quantised is x - acc[b][start[b]+t] (fp32).  Output row = b*cap + start[b] + t.
template <int BITS, int G, bool DELTA>
__global__ __launch_bounds__(256) void quantize_append_kernel(
    const uint4* __restrict__ x, const uint4* __restrict__ acc, uint8_t* __restrict__ codes,
    uint16_t* __restrict__ scale, uint16_t* __restrict__ zero, int T, int cap, int d, BatchI32 start,
    long long nchunks)
{
    constexpr int LANES = G / 8;
    constexpr float QMAX = (float)((1 << BITS) - 1);
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const bool live = i < nchunks;
    const long long ic = live ? i : nchunks - 1;      // keep whole DPP rows active
    const int cpr = d >> 3;                           // chunks per row
    const long long row_in = ic / cpr;
    const int cw = (int)(ic - row_in * cpr);
    const int b = (int)(row_in / T);
    const int t = (int)(row_in - (long long)b * T);
    const long long row_out = (long long)b * cap + start.v[b] + t;

    uint4 raw = x[ic];
    float v[8];
    v[0] = bf16_lo_to_f32(raw.x); v[1] = bf16_hi_to_f32(raw.x);
    v[2] = bf16_lo_to_f32(raw.y); v[3] = bf16_hi_to_f32(raw.y);
    v[4] = bf16_lo_to_f32(raw.z); v[5] = bf16_hi_to_f32(raw.z);
    v[6] = bf16_lo_to_f32(raw.w); v[7] = bf16_hi_to_f32(raw.w);
    if constexpr (DELTA) {
        uint4 a = acc[row_out * cpr + cw];
        v[0] -= bf16_lo_to_f32(a.x); v[1] -= bf16_hi_to_f32(a.x);
        v[2] -= bf16_lo_to_f32(a.y); v[3] -= bf16_hi_to_f32(a.y);
        v[4] -= bf16_lo_to_f32(a.z); v[5] -= bf16_hi_to_f32(a.z);
        v[6] -= bf16_lo_to_f32(a.w); v[7] -= bf16_hi_to_f32(a.w);
    }
    float mn = fminf(fminf(fminf(v[0], v[1]), fminf(v[2], v[3])), fminf(fminf(v[4], v[5]), fminf(v[6], v[7])));
    float mx = fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
    group_minmax<LANES>(mn, mx);

    uint32_t zb = f32_to_bf16_rne(mn);
    zb = (zb & 0x7FFFu) ? zb : 0u;                    // -0 -> +0
    const float range = mx - mn;
    const float step = range / QMAX;                  // IEEE divide
    const uint32_t sb = f32_to_bf16_rne(step);
    const float zf = bf16_bits_to_f32(zb);
    const float sf = bf16_bits_to_f32(sb);
    const GroupRecip r = make_recip(sf);

    uint32_t q[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        float n = v[k] - zf;
        float y = __builtin_fmaf(n, r.rh, n * r.rl);
        y = fminf(fmaxf(y, 0.0f), QMAX);
        q[k] = (uint32_t)__builtin_rintf(y);
    }

    const int g = cw / LANES;
    const int ngroups = d / G;
    if (live && (cw % LANES) == 0) {
        scale[row_out * ngroups + g] = (uint16_t)sb;
        zero[row_out * ngroups + g] = (uint16_t)zb;
    }

    uint8_t* rowp = codes + row_out * ((long long)d * BITS / 8);
    if constexpr (BITS == 8) {
        uint2 w;
        w.x = q[0] | (q[1] << 8) | (q[2] << 16) | (q[3] << 24);
        w.y = q[4] | (q[5] << 8) | (q[6] << 16) | (q[7] << 24);
        if (live) reinterpret_cast<uint2*>(rowp)[cw] = w;
    } else if constexpr (BITS == 4) {
        uint32_t w = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) w |= q[k] << (4 * k);
        if (live) reinterpret_cast<uint32_t*>(rowp)[cw] = w;
    } else if constexpr (BITS == 2) {
        uint32_t w = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) w |= q[k] << (2 * k);
        if (live) reinterpret_cast<uint16_t*>(rowp)[cw] = (uint16_t)w;
    } else {   // 3 bits: 24 bits per lane, four lanes make three dwords
        uint32_t w = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) w |= q[k] << (3 * k);
        const uint32_t nxt = dpp_u32<DPP_QUAD_NEXT>(w);
        const int j = threadIdx.x & 3;
        const uint32_t out = (w >> (8 * j)) | (nxt << (24 - 8 * j));
        if (live && j < 3) reinterpret_cast<uint32_t*>(rowp)[(cw >> 2) * 3 + j] = out;
    }
}

template <int BITS, int G, bool DELTA>
static hipError_t launch(const uint16_t* x, const uint16_t* acc, const xq_cache_t* c, int T,
                         const BatchI32& start, hipStream_t s)
{
    const long long nchunks = (long long)c->B * T * (c->fmt.d / 8);
    const int block = 256;
    const long long grid = (nchunks + block - 1) / block;
    quantize_append_kernel<BITS, G, DELTA><<<dim3((unsigned)grid), dim3(block), 0, s>>>(
        reinterpret_cast<const uint4*>(x), reinterpret_cast<const uint4*>(acc), c->codes, c->scale,
        c->zero, T, c->cap, c->fmt.d, start, nchunks);
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

}  // namespace xq
