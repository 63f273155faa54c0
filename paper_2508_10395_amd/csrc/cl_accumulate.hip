// Cross-layer accumulate (Sec. 3.2 of arxiv 2508.10395): X^_i = X^_{i-1} + dX^_i on
// a bf16 accumulator, streamed once over [B][len][d].  HBM-bound: per element it
// reads b/8 bytes of codes plus 2 bytes of accumulator (unless initialising) and
// writes 2 bytes.
#include "common.hpp"

namespace xq {

template <int BITS>
__device__ __forceinline__ uint32_t load_codes8(const uint8_t* __restrict__ rowp, int cw, int row_dwords)
{
    if constexpr (BITS == 4) {
        return reinterpret_cast<const uint32_t*>(rowp)[cw];
    } else if constexpr (BITS == 2) {
        return reinterpret_cast<const uint16_t*>(rowp)[cw];
    } else {   // 3 bits: 24 bits starting at byte 3*cw, taken from two aligned dwords
        const int byte = 3 * cw;
        const int dw = byte >> 2;
        const uint32_t lo = reinterpret_cast<const uint32_t*>(rowp)[dw];
        const uint32_t hi = reinterpret_cast<const uint32_t*>(rowp)[min(dw + 1, row_dwords - 1)];
        const uint64_t both = ((uint64_t)hi << 32) | lo;
        return (uint32_t)(both >> ((byte & 3) * 8)) & 0xFFFFFFu;
    }
}

// grid.y = sequence; one thread = 8 channels of one token row.
template <int BITS, int G, bool INIT>
__global__ __launch_bounds__(256) void cl_accumulate_kernel(
    uint4* __restrict__ acc, const uint8_t* __restrict__ codes, const uint16_t* __restrict__ scale,
    const uint16_t* __restrict__ zero, int cap, int d, BatchI32 len)
{
    const int b = blockIdx.y;
    const int cpr = d >> 3;
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (long long)len.v[b] * cpr) return;
    const int t = (int)(i / cpr);
    const int cw = (int)(i - (long long)t * cpr);
    const long long row = (long long)b * cap + t;
    const int ngroups = d / G;
    const int g = (cw * 8) / G;
    const float sf = bf16_bits_to_f32(scale[row * ngroups + g]);
    const float zf = bf16_bits_to_f32(zero[row * ngroups + g]);
    const long long row_bytes = (long long)d * BITS / 8;
    const uint8_t* rowp = codes + row * row_bytes;

    uint32_t q[8];
    if constexpr (BITS == 8) {
        const uint2 w = reinterpret_cast<const uint2*>(rowp)[cw];
#pragma unroll
        for (int k = 0; k < 4; ++k) { q[k] = (w.x >> (8 * k)) & 0xFFu; q[4 + k] = (w.y >> (8 * k)) & 0xFFu; }
    } else {
        const uint32_t w = load_codes8<BITS>(rowp, cw, (int)(row_bytes >> 2));
#pragma unroll
        for (int k = 0; k < 8; ++k) q[k] = (w >> (BITS * k)) & ((1u << BITS) - 1u);
    }

    float prev[8];
    if constexpr (INIT) {
#pragma unroll
        for (int k = 0; k < 8; ++k) prev[k] = 0.0f;
    } else {
        const uint4 a = acc[row * cpr + cw];
        prev[0] = bf16_lo_to_f32(a.x); prev[1] = bf16_hi_to_f32(a.x);
        prev[2] = bf16_lo_to_f32(a.y); prev[3] = bf16_hi_to_f32(a.y);
        prev[4] = bf16_lo_to_f32(a.z); prev[5] = bf16_hi_to_f32(a.z);
        prev[6] = bf16_lo_to_f32(a.w); prev[7] = bf16_hi_to_f32(a.w);
    }
    uint32_t o[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const float dq = __builtin_fmaf((float)q[k], sf, zf);
        const float sum = prev[k] + dq;
        o[k] = f32_to_bf16_rne(sum);
    }
    uint4 w;
    w.x = o[0] | (o[1] << 16); w.y = o[2] | (o[3] << 16);
    w.z = o[4] | (o[5] << 16); w.w = o[6] | (o[7] << 16);
    acc[row * cpr + cw] = w;
}

template <int BITS, int G>
static hipError_t launch(uint16_t* acc, const xq_cache_t* c, const BatchI32& len, int max_len, bool init,
                         hipStream_t s)
{
    if (max_len == 0) return hipSuccess;
    const int block = 256;
    const long long per_seq = (long long)max_len * (c->fmt.d / 8);
    dim3 grid((unsigned)((per_seq + block - 1) / block), (unsigned)c->B);
    if (init)
        cl_accumulate_kernel<BITS, G, true><<<grid, dim3(block), 0, s>>>(
            reinterpret_cast<uint4*>(acc), c->codes, c->scale, c->zero, c->cap, c->fmt.d, len);
    else
        cl_accumulate_kernel<BITS, G, false><<<grid, dim3(block), 0, s>>>(
            reinterpret_cast<uint4*>(acc), c->codes, c->scale, c->zero, c->cap, c->fmt.d, len);
    return hipGetLastError();
}

hipError_t run_cl_accumulate(uint16_t* acc, const xq_cache_t* c, const BatchI32& len, int max_len,
                             bool init, hipStream_t s)
{
    const int key = c->fmt.bits * 1000 + c->fmt.group;
    switch (key) {
        case 2064: return launch<2, 64>(acc, c, len, max_len, init, s);
        case 2128: return launch<2, 128>(acc, c, len, max_len, init, s);
        case 3064: return launch<3, 64>(acc, c, len, max_len, init, s);
        case 3128: return launch<3, 128>(acc, c, len, max_len, init, s);
        case 4064: return launch<4, 64>(acc, c, len, max_len, init, s);
        case 4128: return launch<4, 128>(acc, c, len, max_len, init, s);
        case 8064: return launch<8, 64>(acc, c, len, max_len, init, s);
        case 8128: return launch<8, 128>(acc, c, len, max_len, init, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace xq
