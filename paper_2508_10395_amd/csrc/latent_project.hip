// Down-projection of layer inputs into the latent spaces of the K and V projections
// (Sec. 3.3.1 of arxiv 2508.10395: for GQA models the cache holds X Uk and X Uv, where
// Wk = Uk Sk Bk^T and Wv = Uv Sv Bv^T are SVDs computed offline).
//
// out[m][n] = bf16( sum_c x[m][c] * Ut[n][c] ),  fp32 accumulation, one RNE rounding.
// Ut is U transposed (one row per latent channel), so both MFMA operands read 8 consecutive
// contraction indices with one 16-byte load.  A workgroup computes a 32 x 32 output tile; its 8
// waves each take one eighth of the contraction and the partial tiles are summed through LDS in
// fixed order.  At decode (M = batch) the kernel is bound by reading Ut once.
//
// Cross-layer variant (Sec. 3.3.2): the projected rows are deltas x - a against the accumulator
// rows X^_{i-1}.  The fp32 difference of two bf16 values does not fit one bf16, so it enters the
// MFMA as a bf16 hi part plus a bf16 lo part (two MFMAs per k-step; what is left is below 2^-16 of
// the delta).
#include "common.hpp"

namespace xq {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

// 8 bf16 (one 16-byte load) -> fp32
__device__ __forceinline__ void widen8(const uint4& v, float (&f)[8])
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = bf16_lo_to_f32(w[i]);
        f[2 * i + 1] = bf16_hi_to_f32(w[i]);
    }
}

// DELTA: row m = b * T + t of x is paired with accumulator row start[b] + t of sequence b
template <bool DELTA>
__global__ __launch_bounds__(512) void latent_project_kernel(const uint16_t* __restrict__ x,
                                                             const uint16_t* __restrict__ ut,
                                                             uint16_t* __restrict__ out, int M, int d, int n_lat,
                                                             const uint16_t* __restrict__ a, int T, int cap,
                                                             const BatchI32 start)
{
    __shared__ float red[8][32][33];
    const int nb = blockIdx.x, mb = blockIdx.y;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 31, kb = lane >> 5;
    const int row = min(mb * 32 + r, M - 1);            // rows past M repeat the last one, never stored
    const int col = nb * 32 + r;
    const int kchunk = d >> 3;                           // contraction share of one wave (multiple of 16)
    const uint16_t* ap = x + (long long)row * d + wave * kchunk + kb * 8;
    const uint16_t* bp = ut + (long long)col * d + wave * kchunk + kb * 8;
    const uint16_t* sp = nullptr;
    if constexpr (DELTA) {
        const int b = row / T, t = row - b * T;
        sp = a + ((long long)b * cap + start.v[b] + t) * d + wave * kchunk + kb * 8;
    }
    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
#pragma unroll 4
    for (int k = 0; k < kchunk; k += 16) {
        const uint4 xa = *reinterpret_cast<const uint4*>(ap + k);
        const uint4 b = *reinterpret_cast<const uint4*>(bp + k);
        if constexpr (DELTA) {
            const uint4 sa = *reinterpret_cast<const uint4*>(sp + k);
            float xf[8], sf[8];
            widen8(xa, xf);
            widen8(sa, sf);
            uint32_t hi[4], lo[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float d0 = xf[2 * i] - sf[2 * i], d1 = xf[2 * i + 1] - sf[2 * i + 1];
                hi[i] = pack_bf16x2_rne(d0, d1);
                lo[i] = pack_bf16x2_rne(d0 - bf16_lo_to_f32(hi[i]), d1 - bf16_hi_to_f32(hi[i]));
            }
            const uint4 vh = make_uint4(hi[0], hi[1], hi[2], hi[3]), vl = make_uint4(lo[0], lo[1], lo[2], lo[3]);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vl), __builtin_bit_cast(bf16x8, b),
                                                          acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vh), __builtin_bit_cast(bf16x8, b),
                                                          acc, 0, 0, 0);
        } else {
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, xa), __builtin_bit_cast(bf16x8, b),
                                                          acc, 0, 0, 0);
        }
    }
    // accumulator element i of lane (r, kb) is D[m][n] with n = r, m = 8 (i/4) + 4 kb + i%4
#pragma unroll
    for (int i = 0; i < 16; ++i) red[wave][8 * (i >> 2) + 4 * kb + (i & 3)][r] = acc[i];
    __syncthreads();
    for (int idx = threadIdx.x; idx < 1024; idx += 512) {
        const int m = idx >> 5, n = idx & 31;
        float s = red[0][m][n];
#pragma unroll
        for (int w = 1; w < 8; ++w) s += red[w][m][n];
        if (mb * 32 + m < M) out[(long long)(mb * 32 + m) * n_lat + nb * 32 + n] = (uint16_t)f32_to_bf16_rne(s);
    }
}

hipError_t run_latent_project(const uint16_t* x, const uint16_t* ut, int M, int d, int n_lat, uint16_t* out,
                              hipStream_t s)
{
    latent_project_kernel<false><<<dim3(n_lat / 32, (M + 31) / 32), dim3(512), 0, s>>>(x, ut, out, M, d, n_lat, nullptr,
                                                                                        1, 0, BatchI32{});
    return hipGetLastError();
}

// x [B][T][d] against accumulator rows start[b] + t of acc [B][cap][d]
hipError_t run_latent_delta_project(const uint16_t* x, const uint16_t* acc, const uint16_t* ut, int B, int T, int cap,
                                    const BatchI32& start, int d, int n_lat, uint16_t* out, hipStream_t s)
{
    const int M = B * T;
    latent_project_kernel<true><<<dim3(n_lat / 32, (M + 31) / 32), dim3(512), 0, s>>>(x, ut, out, M, d, n_lat, acc, T,
                                                                                       cap, start);
    return hipGetLastError();
}

}  // namespace xq
