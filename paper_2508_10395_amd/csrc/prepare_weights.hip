// Offline weight preparation for the rematerialisation kernel (weights are static;
// run once per layer).  Re-lays [Wk_h | Wv_h] (Sec. 3.1 / the W_kv concatenation of
// Sec. 3.3.2 in arxiv 2508.10395) into the slab stream described in
// remat_layout.hpp and appends the per-group column sums the kernel needs to apply the
// zero-points.  For coded sources the stream holds fp16 (the codes are fp16 operands, see
// unpack.hpp): a bf16 weight times a power of two is exact in fp16 unless it falls below
// 2^-14 (then it is rounded to the fp16 subnormal grid) or above 65504.  Neither happens to a weight that
// matters: each head's stream is first normalised by a power of two, 2^shift[h], that puts the head's
// largest entry just below 2^15 (shift_kernel), so only entries 2^-29 below the largest reach the
// subnormal grid, with an error of at most 2^-40 of the largest.  The kernels undo the shift in their
// final scale.  Dense (bf16) streams need none: shift = 0.
#include "common.hpp"
#include "remat_layout.hpp"
#include "unpack.hpp"

namespace xq {

struct PrepArgs {
    const uint16_t* Wk;
    const uint16_t* Wv;
    uint8_t* out;
    float* colsum;   // [Hkv][ng][256]: per-group sums of the weight rows
    int32_t* shift;  // [Hkv]: exponent shift of the head's fp16 stream (0 for bf16 streams)
    int d, G, bits, Hkv, ncols;
    int head_stride; // columns between consecutive heads in Wk / Wv (128; 256 when a "head" is a pair of heads)
    int transposed;  // the matrices are given transposed ([column][d], as the projection matrices are): d = row length
    int nibbles;     // stream for an 8-bit cache read as 4-bit codes: channel c stands for nibble c & 1 of code c >> 1,
                     //   i.e. weight row c >> 1 times 16^(c & 1); d counts nibbles, the matrices have d / 2 rows
    int n_main_slabs, ng, ng_pad, n_corr_slabs;
    long long head_bytes;
    UnpackTable tab;
};

// element (channel c, column n of [Wk_h | Wv_h]) of the matrix the stream encodes
__device__ __forceinline__ float wval(const PrepArgs& a, int h, int c, int n)
{
    const uint16_t* W = n < 128 ? a.Wk : a.Wv;
    const long long col = h * a.head_stride + (n & 127);
    if (a.nibbles) {
        const int row = c >> 1, rows = a.d >> 1;
        const float w = bf16_bits_to_f32(a.transposed ? W[col * rows + row] : W[(long long)row * a.ncols + col]);
        return (c & 1) ? 16.0f * w : w;
    }
    return bf16_bits_to_f32(a.transposed ? W[col * a.d + c] : W[(long long)c * a.ncols + col]);
}

// shift[h] = 12 - ceil(log2(max |w|)) over the head's d x 256 entries: max |w| 2^shift <= 2^12, and with the
// largest per-slot factor of the unpack table (2^3) the stream's largest entry is at most 2^15.
__global__ __launch_bounds__(1024) void shift_kernel(PrepArgs a)
{
    __shared__ uint32_t red[1024];
    const int h = blockIdx.x, n = threadIdx.x & 255, part = threadIdx.x >> 8;     // column, quarter of the rows
    uint32_t mx = 0;                                      // |w| as fp32 bits: ordered as integers
    for (int c = part; c < a.d; c += 4) mx = max(mx, __float_as_uint(wval(a, h, c, n)) & 0x7FFFFFFFu);
    red[threadIdx.x] = mx;
    __syncthreads();
    for (int st = 512; st > 0; st >>= 1) {
        if ((int)threadIdx.x < st) red[threadIdx.x] = max(red[threadIdx.x], red[threadIdx.x + st]);
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        int sh = 0;
        if (red[0]) {
            const int e = (int)(red[0] >> 23) - 127;      // max = m 2^e, 1 <= m < 2 (subnormals: e = -127, m < 1)
            const int ceil_log2 = (red[0] & 0x7FFFFFu) ? e + 1 : e;
            sh = min(max(12 - ceil_log2, -60), 60);
        }
        a.shift[h] = sh;
    }
}

__global__ __launch_bounds__(256) void colsum_kernel(PrepArgs a)
{
    const int n = threadIdx.x;
    const int g = blockIdx.x, h = blockIdx.y;
    float s = 0.0f;
    // (nibble streams: the zero-point of a code multiplies its weight row once: the even channels)
    for (int k = 0; k < a.G; k += a.nibbles ? 2 : 1) s += wval(a, h, g * a.G + k, n);
    a.colsum[((long long)h * a.ng + g) * 256 + n] = s;
}

// one thread = one lane's 16 bytes of one fragment; grid (slab, head), block 512 x 8 k-steps... see launch
__global__ __launch_bounds__(256) void pack_main_kernel(PrepArgs a)
{
    const int s = blockIdx.x, h = blockIdx.y;
    const bool dense = a.bits == 16;
    const int ksg_n = a.G / 16;
    const int n_ksteps = a.n_main_slabs * SLAB_KSTEPS;
    const int head_shift = dense ? 0 : a.shift[h];
    for (int f = threadIdx.x; f < SLAB_KSTEPS * 8 * 64; f += blockDim.x) {
        const int lane = f & 63, nb = (f >> 6) & 7, ks = f >> 9;
        const int half = lane >> 5, n = nb * 32 + (lane & 31);
        // coded sources: position (slab s, tick ks, block nb) holds k-step 8 s + ks - (7 - nb), cyclically
        int kappa = s * SLAB_KSTEPS + ks - (COL_BLOCK_LAG_MAX - nb);
        if (kappa < 0) kappa += n_ksteps;
        const int cs_ = kappa / SLAB_KSTEPS, cks = kappa % SLAB_KSTEPS;
        uint32_t v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            int c, e = 0;
            if (dense) {
                c = s * 128 + ks * 16 + half * 8 + i;
            } else {
                const int gi = cks / ksg_n, ksg = cks % ksg_n;
                const int u = ksg >> 2, j = ksg & 3;
                const int p = a.tab.code_of_slot[j][i];
                c = cs_ * 128 + gi * a.G + half * (a.G / 2) + u * 32 + p;
                e = a.tab.wexp_of_code[p] + head_shift;
            }
            const float wv = ldexpf(wval(a, h, c, n), e);          // exact: power-of-two scaling
            if (dense) {
                v[i] = f32_to_bf16_rne(wv);
            } else {
                const _Float16 hv = (_Float16)fminf(fmaxf(wv, -65504.0f), 65504.0f);
                v[i] = (uint32_t)__builtin_bit_cast(uint16_t, hv);
            }
        }
        uint4 o;
        o.x = v[0] | (v[1] << 16); o.y = v[2] | (v[3] << 16);
        o.z = v[4] | (v[5] << 16); o.w = v[6] | (v[7] << 16);
        *reinterpret_cast<uint4*>(a.out + (long long)h * a.head_bytes + (long long)s * SLAB_BYTES + (long long)f * 16) = o;
    }
}

__device__ __forceinline__ uint32_t split_part(float x, int part)
{
    uint32_t hi = f32_to_bf16_rne(x);
    if (part == 0) return hi;
    float r1 = x - bf16_bits_to_f32(hi);
    uint32_t mid = f32_to_bf16_rne(r1);
    if (part == 1) return mid;
    float r2 = r1 - bf16_bits_to_f32(mid);
    return f32_to_bf16_rne(r2);
}

__global__ __launch_bounds__(256) void pack_corr_kernel(PrepArgs a)
{
    const int cs = blockIdx.x, h = blockIdx.y;
    for (int f = threadIdx.x; f < SLAB_KSTEPS * 8 * 64; f += blockDim.x) {
        const int lane = f & 63, nb = (f >> 6) & 7, ks = f >> 9;
        const int half = lane >> 5, n = nb * 32 + (lane & 31);
        uint32_t v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int kappa = (cs * SLAB_KSTEPS + ks) * 16 + half * 8 + i;
            const int term = kappa / a.ng_pad, g = kappa % a.ng_pad;
            uint32_t bits = 0;
            if (term < N_CORR_TERMS && g < a.ng) {
                const long long idx = ((long long)h * a.ng + g) * 256 + n;
                bits = split_part(a.colsum[idx], term);
            }
            v[i] = bits;
        }
        uint4 o;
        o.x = v[0] | (v[1] << 16); o.y = v[2] | (v[3] << 16);
        o.z = v[4] | (v[5] << 16); o.w = v[6] | (v[7] << 16);
        *reinterpret_cast<uint4*>(a.out + (long long)h * a.head_bytes +
                                  (long long)(a.n_main_slabs + cs) * SLAB_BYTES + (long long)f * 16) = o;
    }
}

// ---- the second stream: 16-column fragments for the v_mfma_f32_16x16x32 kernel (layout in remat_layout.hpp)
__global__ __launch_bounds__(256) void pack_main16_kernel(PrepArgs a, uint8_t* out16, long long head_bytes16)
{
    const int s = blockIdx.x, h = blockIdx.y;
    const int n_k32 = a.n_main_slabs * TILE16_TICKS;
    const bool dense = a.bits == 16;
    const int head_shift = dense ? 0 : a.shift[h];
    for (int f = threadIdx.x; f < TILE16_TICKS * 16 * 64; f += blockDim.x) {
        const int lane = f & 63, ct = (f >> 6) & 15, j = f >> 10;
        const int q = lane >> 4, n = ct * 16 + (lane & 15);
        int kappa = s * TILE16_TICKS + j - (dense ? 0 : tile16_lag(ct));
        if (kappa < 0) kappa += n_k32;
        const int cs_ = kappa / TILE16_TICKS, cj = kappa % TILE16_TICKS;
        uint32_t v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (dense) {
                v[i] = f32_to_bf16_rne(wval(a, h, cs_ * 128 + cj * 32 + q * 8 + i, n));              // (exact: the weights are bf16)
                continue;
            }
            // groups of 128: quarter q unpacks unit q, tick cj is its k-step; groups of 64: tick cj is unit cj, quarter
            // q its k-step (a tick then lies inside one group)
            const int p = a.G == 64 ? a.tab.code_of_slot[q][i] : a.tab.code_of_slot[cj][i];
            const int c = a.G == 64 ? cs_ * 128 + cj * 32 + p : cs_ * 128 + q * 32 + p;
            const float wv = ldexpf(wval(a, h, c, n), a.tab.wexp_of_code[p] + head_shift);          // exact: power-of-two scaling
            const _Float16 hv = (_Float16)fminf(fmaxf(wv, -65504.0f), 65504.0f);
            v[i] = (uint32_t)__builtin_bit_cast(uint16_t, hv);
        }
        uint4 o;
        o.x = v[0] | (v[1] << 16); o.y = v[2] | (v[3] << 16);
        o.z = v[4] | (v[5] << 16); o.w = v[6] | (v[7] << 16);
        *reinterpret_cast<uint4*>(out16 + (long long)h * head_bytes16 + (long long)s * SLAB_BYTES + (long long)f * 16) = o;
    }
}

__global__ __launch_bounds__(256) void pack_corr16_kernel(PrepArgs a, uint8_t* out16, long long head_bytes16)
{
    const int cs = blockIdx.x, h = blockIdx.y;
    for (int f = threadIdx.x; f < TILE16_TICKS * 16 * 64; f += blockDim.x) {
        const int lane = f & 63, ct = (f >> 6) & 15, j = f >> 10;
        const int q = lane >> 4, n = ct * 16 + (lane & 15);
        uint32_t v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int kappa = (cs * TILE16_TICKS + j) * 32 + q * 8 + i;
            const int term = kappa / a.ng_pad, g = kappa % a.ng_pad;
            uint32_t bits = 0;
            if (term < N_CORR_TERMS && g < a.ng) bits = split_part(a.colsum[((long long)h * a.ng + g) * 256 + n], term);
            v[i] = bits;
        }
        uint4 o;
        o.x = v[0] | (v[1] << 16); o.y = v[2] | (v[3] << 16);
        o.z = v[4] | (v[5] << 16); o.w = v[6] | (v[7] << 16);
        *reinterpret_cast<uint4*>(out16 + (long long)h * head_bytes16 +
                                  (long long)(a.n_main_slabs + cs) * SLAB_BYTES + (long long)f * 16) = o;
    }
}

bool unpack_table_for(int bits, UnpackTable* t)
{
    switch (bits) {
        case 2: *t = build_unpack_table<2>(); break;
        case 3: *t = build_unpack_table<3>(); break;
        case 4: *t = build_unpack_table<4>(); break;
        case 16: *t = UnpackTable{}; t->valid = 1; break;
        default: return false;
    }
    return t->valid != 0;
}

// Wk / Wv: [d][ncols] row-major; head h takes columns [h * head_stride, +128) of each
hipError_t run_prepare_weights(const WPrepLayout& L, const uint16_t* Wk, const uint16_t* Wv, int ncols,
                               int head_stride, void* out, hipStream_t s, bool transposed, bool nibbles)
{
    PrepArgs a{};
    a.nibbles = nibbles ? 1 : 0;
    a.head_stride = head_stride;
    a.transposed = transposed ? 1 : 0;
    a.Wk = Wk; a.Wv = Wv;
    a.out = static_cast<uint8_t*>(out);
    a.colsum = reinterpret_cast<float*>(a.out + L.stream_bytes);
    a.shift = reinterpret_cast<int32_t*>(a.out + L.stream_bytes + L.colsum_bytes);
    a.d = L.d; a.G = L.G; a.bits = L.bits; a.Hkv = L.Hkv; a.ncols = ncols;
    a.n_main_slabs = L.n_main_slabs; a.ng = L.ng; a.ng_pad = L.ng_pad; a.n_corr_slabs = L.n_corr_slabs;
    a.head_bytes = (long long)L.head_bytes;
    if (!unpack_table_for(L.bits, &a.tab)) return hipErrorInvalidValue;
    if (L.bits != 16) shift_kernel<<<dim3(L.Hkv), dim3(1024), 0, s>>>(a);
    pack_main_kernel<<<dim3(L.n_main_slabs, L.Hkv), dim3(256), 0, s>>>(a);
    if (L.bits != 16) {
        colsum_kernel<<<dim3(L.ng, L.Hkv), dim3(256), 0, s>>>(a);
        pack_corr_kernel<<<dim3(L.n_corr_slabs, L.Hkv), dim3(256), 0, s>>>(a);
    }
    if (L.t16_bytes) {
        uint8_t* out16 = a.out + L.t16_offset;
        pack_main16_kernel<<<dim3(L.n_main_slabs, L.Hkv), dim3(256), 0, s>>>(a, out16, (long long)L.t16_head_bytes);
        if (L.t16_n_corr_slabs)
            pack_corr16_kernel<<<dim3(L.t16_n_corr_slabs, L.Hkv), dim3(256), 0, s>>>(a, out16, (long long)L.t16_head_bytes);
    }
    return hipGetLastError();
}

}  // namespace xq
