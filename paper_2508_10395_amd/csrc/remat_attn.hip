// Fused dequantise -> rematerialise K,V -> flash-decode attention (Sec. 3.1 and the
// cost model of Sec. 3.4 in arxiv 2508.10395), plus the split-context combine.
//
// One workgroup (8 waves) owns a tile of 256 cached tokens of one (sequence, KV
// head).  Wave w handles tokens [64 (w%4), +64) of the tile and the K columns
// (w < 4) or the V columns (w >= 4) of [Wk_h | Wv_h]: a 128 x 64 fp32 accumulator
// block = 128 VGPRs, computed as D[n][t] = sum_c W[c][n] * x^[t][c] with
// v_mfma_f32_32x32x16_bf16, weights as the A operand (streamed HBM -> LDS as
// prepared 64 KiB slabs, double buffered) and tokens along the lanes of the B
// operand, so that everything per token (its scales, its score, its softmax weight)
// is a per-lane scalar.
//
// The cached codes are not dequantised to bf16 (that rounding alone would exceed
// the 2e-3 budget): each lane reads its token's packed codes straight from HBM,
// drops them into bf16 mantissas (1 + code*2^(o-7), exact) and the MFMA accumulates
// per quantisation group  P_g = sum_k (1 + c_k 2^(o_k-7)) W'_k.  With e_g = 2^b *
// scale_g the rematerialised value is
//     K[n][t] = sum_g e_g P_g[n]  +  sum_g ( zero_g S_g[n] - e_g S'_g[n] ),
// The first sum is carried in one accumulator by rescaling it with e_{g-1}/e_g at
// each group boundary (Horner form, one v_mul per register per group, relative
// error ~2^-23 per group); the second is a rank-(5 d/G) product done by a few extra
// MFMA k-steps whose token-side operands are the stored zero-points and scales
// (exact in bf16) and whose weight-side operands are 2- and 3-way bf16 splits of
// the column sums.  A zero stored scale uses e_g = 1 (its codes are all zero, so
// only the column-sum term matters and it cancels exactly as for any other e_g).
//
// After the contraction the K waves form the scores q.K[t] for each query head of
// the KV group, hand them to the V waves through LDS, and each V wave emits one
// online-softmax partial (m, l, o[128]) per query head for its 64 tokens.  A second
// small kernel merges the partials of a sequence in fixed order.
#include "common.hpp"
#include "remat_layout.hpp"
#include "unpack.hpp"

namespace xq {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int MAX_GQ = 16;   // query heads per KV head the epilogue's LDS scratch is sized for

struct RematParams {
    const uint16_t* q;       // [B][Hq][128]
    const uint8_t* codes;    // coded source
    const uint16_t* scale;
    const uint16_t* zero;
    const uint16_t* acc;     // dense source
    const uint8_t* wprep;
    float* part_o;           // [B][Hq][chunks_per_seq][128]
    float* part_ml;          // [B][Hq][chunks_per_seq][2]
    int B, cap, d, Hq, Hkv;
    int tiles_per_seq, chunks_per_seq;
    int n_main_slabs, n_corr_ksteps, ng, ng_pad;
    long long head_bytes;
    float scale_log2e;       // softmax_scale * log2(e)
    BatchI32 len;
};

// LDS-DMA of 16 bytes per lane: the wave's 1 KiB lands at lds_off + 16*lane.  Issued
// through inline asm so that the compiler's wait-count insertion does not serialise
// later LDS reads of the *other* buffer against it; completion is awaited explicitly
// (s_waitcnt vmcnt(0) + workgroup barrier) before the buffer is read.  M0 is not
// otherwise used by this kernel.
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_off)
{
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_off) : "memory");
}

__device__ __forceinline__ void issue_slab(const uint8_t* src, uint32_t lds_base, int wave, int lane)
{
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const int chunk = wave + 8 * c;
        dma16(src + chunk * 1024 + lane * 16, lds_base + chunk * 1024);
    }
}

template <int NDW>
__device__ __forceinline__ void load_dwords(const uint8_t* p, uint32_t* dst)
{
    if constexpr (NDW % 4 == 0 && true) {
#pragma unroll
        for (int i = 0; i < NDW / 4; ++i) {
            const uint4 v = reinterpret_cast<const uint4*>(p)[i];
            dst[4 * i] = v.x; dst[4 * i + 1] = v.y; dst[4 * i + 2] = v.z; dst[4 * i + 3] = v.w;
        }
    } else if constexpr (NDW % 2 == 0) {
#pragma unroll
        for (int i = 0; i < NDW / 2; ++i) {
            const uint2 v = reinterpret_cast<const uint2*>(p)[i];
            dst[2 * i] = v.x; dst[2 * i + 1] = v.y;
        }
    } else {
#pragma unroll
        for (int i = 0; i < NDW; ++i) dst[i] = reinterpret_cast<const uint32_t*>(p)[i];
    }
}

__device__ __forceinline__ float eff_scale(uint32_t sbits, int bits)
{
    // e = 2^bits * scale, or 1 for a zero scale
    return sbits ? __uint_as_float((sbits << 16) + ((uint32_t)bits << 23)) : 1.0f;
}

__device__ __forceinline__ bf16x8 as_frag(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    uint4 v; v.x = a; v.y = b; v.z = c; v.w = d;
    return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ float wave32_max(float v)   // all-reduce over each 32-lane half
{
    v = fmaxf(v, dpp_f32<DPP_QUAD_XOR1>(v));
    v = fmaxf(v, dpp_f32<DPP_QUAD_XOR2>(v));
    v = fmaxf(v, dpp_f32<DPP_ROW_HALF_MIRROR>(v));
    v = fmaxf(v, dpp_f32<DPP_ROW_MIRROR>(v));
    v = fmaxf(v, __shfl_xor(v, 16));
    return v;
}
__device__ __forceinline__ float wave32_sum(float v)
{
    v += dpp_f32<DPP_QUAD_XOR1>(v);
    v += dpp_f32<DPP_QUAD_XOR2>(v);
    v += dpp_f32<DPP_ROW_HALF_MIRROR>(v);
    v += dpp_f32<DPP_ROW_MIRROR>(v);
    v += __shfl_xor(v, 16);
    return v;
}

template <int BITS, int G>   // BITS in {2,3,4}: coded source; 16: dense bf16 accumulator source
__global__ __launch_bounds__(512) void remat_attn_kernel(const RematParams p)
{
    constexpr bool DENSE = BITS == 16;
    constexpr int KSG = DENSE ? 8 : G / 16;               // k-steps per quantisation group
    constexpr int GPS = 8 / KSG;                          // groups per slab
    constexpr int NDW_G = DENSE ? 0 : (G / 2) * BITS / 32;  // code dwords per lane per group
    constexpr int NDW = DENSE ? 1 : GPS * NDW_G;
    constexpr int GROUP_BYTES = DENSE ? 0 : G * BITS / 8;

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int part = wave >> 2;          // 0: K columns, 1: V columns
    const int tq = wave & 3;             // which 64 tokens of the tile
    const int half = lane >> 5, tl = lane & 31;

    // workgroup -> (KV head, sequence, tile); heads are dealt so that the workgroups
    // resident on one XCD (blockIdx % 8) stream the same head's slabs through its L2
    const int NT = p.B * p.tiles_per_seq;
    int hk, tile_lin;
    if ((p.Hkv & 7) == 0) {
        const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
        hk = xcd + 8 * (j / NT);
        tile_lin = j % NT;
    } else {
        hk = blockIdx.x / NT;
        tile_lin = blockIdx.x % NT;
    }
    const int b = tile_lin / p.tiles_per_seq;
    const int tile = tile_lin % p.tiles_per_seq;
    const int len = p.len.v[b];
    if (tile * TILE_TOKENS >= len) return;

    int tok[2];
    uint32_t rowi[2];                    // row inside the sequence (clamped: padding rows re-read the last one)
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        tok[tb] = tile * TILE_TOKENS + tq * CHUNK_TOKENS + tb * 32 + tl;
        rowi[tb] = (uint32_t)min(tok[tb], len - 1);
    }

    const uint8_t* wsrc = p.wprep + (long long)hk * p.head_bytes;
    const int n_corr_slabs = (p.n_corr_ksteps + SLAB_KSTEPS - 1) / SLAB_KSTEPS;
    const int n_slabs = p.n_main_slabs + n_corr_slabs;

    f32x16 acc[2][4];
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[tb][nb][i] = 0.0f;

    // ---- per-lane token-side sources: wave-uniform sequence base + 32-bit lane offset
    const long long seq_row0 = (long long)b * p.cap;
    const uint8_t* cbase = DENSE ? reinterpret_cast<const uint8_t*>(p.acc) + seq_row0 * p.d * 2
                                 : p.codes + seq_row0 * ((long long)p.d * BITS / 8);
    const uint16_t* sbase = DENSE ? nullptr : p.scale + seq_row0 * p.ng;
    const uint16_t* zbase = DENSE ? nullptr : p.zero + seq_row0 * p.ng;
    uint32_t coff[2], moff[2];
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        if constexpr (DENSE) coff[tb] = rowi[tb] * (uint32_t)(p.d * 2) + half * 128;
        else coff[tb] = rowi[tb] * (uint32_t)(p.d * BITS / 8) + half * (GROUP_BYTES / 2);
        moff[tb] = rowi[tb] * (uint32_t)p.ng;
    }

    uint32_t cur[2][NDW], nxt[2][NDW];
    uint32_t sc_cur[2][GPS], sc_nxt[2][GPS];
    uint4 bd[2][8];                       // dense: one slab of operand fragments per token block
    float e_prev[2] = {1.0f, 1.0f};

    const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) uint8_t*)lds;

    // Workgroups that run side by side on one XCD stream the same head.  Each starts its
    // contraction at a different slab (the sum over groups is order-free), so that at any
    // moment they pull different addresses and the requests spread over all L2 channels.
    const int rot = (int)((blockIdx.x >> 3) % (unsigned)p.n_main_slabs);
    auto main_slab_id = [&](int it) { const int s = it + rot; return s >= p.n_main_slabs ? s - p.n_main_slabs : s; };

    // prologue: first slab
    issue_slab(wsrc + (long long)rot * SLAB_BYTES, lds0, wave, lane);
    if constexpr (DENSE) {
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) bd[tb][ks] = reinterpret_cast<const uint4*>(cbase + coff[tb] + rot * 256)[ks];
    } else {
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int gi = 0; gi < GPS; ++gi) {
                load_dwords<NDW_G>(cbase + coff[tb] + (rot * GPS + gi) * GROUP_BYTES, &nxt[tb][gi * NDW_G]);
                sc_nxt[tb][gi] = sbase[moff[tb] + rot * GPS + gi];
            }
    }

    // ---- main slabs: the d x 256 contraction
    for (int it = 0; it < p.n_main_slabs; ++it) {
        // this slab (and this lane's token-side data for it) has landed; everyone is done with the one before
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        const bool more_main = it + 1 < p.n_main_slabs;
        const int s_next = more_main ? main_slab_id(it + 1) : p.n_main_slabs;   // then the correction slabs
        if (it + 1 < n_slabs)
            issue_slab(wsrc + (long long)s_next * SLAB_BYTES, lds0 + (uint32_t)(((it + 1) & 1) * SLAB_BYTES), wave, lane);
        const uint8_t* slab = lds + (it & 1) * SLAB_BYTES + (part * 4 * 64 + lane) * 16;

        if constexpr (!DENSE) {
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
#pragma unroll
                for (int i = 0; i < NDW; ++i) cur[tb][i] = nxt[tb][i];
#pragma unroll
                for (int gi = 0; gi < GPS; ++gi) sc_cur[tb][gi] = sc_nxt[tb][gi];
            }
            if (more_main) {
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                    for (int gi = 0; gi < GPS; ++gi) {
                        load_dwords<NDW_G>(cbase + coff[tb] + (s_next * GPS + gi) * GROUP_BYTES, &nxt[tb][gi * NDW_G]);
                        sc_nxt[tb][gi] = sbase[moff[tb] + s_next * GPS + gi];
                    }
            }
        }

        uint32_t bu[2][16];
#pragma unroll
        for (int ks = 0; ks < SLAB_KSTEPS; ++ks) {
            __builtin_amdgcn_sched_barrier(0);   // keep each k-step's loads and unpack local
            bf16x8 bfrag[2];
            if constexpr (DENSE) {
#pragma unroll
                for (int tb = 0; tb < 2; ++tb) {
                    bfrag[tb] = __builtin_bit_cast(bf16x8, bd[tb][ks]);
                    if (more_main)   // refill this ring slot for the next slab
                        bd[tb][ks] = reinterpret_cast<const uint4*>(cbase + coff[tb] + s_next * 256)[ks];
                }
            } else {
                const int gi = ks / KSG, ksg = ks % KSG;
                if (ksg == 0) {
#pragma unroll
                    for (int tb = 0; tb < 2; ++tb) {
                        const float e = eff_scale(sc_cur[tb][gi], BITS);
                        const float r = e_prev[tb] * __builtin_amdgcn_rcpf(e);
                        e_prev[tb] = e;
#pragma unroll
                        for (int nb = 0; nb < 4; ++nb) acc[tb][nb] *= r;
                    }
                }
                if ((ksg & 3) == 0) {
#pragma unroll
                    for (int tb = 0; tb < 2; ++tb)
                        UnpackUnit<BITS>::run(&cur[tb][gi * NDW_G + (ksg >> 2) * BITS], bu[tb]);
                }
#pragma unroll
                for (int tb = 0; tb < 2; ++tb) {
                    const int o = (ksg & 3) * 4;
                    bfrag[tb] = as_frag(bu[tb][o], bu[tb][o + 1], bu[tb][o + 2], bu[tb][o + 3]);
                }
            }
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) {
                const bf16x8 a = __builtin_bit_cast(
                    bf16x8, *reinterpret_cast<const uint4*>(slab + (ks * 8 + nb) * 1024));
                acc[0][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bfrag[0], acc[0][nb], 0, 0, 0);
                acc[1][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bfrag[1], acc[1][nb], 0, 0, 0);
            }
        }
    }

    // ---- correction slabs: token-side operands are the stored zero-points / minus the scales
    if constexpr (!DENSE) {
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) acc[tb][nb] *= e_prev[tb];

        for (int s = p.n_main_slabs; s < n_slabs; ++s) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (s + 1 < n_slabs)
                issue_slab(wsrc + (long long)(s + 1) * SLAB_BYTES, lds0 + (uint32_t)(((s + 1) & 1) * SLAB_BYTES), wave, lane);
            const uint8_t* slab = lds + (s & 1) * SLAB_BYTES + (part * 4 * 64 + lane) * 16;
            const int kk0 = (s - p.n_main_slabs) * SLAB_KSTEPS;
            const int nks = min(SLAB_KSTEPS, p.n_corr_ksteps - kk0);
#pragma unroll 1
            for (int ks = 0; ks < nks; ++ks) {
                const int kappa0 = (kk0 + ks) * 16 + half * 8;
                const int term = kappa0 / p.ng_pad, g0 = kappa0 % p.ng_pad;
                const bool term_ok = term < N_CORR_TERMS;
                const uint16_t* mbase = term < 2 ? zbase : sbase;
                bf16x8 bfrag[2];
#pragma unroll
                for (int tb = 0; tb < 2; ++tb) {
                    uint32_t h[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int g = g0 + i;
                        uint32_t v = mbase[moff[tb] + min(g, p.ng - 1)];
                        if (term >= 2) v = (v ? v + ((uint32_t)BITS << 7) : 0x3F80u) | 0x8000u;
                        h[i] = (term_ok && g < p.ng) ? v : 0u;
                    }
                    bfrag[tb] = as_frag(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16),
                                        h[6] | (h[7] << 16));
                }
#pragma unroll
                for (int nb = 0; nb < 4; ++nb) {
                    const bf16x8 a = __builtin_bit_cast(
                        bf16x8, *reinterpret_cast<const uint4*>(slab + (ks * 8 + nb) * 1024));
                    acc[0][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bfrag[0], acc[0][nb], 0, 0, 0);
                    acc[1][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bfrag[1], acc[1][nb], 0, 0, 0);
                }
            }
        }
    }

    // ------------------------------------------------------------ attention epilogue
    // accumulator element i of column block nb <-> output column n = 32 nb + 8 (i/4) + 4 half + i%4
    __syncthreads();                                   // slabs are dead: LDS becomes score scratch
    float* sc_lds = reinterpret_cast<float*>(lds);     // [4 tq][gq][64]
    const int gq = p.Hq / p.Hkv;
    const int chunk = tile * 4 + tq;
    const bool chunk_live = tile * TILE_TOKENS + tq * CHUNK_TOKENS < len;

    if (part == 0) {
        for (int j = 0; j < gq; ++j) {
            const uint16_t* qv = p.q + ((long long)b * p.Hq + hk * gq + j) * 128;
            float dot[2] = {0.0f, 0.0f};
#pragma unroll
            for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const uint2 qq = *reinterpret_cast<const uint2*>(qv + nb * 32 + i4 * 8 + half * 4);
                    const float q0 = bf16_lo_to_f32(qq.x), q1 = bf16_hi_to_f32(qq.x);
                    const float q2 = bf16_lo_to_f32(qq.y), q3 = bf16_hi_to_f32(qq.y);
#pragma unroll
                    for (int tb = 0; tb < 2; ++tb) {
                        dot[tb] = __builtin_fmaf(q0, acc[tb][nb][i4 * 4 + 0], dot[tb]);
                        dot[tb] = __builtin_fmaf(q1, acc[tb][nb][i4 * 4 + 1], dot[tb]);
                        dot[tb] = __builtin_fmaf(q2, acc[tb][nb][i4 * 4 + 2], dot[tb]);
                        dot[tb] = __builtin_fmaf(q3, acc[tb][nb][i4 * 4 + 3], dot[tb]);
                    }
                }
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
                float sfull = dot[tb] + __shfl_xor(dot[tb], 32);
                sfull = tok[tb] < len ? sfull * p.scale_log2e : -INFINITY;
                if (half == 0) sc_lds[(tq * gq + j) * 64 + tb * 32 + tl] = sfull;
            }
        }
    }
    __syncthreads();
    if (part == 1 && chunk_live) {
        for (int j = 0; j < gq; ++j) {
            const int hq = hk * gq + j;
            float sv[2], pv[2];
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) sv[tb] = sc_lds[(tq * gq + j) * 64 + tb * 32 + tl];
            const float m = wave32_max(fmaxf(sv[0], sv[1]));
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) pv[tb] = __builtin_amdgcn_exp2f(sv[tb] - m);
            const float l = wave32_sum(pv[0] + pv[1]);
            const long long pidx = ((long long)b * p.Hq + hq) * p.chunks_per_seq + chunk;
            float* po = p.part_o + pidx * 128;
#pragma unroll
            for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    float o[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        // p = 0 rows (masked tokens) must not import garbage: rows are clamped, so finite
                        float v = pv[0] * acc[0][nb][i4 * 4 + k];
                        v = __builtin_fmaf(pv[1], acc[1][nb][i4 * 4 + k], v);
                        o[k] = wave32_sum(v);
                    }
                    if (tl == 0) {
                        float4 w; w.x = o[0]; w.y = o[1]; w.z = o[2]; w.w = o[3];
                        *reinterpret_cast<float4*>(po + nb * 32 + i4 * 8 + half * 4) = w;
                    }
                }
            if (lane == 0) {
                p.part_ml[pidx * 2] = m;
                p.part_ml[pidx * 2 + 1] = l;
            }
        }
    }
}

// ---- split-context combine: out[b][h][:] = sum_c w_c o_c / sum_c w_c l_c, w_c = 2^(m_c - M)
__global__ __launch_bounds__(128) void combine_kernel(const float* __restrict__ part_o,
                                                      const float* __restrict__ part_ml,
                                                      float* __restrict__ out, int Hq, int chunks_per_seq,
                                                      BatchI32 len)
{
    const int h = blockIdx.x, b = blockIdx.y, n = threadIdx.x;
    const int nchunks = (len.v[b] + CHUNK_TOKENS - 1) / CHUNK_TOKENS;
    const long long base = ((long long)b * Hq + h) * chunks_per_seq;
    float M = -INFINITY;
    for (int c = 0; c < nchunks; ++c) M = fmaxf(M, part_ml[(base + c) * 2]);
    float L = 0.0f, o = 0.0f;
    for (int c = 0; c < nchunks; ++c) {
        const float w = __builtin_amdgcn_exp2f(part_ml[(base + c) * 2] - M);
        L = __builtin_fmaf(w, part_ml[(base + c) * 2 + 1], L);
        o = __builtin_fmaf(w, part_o[(base + c) * 128 + n], o);
    }
    out[((long long)b * Hq + h) * 128 + n] = o / L;
}

template <int BITS, int G>
static hipError_t launch_remat(const RematParams& p, int grid, hipStream_t s)
{
    static bool attr_set = false;
    const int lds_bytes = 2 * SLAB_BYTES;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&remat_attn_kernel<BITS, G>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    remat_attn_kernel<BITS, G><<<dim3(grid), dim3(512), lds_bytes, s>>>(p);
    return hipGetLastError();
}

hipError_t run_remat_attn_decode(const xq_attn_t* a, const uint16_t* q, const xq_cache_t* xc,
                                 const uint16_t* acc, int B, int cap, int d, const void* wprep,
                                 const BatchI32& len, int max_len, float* out, void* ws, hipStream_t s)
{
    const int bits = xc ? xc->fmt.bits : 16;
    const int G = xc ? xc->fmt.group : 128;
    const WPrepLayout L = make_wprep_layout(d, G, bits, a->n_kv_heads);
    RematParams p{};
    p.q = q;
    p.codes = xc ? xc->codes : nullptr;
    p.scale = xc ? xc->scale : nullptr;
    p.zero = xc ? xc->zero : nullptr;
    p.acc = acc;
    p.wprep = static_cast<const uint8_t*>(wprep);
    p.B = B; p.cap = cap; p.d = d; p.Hq = a->n_q_heads; p.Hkv = a->n_kv_heads;
    p.tiles_per_seq = (max_len + TILE_TOKENS - 1) / TILE_TOKENS;
    p.chunks_per_seq = p.tiles_per_seq * (TILE_TOKENS / CHUNK_TOKENS);
    p.n_main_slabs = L.n_main_slabs; p.n_corr_ksteps = L.n_corr_ksteps; p.ng = L.ng; p.ng_pad = L.ng_pad;
    p.head_bytes = (long long)L.head_bytes;
    p.scale_log2e = a->softmax_scale * 1.44269504088896340736f;
    p.len = len;
    p.part_o = static_cast<float*>(ws);
    p.part_ml = p.part_o + (size_t)B * p.Hq * p.chunks_per_seq * 128;

    const int grid = p.Hkv * p.B * p.tiles_per_seq;
    hipError_t e = hipErrorInvalidValue;
    switch (bits * 1000 + (bits == 16 ? 0 : G)) {
        case 2064: e = launch_remat<2, 64>(p, grid, s); break;
        case 2128: e = launch_remat<2, 128>(p, grid, s); break;
        case 3064: e = launch_remat<3, 64>(p, grid, s); break;
        case 3128: e = launch_remat<3, 128>(p, grid, s); break;
        case 4064: e = launch_remat<4, 64>(p, grid, s); break;
        case 4128: e = launch_remat<4, 128>(p, grid, s); break;
        case 16000: e = launch_remat<16, 128>(p, grid, s); break;
    }
    if (e != hipSuccess) return e;
    combine_kernel<<<dim3(p.Hq, p.B), dim3(128), 0, s>>>(p.part_o, p.part_ml, out, p.Hq, p.chunks_per_seq, p.len);
    return hipGetLastError();
}

}  // namespace xq
