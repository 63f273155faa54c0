// Shared pieces of the rematerialisation kernels: kernel parameters, LDS layout of the contraction loop,
// LDS-DMA helpers, half-wave reductions, the tile a workgroup owns.
#pragma once
#include <type_traits>

#include "common.hpp"
#include "remat_layout.hpp"
#include "unpack.hpp"

namespace xq {

constexpr int floordiv_c(int a, int b) { return a >= 0 ? a / b : -((-a + b - 1) / b); }

// f(integral_constant<int, I>) for I = BEGIN .. END-1, unrolled by construction: the contraction
// loop indexes register arrays with these values, so they must be compile-time constants
template <int BEGIN, int END, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (BEGIN < END) {
        f(std::integral_constant<int, BEGIN>{});
        static_for<BEGIN + 1, END>(f);
    }
}
#define XQ_INLINE_LAMBDA __attribute__((always_inline))

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

// LDS: two weight slabs, then (coded sources) the tile's packed codes of one slab -- two such
// images when they fit, so that no barrier is needed between taking one slab's codes out and the
// arrival of the next-but-one's -- then three 1 KiB buffers of effective scales (2 groups x 256
// tokens each; the third is used once, for the slab the lagging column blocks start in)
constexpr int LDS_CODES_OFF = 2 * SLAB_BYTES;
constexpr int LDS_SCALES_BYTES = 1024;
constexpr int LDS_MAX = 160 * 1024;
constexpr int code_image_bytes(int bits) { return TILE_TOKENS * 16 * bits; }
constexpr int n_code_images(int bits)
{
    return LDS_CODES_OFF + 2 * code_image_bytes(bits) + 3 * LDS_SCALES_BYTES <= LDS_MAX ? 2 : 1;
}
constexpr int lds_scales_off(int bits) { return LDS_CODES_OFF + n_code_images(bits) * code_image_bytes(bits); }
constexpr int lds_coded_total(int bits) { return lds_scales_off(bits) + 3 * LDS_SCALES_BYTES; }

struct RematParams {
    const uint16_t* q;       // [B][Hq][128]; prefill: [B][Tq][Hq][128]
    int Tq;                  // prefill: new tokens (queries) per sequence
    const uint8_t* codes;    // coded source (its scales reach the kernel through eT)
    const uint16_t* zero;
    const uint16_t* acc;     // dense source
    const uint8_t* wprep;
    const int32_t* head_shift;   // coded source: per-head exponent shift of the fp16 stream (taken out with the final scale)
    const uint16_t* eT;      // coded source: effective scales [B][tiles][ng (+1 pad)][256], bf16
    float* part_o;           // [B][Hq][chunks_per_seq][128]  (prefill: [B][Tq][Hq][tiles_per_seq][128])
    float* part_ml;          // [B][Hq][chunks_per_seq][2]
    int B, cap, d, Hq, Hkv;
    int row_d, ng_row;       // coded source: channels / groups per cache row (>= d, ng when a sub-range is contracted)
    int meta_shift;          // coded source: group g of the walk takes scale and zero-point g >> meta_shift of the row
                             //   (1 when an 8-bit cache with groups of 128 is walked as 4-bit groups of 128 nibbles)
    int grid_heads;          // heads (or head pairs) the grid is laid over
    int tile_major;          // workgroup order inside an XCD: 0 = a head's tiles one after the other, 1 = a tile's heads side by side
    float* scores;           // latent passes: q.K * scale * log2(e), [B][Hq][score_stride]
    int score_stride;        // floats per (sequence, query head) in scores
    BatchI32 tok0;           // pass 1: token index of this launch's row 0 in scores (0 unless a launch continues another)
    int tiles_per_seq, chunks_per_seq;
    int n_main_slabs, n_corr_ksteps, ng, ng_pad;
    long long head_bytes;
    float scale_log2e;       // softmax_scale * log2(e)
    BatchI32 len;
    uint16_t* acc_out;       // up-projection mode: accumulator [B][cap][d_out] bf16, updated in place
    int d_out;
    BatchI32 chunk0;         // first partial-chunk index of each sequence in this launch (0 unless a launch continues another)
    // per-channel source (groups along the token axis): factor images, per-block scale and z W rows
    const float* pc_fscale;  // [B][pc_blocks_cap]: 2^(E_blk + bits - 1)
    const float* pc_zw;      // [B][pc_blocks_cap][grid_heads][256] fp32: zero-points of the block times the head's 256 columns
                             //   (4-bit codes: plus 8 times the scales of the block times those columns)
    float store_scale;       // dense store mode: kv_out = (store_add ? kv_out : 0) + store_scale * row
    int store_add;
    uint16_t* rows_out;      // dense bf16 store mode: [rows][grid_heads * 256] bf16 (one sequence)
    // dense bf16 store mode, optional second source: out = (x - acc2) W.  The walk covers 2 w_slabs slabs: the
    // first w_slabs take the rows of `acc` (= x, M rows), the others the matching rows of acc2 with flipped
    // signs against the same weights (the stream is walked twice).  Row m = b * Tq + t of x matches row
    // b * cap2 + tok0[b] + t of acc2.  acc2 == nullptr: one source, w_slabs == n_main_slabs.
    const uint16_t* acc2;
    int w_slabs, cap2;
    float* kv_out;           // dense store mode: [B][pc_blocks_cap][grid_heads][256] fp32 rematerialised rows
    int pc_block, pc_blocks_cap;   // tokens per block (64 or 128), blocks per sequence in the arrays above
    const float* rope;       // optional [n_pos][64][2] cos, sin: rotate the keys (half-split pairs)
    BatchI32 pos0;           // with rope: position of cache row 0 of each sequence
};

// LDS-DMA: every active lane copies 16 bytes from saddr + voff to LDS at lds_dst + 16 * lane.
// Issued through inline asm so that the compiler's wait-count insertion does not serialise
// later LDS reads of other buffers against it; completion is awaited explicitly
// (s_waitcnt vmcnt(0) + workgroup barrier) before the data is read.  The asm overwrites M0 (the
// LDS destination of the DMA) and says so in its clobber list, so the compiler keeps nothing live in it.
__device__ __forceinline__ void dma_b128(const void* saddr, uint32_t voff, uint32_t lds_dst)
{
    const uint64_t a = reinterpret_cast<uint64_t>(saddr);      // wave-uniform by construction
    const uint32_t a_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32));   // (the builtin
    const uint32_t a_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)a);           //  returns int)
    const uint64_t ua = ((uint64_t)a_hi << 32) | (uint64_t)a_lo;
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(ua), "s"(lds_dst) : "memory", "m0");
}

// one 64 KiB weight slab: 8 DMA instructions per wave (src / lds_dst already offset by the wave's 1 KiB)
__device__ __forceinline__ void issue_slab(const uint8_t* src, uint32_t lds_dst, uint32_t voff)
{
#pragma unroll
    for (int c = 0; c < 8; ++c) dma_b128(src + c * 8192, voff, lds_dst + c * 8192);
}

// the first n_chunks 8 KiB chunks of a slab only (a correction slab's k-steps past the last one hold nothing)
__device__ __forceinline__ void issue_slab_chunks(const uint8_t* src, uint32_t lds_dst, uint32_t voff, int n_chunks)
{
#pragma unroll
    for (int c = 0; c < 8; ++c)
        if (c < n_chunks) dma_b128(src + c * 8192, voff, lds_dst + c * 8192);
}

__device__ __forceinline__ f16x8 as_frag(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    uint4 v; v.x = a; v.y = b; v.z = c; v.w = d;
    return __builtin_bit_cast(f16x8, v);
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
// sum over each 32-lane half, valid in lanes 16-31 of the half only: the last step adds lane 15 of
// the lower 16-lane row into the upper row with a DPP row broadcast instead of a cross-row permute
__device__ __forceinline__ float wave32_sum_upper(float v)
{
    v += dpp_f32<DPP_QUAD_XOR1>(v);
    v += dpp_f32<DPP_QUAD_XOR2>(v);
    v += dpp_f32<DPP_ROW_HALF_MIRROR>(v);
    v += dpp_f32<DPP_ROW_MIRROR>(v);
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x142 /* row_bcast:15 */, 0xA, 0xF, false));
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

// One k-step of one unit for one token block, dispatching on the (compile-time after
// unrolling) k-step index inside the unit.
template <int BITS>
__device__ __forceinline__ void unpack_kstep(const uint32_t* unit, int j, uint32_t* out)
{
    switch (j & 3) {
        case 0: UnpackKStep<BITS, 0>::run(unit, out); break;
        case 1: UnpackKStep<BITS, 1>::run(unit, out); break;
        case 2: UnpackKStep<BITS, 2>::run(unit, out); break;
        default: UnpackKStep<BITS, 3>::run(unit, out); break;
    }
}

// which tile this workgroup owns, and this lane's place in it
struct TileCtx {
    int hk, b, tile, len, half, tl, lane, wave;
    int tok;       // this lane's token (tile * 256 + wave * 32 + lane % 32), may lie past len
};

__device__ __forceinline__ bool locate_tile(const RematParams& p, TileCtx& c)
{
    const int tid = threadIdx.x;
    c.lane = tid & 63;
    c.wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    c.half = c.lane >> 5;
    c.tl = c.lane & 31;
    // workgroup -> (KV head, sequence, tile); heads are dealt so that the workgroups
    // resident on one XCD (blockIdx % 8) stream the same head's slabs through its L2
    const int NT = p.B * p.tiles_per_seq;
    int tile_lin;
    if ((p.grid_heads & 7) == 0) {
        const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
        if (p.tile_major) {
            // the heads of an XCD take the same tile side by side: what they share is then the tile's token rows
            const int hpx = p.grid_heads >> 3;
            c.hk = xcd + 8 * (j % hpx);
            tile_lin = j / hpx;
        } else {
            c.hk = xcd + 8 * (j / NT);
            tile_lin = j % NT;
        }
    } else {
        c.hk = blockIdx.x / NT;
        tile_lin = blockIdx.x % NT;
    }
    // (runtime divisions are done on the vector ALU: bring the wave-uniform results back to scalar
    // registers, or every address derived from them would live in vector registers)
    c.hk = __builtin_amdgcn_readfirstlane(c.hk);
    c.b = __builtin_amdgcn_readfirstlane(tile_lin / p.tiles_per_seq);
    c.tile = __builtin_amdgcn_readfirstlane(tile_lin % p.tiles_per_seq);
    c.len = p.len.v[c.b];
    c.tok = c.tile * TILE_TOKENS + c.wave * CHUNK_TOKENS + c.tl;
    return c.tile * TILE_TOKENS < c.len;
}

constexpr int MODE_ATTENTION = 0, MODE_SCORES = 1, MODE_WEIGHTED_SUM = 2, MODE_ACCUMULATE = 3, MODE_PREFILL = 4,
              MODE_ATTENTION_PC = 5, MODE_SCORES_PC = 6;

// packed fp16 multiply of two operand dwords (v_pk_mul_f16; fp16 subnormals are honoured)
typedef _Float16 xq_f16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_mul_f16(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(xq_f16x2, a) * __builtin_bit_cast(xq_f16x2, b));
}
__device__ __forceinline__ uint32_t pk_add_f16(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(xq_f16x2, a) + __builtin_bit_cast(xq_f16x2, b));
}

}  // namespace xq
