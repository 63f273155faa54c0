// Fused dequantise -> rematerialise K,V -> flash-decode attention (Sec. 3.1 and the
// cost model of Sec. 3.4 in arxiv 2508.10395), plus the split-context combine.
//
// One workgroup (8 waves) owns a tile of 256 cached tokens of one (sequence, KV
// head).  Wave w handles tokens [32 w, 32 w + 32) of the tile and all 256 columns of
// [Wk_h | Wv_h]: eight 32 x 32 fp32 accumulator blocks = 128 VGPRs, computed as
// D[n][t] = sum_c W[c][n] * x^[t][c] with v_mfma_f32_32x32x16_f16 (coded sources) or
// _bf16 (the XQuant-CL accumulator), weights as the A operand (streamed HBM -> LDS
// as prepared 64 KiB slabs, double buffered) and tokens
// along the lanes of the B operand, so that everything per token (its codes, its
// scales, its score, its softmax weight) is a per-lane scalar and is unpacked once.
//
// The cached codes are not dequantised to bf16 (that rounding alone would exceed
// the 2e-3 budget): the code bits are masked into fp16 mantissas under a zero
// exponent, i.e. they enter the fp16 MFMA as the subnormals c_k 2^(o_k-24), exactly,
// at one v_and_b32 per pair of codes, and the MFMA accumulates per quantisation group
//     P_g = sum_k (c_k 2^(o_k-24)) W'_k,      W'_k = W_k 2^(10-o_k-b)  (fp16, exact).
// With e_g = 2^(b+14) * scale_g the rematerialised value is
//     K[n][t] = sum_g e_g P_g[n]  +  sum_g zero_g S_g[n],    S_g = sum of the group's weight rows.
// The first sum is carried in one accumulator by rescaling it with e_{g-1}/e_g at
// each group boundary (Horner form, one v_mul per register per group, relative
// error ~2^-23 per group); the second is a rank-(3 d/G) product done by a few extra
// bf16 MFMA k-steps whose token-side operands are the stored zero-points (exact in
// bf16) and whose weight-side operands are bf16 hi/mid/lo splits of the column sums.
// A zero stored scale uses e_g = 1 (its codes are all zero).
//
// Data movement of the coded kernel: everything the contraction loop consumes
// arrives by LDS-DMA (global_load_lds): the weight slab, the tile's packed codes of
// the next 128 channels (16-byte pieces, three adjacent lanes per 3-bit row) and the
// tile's effective scales (from a [tile][group][token] copy made by a small
// pre-pass, so that they are contiguous).  The loop therefore contains no
// compiler-visible global load, and one explicit s_waitcnt vmcnt(0) per slab.
//
// After the contraction each wave holds K (blocks 0-3) and V (blocks 4-7) of its 32
// tokens, forms the scores q.K[t] for each query head of the KV group, and emits one
// online-softmax partial (m, l, o[128]) per query head and 32-token chunk without
// leaving the wave.  A second small kernel merges the partials of a sequence in
// fixed order.
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
    const uint16_t* eT;      // coded source: effective scales [B][tiles][ng (+1 pad)][256], bf16
    float* part_o;           // [B][Hq][chunks_per_seq][128]  (prefill: [B][Tq][Hq][tiles_per_seq][128])
    float* part_ml;          // [B][Hq][chunks_per_seq][2]
    int B, cap, d, Hq, Hkv;
    int row_d, ng_row;       // coded source: channels / groups per cache row (>= d, ng when a sub-range is contracted)
    int grid_heads;          // heads (or head pairs) the grid is laid over
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
    float* kv_out;           // dense store mode: [B][pc_blocks_cap][grid_heads][256] fp32 rematerialised rows
    int pc_block, pc_blocks_cap;   // tokens per block (64 or 128), blocks per sequence in the arrays above
    const float* rope;       // optional [n_pos][64][2] cos, sin: rotate the keys (half-split pairs)
    BatchI32 pos0;           // with rope: position of cache row 0 of each sequence
};

// LDS-DMA: every active lane copies 16 bytes from saddr + voff to LDS at lds_dst + 16 * lane.
// Issued through inline asm so that the compiler's wait-count insertion does not serialise
// later LDS reads of other buffers against it; completion is awaited explicitly
// (s_waitcnt vmcnt(0) + workgroup barrier) before the data is read.  M0 is not otherwise
// used by these kernels.
__device__ __forceinline__ void dma_b128(const void* saddr, uint32_t voff, uint32_t lds_dst)
{
    const uint64_t a = reinterpret_cast<uint64_t>(saddr);      // wave-uniform by construction
    const uint32_t a_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32));   // (the builtin
    const uint32_t a_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)a);           //  returns int)
    const uint64_t ua = ((uint64_t)a_hi << 32) | (uint64_t)a_lo;
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(ua), "s"(lds_dst) : "memory");
}

// one 64 KiB weight slab: 8 DMA instructions per wave (src / lds_dst already offset by the wave's 1 KiB)
__device__ __forceinline__ void issue_slab(const uint8_t* src, uint32_t lds_dst, uint32_t voff)
{
#pragma unroll
    for (int c = 0; c < 8; ++c) dma_b128(src + c * 8192, voff, lds_dst + c * 8192);
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
        c.hk = xcd + 8 * (j / NT);
        tile_lin = j % NT;
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

// Rotary embedding of this lane's key: column n < 64 pairs with n + 64, i.e. accumulator element i
// of block nb with the same element of block nb + 2.  The lane's 4 consecutive columns
// 32 nb + 8 i4 + 4 half + [0, 4) need 8 consecutive floats of its position's row of the table.
__device__ __forceinline__ void rope_rotate(const RematParams& p, const TileCtx& c, f32x16 (&acc)[8])
{
    const float* tab = p.rope + (long long)(p.pos0.v[c.b] + min(c.tok, c.len - 1)) * 128;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            const float* cs = tab + 2 * (nb * 32 + i4 * 8 + c.half * 4);
            const float4 cs0 = *reinterpret_cast<const float4*>(cs);
            const float4 cs1 = *reinterpret_cast<const float4*>(cs + 4);
            const float co[4] = {cs0.x, cs0.z, cs1.x, cs1.z}, si[4] = {cs0.y, cs0.w, cs1.y, cs1.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float a = acc[nb][i4 * 4 + k], b = acc[nb + 2][i4 * 4 + k];
                acc[nb][i4 * 4 + k] = __builtin_fmaf(a, co[k], -b * si[k]);
                acc[nb + 2][i4 * 4 + k] = __builtin_fmaf(b, co[k], a * si[k]);
            }
        }
}

// ---- attention on the rematerialised chunk: each wave holds K (blocks 0-3) and V (blocks 4-7)
// of its 32 tokens.  Accumulator element i of column block nb <-> column 32 (nb%4) + 8 (i/4) +
// 4 half + i%4 of K or V, token = lane % 32.  No LDS and no barrier: scores, softmax weights and
// the weighted sum of V stay inside the wave; it emits one partial (m, l, o[128]) per query head.
__device__ __forceinline__ void attention_epilogue(const RematParams& p, const TileCtx& c, f32x16 (&acc)[8])
{
    if (c.tile * TILE_TOKENS + c.wave * CHUNK_TOKENS >= c.len) return;     // chunk entirely past len
    if (p.rope) rope_rotate(p, c, acc);
    const int gq = p.Hq / p.Hkv;
    const int chunk = p.chunk0.v[c.b] + c.tile * (TILE_TOKENS / CHUNK_TOKENS) + c.wave;
    for (int j = 0; j < gq; ++j) {
        const int hq = c.hk * gq + j;
        const uint16_t* qv = p.q + ((long long)c.b * p.Hq + hq) * 128;
        float dot = 0.0f;
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const uint2 qq = *reinterpret_cast<const uint2*>(qv + nb * 32 + i4 * 8 + c.half * 4);
                dot = __builtin_fmaf(bf16_lo_to_f32(qq.x), acc[nb][i4 * 4 + 0], dot);
                dot = __builtin_fmaf(bf16_hi_to_f32(qq.x), acc[nb][i4 * 4 + 1], dot);
                dot = __builtin_fmaf(bf16_lo_to_f32(qq.y), acc[nb][i4 * 4 + 2], dot);
                dot = __builtin_fmaf(bf16_hi_to_f32(qq.y), acc[nb][i4 * 4 + 3], dot);
            }
        float sc = dot + __shfl_xor(dot, 32);
        sc = c.tok < c.len ? sc * p.scale_log2e : -INFINITY;
        const float m = wave32_max(sc);
        const float pv = __builtin_amdgcn_exp2f(sc - m);
        const float l = wave32_sum(pv);
        const long long pidx = ((long long)c.b * p.Hq + hq) * p.chunks_per_seq + chunk;
        float* po = p.part_o + pidx * 128;
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                float o[4];
#pragma unroll
                for (int k = 0; k < 4; ++k)   // masked tokens have p = 0 and their rows are clamped copies: finite
                    o[k] = wave32_sum_upper(pv * acc[4 + nb][i4 * 4 + k]);
                if (c.tl == 16) {
                    float4 w; w.x = o[0]; w.y = o[1]; w.z = o[2]; w.w = o[3];
                    *reinterpret_cast<float4*>(po + nb * 32 + i4 * 8 + c.half * 4) = w;
                }
            }
        if (c.lane == 0) {
            p.part_ml[pidx * 2] = m;
            p.part_ml[pidx * 2 + 1] = l;
        }
    }
}

// ---- several queries per sequence (chunked prefill, causal): the T newest cache rows of a sequence
// are the queries' own tokens; query t sits at row len - T + t and sees rows 0 .. that row.
// Scores and the weighted sum go through the matrix cores, 32 (query, head) rows at a time:
//   S^T[token][query] = K Q^T : A = the wave's K rows straight from the accumulator (a lane's 8
//       registers of one 16-column k-step are 8 contraction indices in a fixed permuted order that
//       the Q fragment loads mirror), split into bf16 hi + lo (two MFMAs per k-step);
//   the result has lane = query, registers = 16 of the 32 tokens (the other lane half holds the
//       other 16): mask, max, exp2 and sum are per-lane loops plus one exchange between halves;
//   O[query][n] = P V : A = the softmax weights as they sit in those registers (hi + lo), B = V
//       read column-wise, for which V is transposed once per tile through the wave's own piece of
//       LDS (bf16 hi and lo images [n][32 tokens], 64-byte rows whose 8-byte pieces are XOR-swizzled
//       by the row: conflict-free fragment reads); hi*hi + lo*hi + hi*lo, the lo*lo term (2^-16
//       relative) is dropped.
// The eight waves' results are then merged inside the workgroup (maxima and sums exchanged
// through LDS, the rescaled O blocks summed in fixed wave order through a 32 KB staging area), so
// that one partial (m, l, o[128]) per (query, head, 256-token tile) goes to memory; the same
// combine kernel merges the tiles.  LDS: 8 x 16 KB of V images, then the staging area.
constexpr int VT_IMAGE_BYTES = 128 * 64;
constexpr int VT_WAVE_BYTES = 2 * VT_IMAGE_BYTES;
constexpr int PF_STAGE_OFF = 8 * VT_WAVE_BYTES;
constexpr int PF_STAGE_BYTES = 8 * 16 * 64 * 4;        // [wave][register][lane] fp32 of one 32-column block
constexpr int LDS_PREFILL_TOTAL = PF_STAGE_OFF + PF_STAGE_BYTES;
static_assert(LDS_PREFILL_TOTAL <= LDS_MAX, "prefill epilogue LDS");

// byte offset of the 8-byte piece (4 tokens) `piece` of row n inside a V image
__device__ __forceinline__ int vt_offset(int n, int piece) { return n * 64 + ((piece ^ ((n >> 2) & 7)) << 3); }

__device__ __forceinline__ void split_bf16x8(const float (&v)[8], uint4& hi, uint4& lo)
{
    uint32_t h[4], l[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        h[i] = pack_bf16x2_rne(v[2 * i], v[2 * i + 1]);
        l[i] = pack_bf16x2_rne(v[2 * i] - bf16_lo_to_f32(h[i]), v[2 * i + 1] - bf16_hi_to_f32(h[i]));
    }
    hi = make_uint4(h[0], h[1], h[2], h[3]);
    lo = make_uint4(l[0], l[1], l[2], l[3]);
}

__device__ __forceinline__ f32x16 mfma_bf16(const uint4& a, const uint4& b, const f32x16& c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// Called by all eight waves of the workgroup (it contains workgroup barriers); the LDS must not be
// read or written by anything else any more.
__device__ __forceinline__ void prefill_epilogue(const RematParams& p, const TileCtx& c, f32x16 (&acc)[8], uint8_t* lds)
{
    const int tok0 = c.tile * TILE_TOKENS + c.wave * CHUNK_TOKENS;
    const bool active = tok0 < c.len;                                      // wave-uniform: chunk not entirely past len
    uint8_t* vt = lds + c.wave * VT_WAVE_BYTES;
    uint4 khi[8], klo[8];
    if (active) {
        if (p.rope) rope_rotate(p, c, acc);
        // V^T images: element i of block 4 + nb is V[token tl][n], n = 32 nb + 8 (i/4) + 4 half + i%4
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int n = nb * 32 + (i >> 2) * 8 + c.half * 4 + (i & 3);
                const float v = acc[4 + nb][i];
                const uint32_t h = pack_bf16x2_rne(v, 0.0f);
                uint8_t* dst = vt + vt_offset(n, c.tl >> 2) + (c.tl & 3) * 2;
                *reinterpret_cast<uint16_t*>(dst) = (uint16_t)h;
                *reinterpret_cast<uint16_t*>(dst + VT_IMAGE_BYTES) = (uint16_t)pack_bf16x2_rne(v - bf16_lo_to_f32(h), 0.0f);
            }
        // K fragments: k-step ks covers columns [16 ks, 16 ks + 16); this lane's 8 of them are
        // 16 ks + 4 half + [0, 4) and 16 ks + 8 + 4 half + [0, 4)
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            float v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = acc[ks >> 1][(ks & 1) * 8 + k];
            split_bf16x8(v, khi[ks], klo[ks]);
        }
    }
    __builtin_amdgcn_wave_barrier();

    const int gq = p.Hq / p.Hkv, NQ = p.Tq * gq;
    const int jq = c.tl;
    float* mbuf = reinterpret_cast<float*>(lds + PF_STAGE_OFF);            // [wave][32 queries]
    float* lbuf = mbuf + 8 * 32;
    float* stage = reinterpret_cast<float*>(lds + PF_STAGE_OFF);           // [wave][16][64]
    for (int q0 = 0; q0 < NQ; q0 += 32) {
        // this lane's query row of the group (rows past NQ repeat the last one and are not stored)
        const int qi = min(q0 + jq, NQ - 1);
        const int tq = qi / gq, hq = c.hk * gq + (qi - tq * gq);
        const long long qrow = ((long long)c.b * p.Tq + tq) * p.Hq + hq;
        float m = -INFINITY, l = 0.0f;
        float pr[16];
        if (active) {
            const uint16_t* qv = p.q + qrow * 128 + c.half * 4;
            f32x16 S;
#pragma unroll
            for (int i = 0; i < 16; ++i) S[i] = 0.0f;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const uint2 a = *reinterpret_cast<const uint2*>(qv + 16 * ks);
                const uint2 b = *reinterpret_cast<const uint2*>(qv + 16 * ks + 8);
                const uint4 qf = make_uint4(a.x, a.y, b.x, b.y);
                S = mfma_bf16(khi[ks], qf, S);
                S = mfma_bf16(klo[ks], qf, S);
            }
            // register r <-> token tok0 + 8 (r/4) + 4 half + r%4; visible up to the query's own row
            const int limit = c.len - p.Tq + tq - tok0;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int rel = (r >> 2) * 8 + c.half * 4 + (r & 3);
                S[r] = rel <= limit ? S[r] * p.scale_log2e : -INFINITY;
                m = fmaxf(m, S[r]);
            }
            m = fmaxf(m, __shfl_xor(m, 32));
            const float mu = m == -INFINITY ? 0.0f : m;                    // nothing visible: all weights 0
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                pr[r] = __builtin_amdgcn_exp2f(S[r] - mu);
                l += pr[r];
            }
            l += __shfl_xor(l, 32);
        }
        // maxima and sums of the eight chunks -> the tile's maximum M, this wave's factor 2^(m - M)
        if (c.half == 0) {
            mbuf[c.wave * 32 + jq] = m;
            lbuf[c.wave * 32 + jq] = l;
        }
        __syncthreads();
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < 8; ++w) M = fmaxf(M, mbuf[w * 32 + jq]);
        const float Mu = M == -INFINITY ? 0.0f : M;
        float Lt = 0.0f;
#pragma unroll
        for (int w = 0; w < 8; ++w) Lt = __builtin_fmaf(lbuf[w * 32 + jq], __builtin_amdgcn_exp2f(mbuf[w * 32 + jq] - Mu), Lt);
        const float f = __builtin_amdgcn_exp2f(m - Mu);                    // per lane-query
        __syncthreads();                                                   // mbuf / lbuf are reused as staging
        if (c.wave == 0 && c.half == 0 && q0 + jq < NQ) {
            const long long pidx = qrow * p.chunks_per_seq + c.tile;
            p.part_ml[pidx * 2] = M;
            p.part_ml[pidx * 2 + 1] = Lt;
        }
        uint4 phi[2], plo[2];
        float fr[16];                                                      // the factor of register r's query
        if (active) {
#pragma unroll
            for (int k2 = 0; k2 < 2; ++k2) {
                float v[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) v[k] = pr[k2 * 8 + k];
                split_bf16x8(v, phi[k2], plo[k2]);
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) fr[r] = __shfl(f, (r >> 2) * 8 + c.half * 4 + (r & 3));
        }
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) {
            f32x16 O;
#pragma unroll
            for (int i = 0; i < 16; ++i) O[i] = 0.0f;
            if (active) {
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2) {
                    // column n = 32 nb + jq of V, tokens 16 k2 + 4 half + [0, 4) and 16 k2 + 8 + 4 half + [0, 4)
                    const int n = nb * 32 + jq;
                    const uint8_t* v0 = vt + vt_offset(n, 4 * k2 + c.half);
                    const uint8_t* v1 = vt + vt_offset(n, 4 * k2 + c.half + 2);
                    const uint2 h0 = *reinterpret_cast<const uint2*>(v0), h1 = *reinterpret_cast<const uint2*>(v1);
                    const uint2 l0 = *reinterpret_cast<const uint2*>(v0 + VT_IMAGE_BYTES);
                    const uint2 l1 = *reinterpret_cast<const uint2*>(v1 + VT_IMAGE_BYTES);
                    const uint4 vh = make_uint4(h0.x, h0.y, h1.x, h1.y), vl = make_uint4(l0.x, l0.y, l1.x, l1.y);
                    O = mfma_bf16(plo[k2], vh, O);
                    O = mfma_bf16(phi[k2], vl, O);
                    O = mfma_bf16(phi[k2], vh, O);
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) O[r] *= fr[r];
            }
            // O: lane = column 32 nb + jq, register r <-> query q0 + 8 (r/4) + 4 half + r%4.
            // Sum over the waves in fixed order; wave w reduces and stores registers 2 w, 2 w + 1.
#pragma unroll
            for (int r = 0; r < 16; ++r) stage[(c.wave * 16 + r) * 64 + c.lane] = O[r];
            __syncthreads();
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int r = 2 * c.wave + k;
                float sum = stage[r * 64 + c.lane];
#pragma unroll
                for (int w = 1; w < 8; ++w) sum += stage[(w * 16 + r) * 64 + c.lane];
                const int qr = q0 + (r >> 2) * 8 + c.half * 4 + (r & 3);
                if (qr < NQ) {
                    const int tr = qr / gq, hr = c.hk * gq + (qr - tr * gq);
                    p.part_o[((((long long)c.b * p.Tq + tr) * p.Hq + hr) * p.chunks_per_seq + c.tile) * 128 + nb * 32 + jq] = sum;
                }
            }
            __syncthreads();
        }
    }
}

// ---- latent cache (Sec. 3.3.1), pass 1: the wave holds the keys of two KV heads of its 32 tokens
// (blocks 0-3: head 2 pair, blocks 4-7: head 2 pair + 1) and stores the scaled scores of their
// query heads; pass 2 turns them into softmax partials against the values.
__device__ __forceinline__ void scores_epilogue(const RematParams& p, const TileCtx& c, f32x16 (&acc)[8])
{
    if (c.tile * TILE_TOKENS + c.wave * CHUNK_TOKENS >= c.len) return;
    const int gq = p.Hq / p.Hkv;
    const long long srow = p.score_stride;
    const int tok_out = p.tok0.v[c.b] + c.tok;
    static_for<0, 2>([&](auto HH) XQ_INLINE_LAMBDA {       // (compile-time: the accumulator must stay in registers)
        constexpr int hh = decltype(HH)::value;
        for (int j = 0; j < gq; ++j) {
            const int hq = (2 * c.hk + hh) * gq + j;
            const uint16_t* qv = p.q + ((long long)c.b * p.Hq + hq) * 128;
            float dot = 0.0f;
#pragma unroll
            for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const uint2 qq = *reinterpret_cast<const uint2*>(qv + nb * 32 + i4 * 8 + c.half * 4);
                    const f32x16& a = acc[4 * hh + nb];
                    dot = __builtin_fmaf(bf16_lo_to_f32(qq.x), a[i4 * 4 + 0], dot);
                    dot = __builtin_fmaf(bf16_hi_to_f32(qq.x), a[i4 * 4 + 1], dot);
                    dot = __builtin_fmaf(bf16_lo_to_f32(qq.y), a[i4 * 4 + 2], dot);
                    dot = __builtin_fmaf(bf16_hi_to_f32(qq.y), a[i4 * 4 + 3], dot);
                }
            const float sc = (dot + __shfl_xor(dot, 32)) * p.scale_log2e;
            if (c.half == 0 && c.tok < c.len) p.scores[((long long)c.b * p.Hq + hq) * srow + tok_out] = sc;
        }
    });
}

// pass 2: blocks 0-3 / 4-7 hold the values of the two KV heads; one partial (m, l, o[128]) per query head
__device__ __forceinline__ void weighted_sum_epilogue(const RematParams& p, const TileCtx& c, f32x16 (&acc)[8])
{
    if (c.tile * TILE_TOKENS + c.wave * CHUNK_TOKENS >= c.len) return;
    const int gq = p.Hq / p.Hkv;
    const int chunk = c.tile * (TILE_TOKENS / CHUNK_TOKENS) + c.wave;
    const long long srow = p.score_stride;
    static_for<0, 2>([&](auto HH) XQ_INLINE_LAMBDA {
        constexpr int hh = decltype(HH)::value;
        for (int j = 0; j < gq; ++j) {
            const int hq = (2 * c.hk + hh) * gq + j;
            float sc = p.scores[((long long)c.b * p.Hq + hq) * srow + min(c.tok, c.len - 1)];
            sc = c.tok < c.len ? sc : -INFINITY;
            const float m = wave32_max(sc);
            const float pv = __builtin_amdgcn_exp2f(sc - m);
            const float l = wave32_sum(pv);
            const long long pidx = ((long long)c.b * p.Hq + hq) * p.chunks_per_seq + chunk;
            float* po = p.part_o + pidx * 128;
#pragma unroll
            for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const f32x16& a = acc[4 * hh + nb];
                    float o[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) o[k] = wave32_sum_upper(pv * a[i4 * 4 + k]);
                    if (c.tl == 16) {
                        float4 w; w.x = o[0]; w.y = o[1]; w.z = o[2]; w.w = o[3];
                        *reinterpret_cast<float4*>(po + nb * 32 + i4 * 8 + c.half * 4) = w;
                    }
                }
            if (c.lane == 0) {
                p.part_ml[pidx * 2] = m;
                p.part_ml[pidx * 2 + 1] = l;
            }
        }
    });
}

// ---- cross-layer accumulator of grouped-query models (Sec. 3.3.2): the contraction is the
// up-projection of a cached latent delta through U_kv^T, "head" hk = 256 adjacent hidden channels.
// The wave adds its 32 tokens x 256 channels to the bf16 accumulator rows (fp32 add, one RNE
// rounding).  In the accumulator layout a lane owns 4 adjacent channels of one token, which would
// touch 32 rows with 16 bytes each per memory instruction; so 64 channels at a time are turned
// through a wave-private piece of LDS (the weight slabs are dead by now: the last workgroup
// barrier of the contraction loop comes after the last read of them) into rows of 8 lanes x 16
// bytes, and every read-modify-write instruction covers 8 full 128-byte lines.
constexpr int STAGE_ROW_BYTES = 64 * 4 + 16;       // 64 fp32 + 16: rows start 4 banks apart
static_assert(8 * CHUNK_TOKENS * STAGE_ROW_BYTES <= 2 * SLAB_BYTES, "staging fits the slab buffers");

__device__ __forceinline__ void accumulate_epilogue(const RematParams& p, const TileCtx& c, f32x16 (&acc)[8],
                                                    uint8_t* lds)
{
    const int tok0 = c.tile * TILE_TOKENS + c.wave * CHUNK_TOKENS;
    if (tok0 >= c.len) return;                                             // wave-uniform
    uint8_t* stage = lds + c.wave * (CHUNK_TOKENS * STAGE_ROW_BYTES);
    const int r0 = c.lane >> 3, c8 = c.lane & 7;                           // row in a group of 8; 8-channel piece
    uint16_t* gbase = p.acc_out + ((long long)c.b * p.cap + tok0) * p.d_out + c.hk * 256 + c8 * 8;
    // all 16 old pieces first, so that their latency is paid once (rows past len: a clamped copy, not stored)
    uint4 old[4][4];
#pragma unroll
    for (int pb = 0; pb < 4; ++pb)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int r = min(r0 + 8 * k, c.len - 1 - tok0);
            old[pb][k] = *reinterpret_cast<const uint4*>(gbase + (long long)r * p.d_out + pb * 64);
        }
    static_for<0, 4>([&](auto PB) XQ_INLINE_LAMBDA {
        constexpr int pb = decltype(PB)::value;
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const f32x16& a = acc[2 * pb + q];
                float4 v; v.x = a[i4 * 4 + 0]; v.y = a[i4 * 4 + 1]; v.z = a[i4 * 4 + 2]; v.w = a[i4 * 4 + 3];
                *reinterpret_cast<float4*>(stage + c.tl * STAGE_ROW_BYTES + (q * 32 + i4 * 8 + c.half * 4) * 4) = v;
            }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int r = r0 + 8 * k;
            const float4 lo = *reinterpret_cast<const float4*>(stage + r * STAGE_ROW_BYTES + c8 * 32);
            const float4 hi = *reinterpret_cast<const float4*>(stage + r * STAGE_ROW_BYTES + c8 * 32 + 16);
            if (tok0 + r < c.len) {
                const uint4 o = old[pb][k];
                uint4 upd;
                upd.x = pack_bf16x2_rne(bf16_lo_to_f32(o.x) + lo.x, bf16_hi_to_f32(o.x) + lo.y);
                upd.y = pack_bf16x2_rne(bf16_lo_to_f32(o.y) + lo.z, bf16_hi_to_f32(o.y) + lo.w);
                upd.z = pack_bf16x2_rne(bf16_lo_to_f32(o.z) + hi.x, bf16_hi_to_f32(o.z) + hi.y);
                upd.w = pack_bf16x2_rne(bf16_lo_to_f32(o.w) + hi.z, bf16_hi_to_f32(o.w) + hi.w);
                *reinterpret_cast<uint4*>(gbase + (long long)r * p.d_out + pb * 64) = upd;
            }
        }
        __builtin_amdgcn_wave_barrier();
    });
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

// =====================================================================================
// coded source (XQuant cache, BITS in {2,3,4})
// =====================================================================================
// MODE selects what happens to the 256 rematerialised columns of the wave's 32 tokens: decode
// attention ([K_h | V_h]) with the per-query-head vector epilogue; one of the two passes over a
// latent cache, where the columns are the keys (pass 1) or the values (pass 2) of a PAIR of KV
// heads; the up-projection of cross-layer latent deltas into the bf16 accumulator (the columns are
// 256 hidden channels); or attention for many (query, head) rows per KV head through the
// matrix-core epilogue (prefill chunks, and decode when a KV head serves several query heads).
//
// MODE_ATTENTION_PC reads a per-channel cache (Sec. 3.3.1: one scale and zero-point per channel and
// block of 64 or 128 tokens).  The scale now varies along the contraction, so it moves to the token
// operand: each unpacked operand dword is multiplied (packed fp16) by the block's factors
// scale * 2^(15 - E_blk) of its two channels -- an 8-bit significand times a code of at most 3 bits
// is exact in fp16 (4-bit codes enter as code - 8, which makes their products exact too: the
// block-constant 8 * scale term joins the zero-point term), and one exponent per block suffices because fp16
// subnormals keep an absolute precision of 2^-24 against the block's largest scale.  All tokens of
// a wave lie in one block, so the factors come from a small LDS image (one per slab, three
// rotating buffers) by broadcast reads.  There is no Horner rescale and no correction phase; the
// zero-point term z_blk [Wk_h | Wv_h] is the same for every token of a block, comes from a
// pre-pass and is added in the epilogue together with the block's power of two.
template <int BITS, int G, int MODE>
__global__ __launch_bounds__(512) void remat_attn_coded_kernel(const RematParams p)
{
    constexpr int KSG = G / 16;                        // k-steps per quantisation group
    constexpr int GPS = 8 / KSG;                       // groups per slab (1 or 2)
    constexpr int NDW_G = (G / 2) * BITS / 32;         // code dwords per lane per group
    constexpr int NDW = GPS * NDW_G;                   // ... per slab (= 2 BITS)
    constexpr int ROW_SLAB_BYTES = 16 * BITS;          // packed bytes of 128 channels of one token
    constexpr int NCI = 4 * BITS;                      // code-DMA wave instructions per slab per workgroup
    constexpr int IMG_BYTES = code_image_bytes(BITS);
    constexpr int NIMG = n_code_images(BITS);
    constexpr int LDS_SCALES_OFF = lds_scales_off(BITS);
    constexpr bool PC = MODE == MODE_ATTENTION_PC || MODE == MODE_SCORES_PC;   // per-channel source: factors on the token operand

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    TileCtx c;
    if (!locate_tile(p, c)) return;
    const int lane = c.lane, wave = c.wave, half = c.half, tl = c.tl;

    const int n_corr_slabs = (p.n_corr_ksteps + SLAB_KSTEPS - 1) / SLAB_KSTEPS;
    const uint8_t* wsrc = p.wprep + (long long)c.hk * p.head_bytes + wave * 1024;   // this wave's DMA share
    const uint32_t dma_voff = (uint32_t)lane * 16u;
    const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) uint8_t*)lds;
    const uint32_t lds_w = lds_base + wave * 1024;
    const uint8_t* my_slab = lds + lane * 16;          // + buffer * SLAB_BYTES + (ks * 8 + nb) * 1024

    // ---- token-side sources
    const long long seq_row0 = (long long)c.b * p.cap;
    const uint32_t row_bytes = (uint32_t)(p.row_d * BITS / 8);
    const uint8_t* cbase = p.codes + seq_row0 * row_bytes;
    const uint16_t* zbase = p.zero + seq_row0 * p.ng_row;
    // per-token source: effective scales, GPS * 512 bytes per slab; per-channel: one 1 KiB factor image per slab
    const int e_slab_bytes = PC ? LDS_SCALES_BYTES : GPS * 512;
    const uint8_t* ebase = reinterpret_cast<const uint8_t*>(p.eT) +
                           (PC ? ((long long)c.b * p.tiles_per_seq + c.tile) * (long long)(p.n_main_slabs + 1) * LDS_SCALES_BYTES
                               : ((long long)c.b * p.tiles_per_seq + c.tile) * (long long)(p.ng + 1) * 512);
    const uint32_t moff = (uint32_t)min(c.tok, c.len - 1) * (uint32_t)p.ng_row;

    // code DMA: 16-byte piece pc of the tile's slab image = (row pc / BITS, part pc % BITS);
    // wave instruction i covers pieces [64 i, 64 i + 64); this wave issues i = wave and wave + 8
    uint32_t cvoff[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int pc = (wave + 8 * k) * 64 + lane;
        const int rl = pc / BITS, prt = pc % BITS;
        cvoff[k] = (uint32_t)min(c.tile * TILE_TOKENS + rl, c.len - 1) * row_bytes + prt * 16;
    }
    // this lane's codes / scales inside the LDS images
    const int my_row = wave * CHUNK_TOKENS + tl;
    const uint8_t* my_codes = lds + LDS_CODES_OFF + my_row * ROW_SLAB_BYTES + half * (NDW_G * 4);
    const uint16_t* my_scale = reinterpret_cast<const uint16_t*>(lds + LDS_SCALES_OFF) + my_row;

    // Workgroups that run side by side on one XCD stream the same head and all start the cyclic
    // walk at slab 0: they advance at about the same pace, so a slab is fetched into the XCD's L2
    // once and hit by the others.  (Starting each workgroup at a different slab was measured: it
    // raises the L2 miss traffic by a third and the kernel time by 7 %.)

    f32x16 acc[8];                       // [column block]: 0-3 K, 4-7 V
#pragma unroll
    for (int nb = 0; nb < 8; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[nb][i] = 0.0f;

    // MFMA operands
    constexpr int NB = 2 * GPS - 1;      // kinds of group boundary a slab's ticks can see
    uint4 af[8];                         // weight fragments, ring over slots (loaded 7 slots ahead)
    uint32_t ub[8][4];                   // token fragments, ring over k-steps
    uint32_t cur[NDW];                   // packed codes of the current slab
    float E[2 * GPS];                    // effective scales: groups of the previous slab, then of the current one
    float hr_b[NB];                      // Horner factors E[k] / E[k+1] of the boundaries seen this slab

    // effective scales of the slab processed at main iteration `iter` (its buffer is iter & 1)
    auto fetch_scales = [&](int sbuf, float* e) {
#pragma unroll
        for (int gi = 0; gi < GPS; ++gi)
            e[gi] = __uint_as_float((uint32_t)my_scale[sbuf * (LDS_SCALES_BYTES / 2) + gi * TILE_TOKENS] << 16);
    };
    // pull this lane's codes of the landed slab out of LDS
    auto fetch_tokens = [&](int img) {
#pragma unroll
        for (int gi = 0; gi < GPS; ++gi) {
            const uint8_t* src = my_codes + img * IMG_BYTES + gi * (2 * NDW_G * 4);
            if constexpr (NDW_G % 4 == 0) {
#pragma unroll
                for (int i = 0; i < NDW_G / 4; ++i) {
                    const uint4 v = reinterpret_cast<const uint4*>(src)[i];
                    cur[gi * NDW_G + 4 * i] = v.x; cur[gi * NDW_G + 4 * i + 1] = v.y;
                    cur[gi * NDW_G + 4 * i + 2] = v.z; cur[gi * NDW_G + 4 * i + 3] = v.w;
                }
            } else if constexpr (NDW_G % 2 == 0) {
#pragma unroll
                for (int i = 0; i < NDW_G / 2; ++i) {
                    const uint2 v = reinterpret_cast<const uint2*>(src)[i];
                    cur[gi * NDW_G + 2 * i] = v.x; cur[gi * NDW_G + 2 * i + 1] = v.y;
                }
            } else {
#pragma unroll
                for (int i = 0; i < NDW_G; ++i) cur[gi * NDW_G + i] = reinterpret_cast<const uint32_t*>(src)[i];
            }
        }
    };
    // per-channel source: multiply the operand dwords of k-step ks by the block's factors of their channels
    // (image of the slab in scale buffer sbuf: [block of the tile][k-step][lane half][8 fp16], broadcast read)
    const uint8_t* my_factors = lds + LDS_SCALES_OFF + (PC ? ((wave * CHUNK_TOKENS) / p.pc_block) * 256 + half * 16 : 0);
    auto scale_frag = [&](uint32_t* frag, int sbuf, int ks) {
        const uint4 f = *reinterpret_cast<const uint4*>(my_factors + sbuf * LDS_SCALES_BYTES + ks * 32);
        if constexpr (BITS == 4) {
            // a 4-bit code times an 8-bit significand needs 12 bits; (code - 8) times it needs 11 and is exact in
            // fp16.  All 4-bit fields sit at mantissa offset 6, so 8 is the subnormal 2^-15 in both halves; the
            // 8 * scale * W that this takes out is the same for every token of the block and comes back with
            // the zero-point term.
            constexpr uint32_t MINUS_EIGHT = 0x82008200u;
#pragma unroll
            for (int i = 0; i < 4; ++i) frag[i] = pk_add_f16(frag[i], MINUS_EIGHT);
        }
        frag[0] = pk_mul_f16(frag[0], f.x);
        frag[1] = pk_mul_f16(frag[1], f.y);
        frag[2] = pk_mul_f16(frag[2], f.z);
        frag[3] = pk_mul_f16(frag[3], f.w);
    };
    // one piece of the DMA that brings in main slab `slab` (weights to `wdst`): steps 0,1 this wave's
    // code pieces (to code image `img`), 2 scales (wave 7; of slab `slab2`, into scale buffer `sbuf`),
    // 3..10 the weight chunks
    auto dma_step = [&](int step, int slab, int img, int slab2, bool with_scales2, int sbuf, uint32_t wdst) {
        if (step < 2) {
            if (wave + 8 * step < NCI)
                dma_b128(cbase + slab * ROW_SLAB_BYTES, cvoff[step],
                         lds_base + LDS_CODES_OFF + (uint32_t)(img * IMG_BYTES) + (wave + 8 * step) * 1024);
        } else if (step == 2) {
            if (with_scales2 && wave == 7)
                dma_b128(ebase + (long long)slab2 * e_slab_bytes, dma_voff, lds_base + LDS_SCALES_OFF + (uint32_t)(sbuf * LDS_SCALES_BYTES));
        } else {
            dma_b128(wsrc + (long long)slab * SLAB_BYTES + (step - 3) * 8192, dma_voff, wdst + (step - 3) * 8192);
        }
    };

    // ==== phase 1: the zero-point correction (scale 1), a few bf16 k-steps whose token-side
    // operands are the stored zero-points.  Its operands are loaded
    // first thing, so their latency hides behind the first weight DMA.  The codes and scales of the
    // slab that cyclically precedes the first one arrive meanwhile: the lagging column blocks start
    // inside it (see phase 2).
    const bool vec_meta = (p.ng & 7) == 0 && (p.ng_row & 7) == 0 && ((size_t)zbase & 15) == 0;
    auto load_meta = [&](int kk) -> uint4 {
        const int kappa0 = kk * 16 + half * 8;
        const int term = kappa0 / p.ng_pad, g0 = kappa0 % p.ng_pad;
        const uint16_t* mbase = zbase;
        uint4 v = {0u, 0u, 0u, 0u};
        if (kk < p.n_corr_ksteps && term < N_CORR_TERMS) {
            if (vec_meta) {
                v = *reinterpret_cast<const uint4*>(mbase + moff + g0);
            } else {
                uint32_t h[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int g = g0 + i;
                    const uint32_t x = mbase[moff + min(g, p.ng - 1)];
                    h[i] = g < p.ng ? x : 0u;               // padding groups contribute nothing
                }
                v.x = h[0] | (h[1] << 16); v.y = h[2] | (h[3] << 16);
                v.z = h[4] | (h[5] << 16); v.w = h[6] | (h[7] << 16);
            }
        }
        return v;
    };
    const int slab_prev = p.n_main_slabs - 1;           // the walk is cyclic: the slab "before" slab 0
    issue_slab(wsrc + (long long)p.n_main_slabs * SLAB_BYTES, lds_w, dma_voff);        // correction slab 0 -> buffer 0
    dma_step(0, slab_prev, NIMG - 1, 0, false, 0, 0);                                  // predecessor codes -> last image
    dma_step(1, slab_prev, NIMG - 1, 0, false, 0, 0);
    dma_step(2, 0, 0, slab_prev, true, 2, 0);                                          // its scales -> scale buffer 2
    dma_step(2, 0, 0, 0, true, 0, 0);                                                // first slab's scales -> buffer 0
    if (p.n_main_slabs > 1) dma_step(2, 0, 0, 1, true, 1, 0);            // second slab's -> buffer 1
    if constexpr (NIMG == 2) {                                                         // first slab's codes -> image 0
        dma_step(0, 0, 0, 0, false, 0, 0);
        dma_step(1, 0, 0, 0, false, 0, 0);
    }
    uint4 mfr[SLAB_KSTEPS];
    if constexpr (!PC) {
#pragma unroll
        for (int ks = 0; ks < SLAB_KSTEPS; ++ks) mfr[ks] = load_meta(ks);
    }
    for (int cs = 0; cs < n_corr_slabs; ++cs) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        const uint32_t wdst = lds_w + (uint32_t)(((cs + 1) & 1) * SLAB_BYTES);
        if (cs + 1 < n_corr_slabs) issue_slab(wsrc + (long long)(p.n_main_slabs + cs + 1) * SLAB_BYTES, wdst, dma_voff);
        else issue_slab(wsrc, wdst, dma_voff);                                                   // the first main slab
        if (cs == 0) {
            fetch_tokens(NIMG - 1);
            if constexpr (!PC) fetch_scales(2, &E[0]);
        }
        const uint8_t* slab = my_slab + (cs & 1) * SLAB_BYTES;
        const int nks = min(SLAB_KSTEPS, p.n_corr_ksteps - cs * SLAB_KSTEPS);
#pragma unroll
        for (int nb = 0; nb < 8; ++nb) af[nb] = *reinterpret_cast<const uint4*>(slab + nb * 1024);
#pragma unroll
        for (int ks = 0; ks < SLAB_KSTEPS; ++ks) {
            if (!PC && ks < nks) {                    // (per-channel source: the zero-point term comes from a pre-pass)
#pragma unroll
                for (int nb = 0; nb < 8; ++nb) {
                    acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[nb]),
                                                                       __builtin_bit_cast(bf16x8, mfr[ks]), acc[nb], 0, 0, 0);
                    if (ks + 1 < SLAB_KSTEPS)
                        af[nb] = *reinterpret_cast<const uint4*>(slab + ((ks + 1) * 8 + nb) * 1024);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if constexpr (NIMG == 1) {
                if (ks == 0 && cs == 0) {
                    // every wave now holds its predecessor codes in registers: the first slab's
                    // codes may overwrite the only image
                    __syncthreads();
                    dma_step(0, 0, 0, 0, false, 0, 0);
                    dma_step(1, 0, 0, 0, false, 0, 0);
                }
            }
        }
        if constexpr (!PC) {
            if (cs + 1 < n_corr_slabs) {
#pragma unroll
                for (int ks = 0; ks < SLAB_KSTEPS; ++ks) mfr[ks] = load_meta((cs + 1) * SLAB_KSTEPS + ks);
            }
        }
    }

    // ==== phase 2: the d x 256 contraction, as a cyclic walk over the d/16 k-steps that starts
    // at slab 0.  Column block j runs 7 - j k-steps behind the walk: at tick tau it multiplies
    // the weights of k-step tau - 7 + j (the prepared stream is laid out in this order) with the
    // token fragment unpacked 7 - j ticks ago, which waits in an 8-deep ring.  The group
    // boundaries of the eight blocks therefore fall on different ticks, and the Horner rescale
    // of the accumulator (16 multiplies per block and boundary) spreads evenly over the loop
    // instead of piling up at the slab boundary, where every wave would do it at once.
    //
    // Set-up: the ring's lagging fragments are k-steps 1..7 of the predecessor slab, whose group
    // scales E[0..GPS) the lagging blocks start from; the accumulators (holding the correction in
    // units of 1) are brought to those scales.
#pragma unroll
    for (int ks = 1; ks < SLAB_KSTEPS; ++ks) {
        unpack_kstep<BITS>(&cur[(ks / KSG) * NDW_G + ((ks % KSG) >> 2) * BITS], ks % KSG, ub[ks]);
        if constexpr (PC) scale_frag(ub[ks], 2, ks);       // (the predecessor slab's factors wait in buffer 2)
    }
    const int par0 = n_corr_slabs & 1;                 // weight buffer of main iteration 0
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    fetch_tokens(0);
    if constexpr (!PC) fetch_scales(0, &E[GPS]);
    {
        const uint8_t* slab0 = my_slab + par0 * SLAB_BYTES;
#pragma unroll
        for (int sl = 0; sl < 7; ++sl) af[sl] = *reinterpret_cast<const uint4*>(slab0 + sl * 1024);
        if constexpr (!PC) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float r0 = __builtin_amdgcn_rcpf(E[floordiv_c(j - 8, KSG) + GPS]);
                acc[j] *= r0;
            }
#pragma unroll
            for (int k = 0; k < NB; ++k) hr_b[k] = E[k] * __builtin_amdgcn_rcpf(E[k + 1]);
        }
        unpack_kstep<BITS>(&cur[0], 0, ub[0]);
        if constexpr (PC) scale_frag(ub[0], 0, 0);
    }

    // Multiplies chunk CIDX (of 3,3,3,3,2,2 registers) of one block's accumulator by h.  The empty
    // asm statement consumes the products here, in its slot: pure arithmetic is otherwise free to
    // drift to the end of the loop body during instruction selection.
    auto rescale_chunk = [&](f32x16& a, auto CIDX, float h) XQ_INLINE_LAMBDA {
        constexpr int cidx = decltype(CIDX)::value;
        constexpr int off = cidx < 4 ? 3 * cidx : 12 + 2 * (cidx - 4);
        float x0 = a[off] * h, x1 = a[off + 1] * h;
        if constexpr (cidx < 4) {
            float x2 = a[off + 2] * h;
            asm volatile("" :: "v"(x0), "v"(x1), "v"(x2));
            a[off + 2] = x2;
        } else {
            asm volatile("" :: "v"(x0), "v"(x1));
        }
        a[off] = x0; a[off + 1] = x1;
    };
    // The rescale work of slot SIDX (= 8 tick + block, may name the tail of the previous slab):
    // a block whose MFMA 1..6 slots ahead is the first of a group gets one chunk done now.
    auto horner_slot = [&](auto SIDX, const float (&hcur)[NB], const float (&hnext)[NB], auto DO_CUR, bool have_next)
                           XQ_INLINE_LAMBDA {
        static_for<1, 7>([&](auto DELTA) XQ_INLINE_LAMBDA {
            constexpr int delta = decltype(DELTA)::value;
            constexpr int t = decltype(SIDX)::value + delta;
            constexpr int jt = t & 7;
            constexpr int kp = ((t >> 3) & 7) - 7 + jt;    // k-step, relative to the slab of its tick
            if constexpr (floordiv_c(kp, KSG) * KSG == kp) {
                constexpr int kind = floordiv_c(kp, KSG) + GPS - 1;
                if constexpr (t < 64) {
                    if constexpr (decltype(DO_CUR)::value) rescale_chunk(acc[jt], std::integral_constant<int, 6 - delta>{}, hcur[kind]);
                } else {
                    if (have_next) rescale_chunk(acc[jt], std::integral_constant<int, 6 - delta>{}, hnext[kind]);
                }
            }
        });
    };
    // boundaries in the first slots of iteration 0 whose chunks belong to "the slab before"
    if constexpr (!PC)
        static_for<58, 64>([&](auto SIDX) XQ_INLINE_LAMBDA { horner_slot(SIDX, hr_b, hr_b, std::false_type{}, true); });

    // A tick is 8 slots of one MFMA each (slot = column block); the VALU/LDS/DMA work that feeds
    // later slots is spread over the slots and pinned there with scheduling fences so that it runs
    // in the shadow of the MFMAs.
    for (int it = 0; it < p.n_main_slabs; ++it) {
        // With a single code image, everyone must have taken the previous slab's codes out of it
        // before this slab's DMA refills it.  (The weight buffer needs no barrier here: its last
        // read was issued before the landing barrier of the previous iteration.  Iteration 0 keeps
        // one for the scale buffer that the set-up has just read.)
        if (NIMG == 1 || it == 0) __syncthreads();
        const int img_next = NIMG == 2 ? (it + 1) & 1 : 0;
        const bool more_main = it + 1 < p.n_main_slabs;
        const bool more_main2 = it + 2 < p.n_main_slabs;
        // (the last iterations issue their DMA all the same, from slabs that exist into buffers that
        // are not read again: no branches around the issue slots)
        const int s_next = more_main ? it + 1 : it;
        const int s_next2 = more_main2 ? it + 2 : it;
        const uint32_t wdst = lds_w + (uint32_t)(((it + 1 + par0) & 1) * SLAB_BYTES);
        const uint8_t* slab = my_slab + ((it + par0) & 1) * SLAB_BYTES;
        const uint8_t* slab_next = my_slab + ((it + 1 + par0) & 1) * SLAB_BYTES;
        // scale buffers: per-token source, slab s in buffer s & 1 (its scales are taken into registers one slab
        // ahead); per-channel source, slab s in buffer s % 3 (its factors are read all through its own iteration)
        const int sb_dma = PC ? (it + 2) % 3 : (it & 1);
        const int sb_cur = it % 3, sb_nxt = (it + 1) % 3;
        float e_nxt[GPS];                                    // scales of the next slab (landed one slab ago)
        float hr_bn[NB];                                     // boundary factors of the next iteration
#pragma unroll
        for (int k = 0; k < NB; ++k) hr_bn[k] = 1.0f;
        __builtin_amdgcn_sched_barrier(0);

        static_for<0, 64>([&](auto SIDX) XQ_INLINE_LAMBDA {
            {
                constexpr int sidx = decltype(SIDX)::value;
                constexpr int ks = sidx >> 3, m = sidx & 7;
                const uint32_t* b = ub[(ks + 1 + m) & 7];
                acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                    __builtin_bit_cast(f16x8, af[m]), as_frag(b[0], b[1], b[2], b[3]), acc[m], 0, 0, 0);

                // DMA of the next slab: 11 steps per wave, one every other slot.  (Issued in bursts they
                // fill the address FIFO and the issuing wave stalls with its MFMAs behind them.)
                if constexpr ((sidx >> 1) < 11 && (sidx & 1) == 0)
                    dma_step(sidx >> 1, s_next, img_next, s_next2, true, sb_dma, wdst);
                // the old codes are no longer needed: wait until the next slab has landed for everyone,
                // then take the next slab's codes
                if constexpr (ks == SLAB_KSTEPS - 1 && m == 1) {
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                    __syncthreads();
                    if (more_main) fetch_tokens(img_next);
                }
                // weight fragment of the slot 7 ahead (the last 7 slots of a slab read the next slab)
                if constexpr (sidx + 7 < 64) af[(sidx + 7) & 7] = *reinterpret_cast<const uint4*>(slab + (sidx + 7) * 1024);
                else if (more_main) af[(sidx + 7) & 7] = *reinterpret_cast<const uint4*>(slab_next + (sidx + 7 - 64) * 1024);
                // token fragment of the next tick; its ring entry was last read by this tick's slot 0
                if constexpr (ks + 1 < SLAB_KSTEPS) {
                    if constexpr (m == 2) {
                        constexpr int gi1 = (ks + 1) / KSG, ksg1 = (ks + 1) % KSG;
                        unpack_kstep<BITS>(&cur[gi1 * NDW_G + (ksg1 >> 2) * BITS], ksg1, ub[ks + 1]);
                        if constexpr (PC) scale_frag(ub[ks + 1], sb_cur, ks + 1);
                    }
                } else if constexpr (m == 7) {               // cur already holds the next slab's codes
                    if (more_main) {
                        unpack_kstep<BITS>(&cur[0], 0, ub[0]);
                        if constexpr (PC) scale_frag(ub[0], sb_nxt, 0);
                    }
                }
                // the next slab's scales are in LDS since the previous slab
                if constexpr (!PC && ks == SLAB_KSTEPS - 2 && m == 4) { if (more_main) fetch_scales((it + 1) & 1, e_nxt); }
                if constexpr (!PC && ks == SLAB_KSTEPS - 1 && m == 3) {
                    if (more_main) {
                        static_for<0, NB>([&](auto K) XQ_INLINE_LAMBDA {
                            constexpr int k = decltype(K)::value;
                            float en0, en1;
                            if constexpr (k < GPS) en0 = E[k + GPS]; else en0 = e_nxt[k - GPS];
                            if constexpr (k + 1 < GPS) en1 = E[k + 1 + GPS]; else en1 = e_nxt[k + 1 - GPS];
                            hr_bn[k] = en0 * __builtin_amdgcn_rcpf(en1);
                        });
                    }
                }
                if constexpr (!PC) horner_slot(SIDX, hr_b, hr_bn, std::true_type{}, more_main);
                __builtin_amdgcn_sched_barrier(0);
            }
        });
        if constexpr (!PC) {
            if (more_main) {
#pragma unroll
                for (int gi = 0; gi < GPS; ++gi) { E[gi] = E[gi + GPS]; E[gi + GPS] = e_nxt[gi]; }
#pragma unroll
                for (int k = 0; k < NB; ++k) hr_b[k] = hr_bn[k];
            }
        }
    }
    if constexpr (PC) {
        // K | V = accumulator * 2^(E_blk + bits - 1) + z_blk [Wk_h | Wv_h]; waves past len take the last block's
        const int blk = min((c.tile * TILE_TOKENS + wave * CHUNK_TOKENS) / p.pc_block, (c.len - 1) / p.pc_block);
        const long long brow = (long long)c.b * p.pc_blocks_cap + blk;
        const float fs = p.pc_fscale[brow];
        const float* zw = p.pc_zw + (brow * p.grid_heads + c.hk) * 256 + half * 4;
#pragma unroll
        for (int nb = 0; nb < 8; ++nb)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const float4 z = *reinterpret_cast<const float4*>(zw + nb * 32 + i4 * 8);
                acc[nb][i4 * 4 + 0] = __builtin_fmaf(acc[nb][i4 * 4 + 0], fs, z.x);
                acc[nb][i4 * 4 + 1] = __builtin_fmaf(acc[nb][i4 * 4 + 1], fs, z.y);
                acc[nb][i4 * 4 + 2] = __builtin_fmaf(acc[nb][i4 * 4 + 2], fs, z.z);
                acc[nb][i4 * 4 + 3] = __builtin_fmaf(acc[nb][i4 * 4 + 3], fs, z.w);
            }
    } else {
        // every block ends in the slab it started in; leave its group's scale: the accumulator is K | V
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] *= E[GPS + j / KSG];
    }
    if constexpr (MODE == MODE_SCORES || MODE == MODE_SCORES_PC) scores_epilogue(p, c, acc);
    else if constexpr (MODE == MODE_WEIGHTED_SUM) weighted_sum_epilogue(p, c, acc);
    else if constexpr (MODE == MODE_ACCUMULATE) accumulate_epilogue(p, c, acc, lds);
    else if constexpr (MODE == MODE_PREFILL) prefill_epilogue(p, c, acc, lds);
    else attention_epilogue(p, c, acc);
}

// =====================================================================================
// dense source (XQuant-CL accumulator, bf16).  A wave needs, per half slab (4 k-steps = 64
// channels), 128 contiguous bytes of each of its 32 token rows.  Loading them straight into the
// MFMA fragment layout touches 32 rows per instruction and keeps the texture unit busy longer
// than the MFMAs take; instead 4 LDS-DMA instructions fetch 8 rows x 128 B each (8 cache lines
// per instruction) into a 4 KiB staging area private to the wave, and 4 ds_read_b128 bring the
// fragments into registers.  Only the wave itself touches its staging area: the hand-over needs
// s_waitcnt, no barrier.  The 16-byte pieces are placed so that both the DMA's linear LDS
// write and the fragment read are conflict-free:  piece p of row r of block j sits in slot
// 8 (r%8) + (p ^ f),  f = ((r%8) >> 1) | ((j & 1) << 2).
// Per half slab h (32 MFMA slots): slot 16 takes the fragments of half h+1 out of staging, slots
// 20-23 issue the DMA of half h+2.
// =====================================================================================
constexpr int LDS_DENSE_STAGE_OFF = 2 * SLAB_BYTES;
constexpr int LDS_DENSE_STAGE_BYTES = 4096;            // per wave
constexpr int LDS_DENSE_TOTAL = LDS_DENSE_STAGE_OFF + 8 * LDS_DENSE_STAGE_BYTES;
static_assert(LDS_DENSE_TOTAL <= LDS_MAX, "dense kernel LDS");

// DMODE: 0 decode attention, 1 matrix-core epilogue (prefill), 2 store the rematerialised rows
// as fp32 (used for the zero-point term of a per-channel cache), 3 pass 1 of the latent path (scores of a
// pair of KV heads) for the rows of a residual window
constexpr int DENSE_ATTENTION = 0, DENSE_PREFILL = 1, DENSE_STORE = 2, DENSE_SCORES = 3;
template <int DMODE>
__global__ __launch_bounds__(512) void remat_attn_dense_kernel(const RematParams p)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    TileCtx c;
    if (!locate_tile(p, c)) return;
    const int lane = c.lane, wave = c.wave, half = c.half, tl = c.tl;

    const uint8_t* wsrc = p.wprep + (long long)c.hk * p.head_bytes + wave * 1024;
    const uint32_t dma_voff = (uint32_t)lane * 16u;
    const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) uint8_t*)lds;
    const uint32_t lds_w = lds_base + wave * 1024;
    const uint8_t* my_slab = lds + lane * 16;
    const uint8_t* cbase = reinterpret_cast<const uint8_t*>(p.acc) + (long long)c.b * p.cap * p.d * 2;
    const uint32_t row_bytes = (uint32_t)p.d * 2u;
    const int n_halves = 2 * p.n_main_slabs;

    // DMA side: lane = (row r8 of the block, slot column); block j covers the wave's tokens 8j .. 8j+7
    uint32_t xvoff[4];
    {
        const int r8 = lane >> 3, sc = lane & 7;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int piece = sc ^ ((r8 >> 1) | ((j & 1) << 2));
            const int tok = c.tile * TILE_TOKENS + wave * CHUNK_TOKENS + 8 * j + r8;
            xvoff[j] = (uint32_t)min(tok, c.len - 1) * row_bytes + (uint32_t)piece * 16u;
        }
    }
    const uint32_t stage = lds_base + LDS_DENSE_STAGE_OFF + wave * LDS_DENSE_STAGE_BYTES;
    // fragment side: this lane's token tl, k-step kk of the half slab -> piece 2 kk + half
    const uint8_t* my_stage = lds + LDS_DENSE_STAGE_OFF + wave * LDS_DENSE_STAGE_BYTES + (tl >> 3) * 1024 + (tl & 7) * 128;
    const int fx = ((tl & 7) >> 1) | (((tl >> 3) & 1) << 2);
    auto issue_x = [&](int h) {                           // token rows of half slab h -> staging
        const int hc = min(h, n_halves - 1);              // (past the end: a harmless repeat)
        const uint8_t* src = cbase + (long long)hc * 128;
#pragma unroll
        for (int j = 0; j < 4; ++j) dma_b128(src, xvoff[j], stage + j * 1024);
    };
    auto take_x = [&](uint4 (&dst)[4]) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            dst[kk] = *reinterpret_cast<const uint4*>(my_stage + (((2 * kk + half) ^ fx) * 16));
    };

    f32x16 acc[8];
#pragma unroll
    for (int nb = 0; nb < 8; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[nb][i] = 0.0f;

    uint4 af[8];                         // weight fragments, ring over slots (loaded 7 slots ahead)
    uint4 bd[2][4];                      // token fragments of the two halves of a slab

    issue_slab(wsrc, lds_w, dma_voff);
    issue_x(0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    take_x(bd[0]);
#pragma unroll
    for (int sl = 0; sl < 7; ++sl) af[sl] = *reinterpret_cast<const uint4*>(my_slab + sl * 1024);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // staging has been read: it may be refilled
    issue_x(1);

    for (int it = 0; it < p.n_main_slabs; ++it) {
        const bool more_main = it + 1 < p.n_main_slabs;
        const int s_next = more_main ? it + 1 : it;       // (the last iteration repeats itself into unused buffers)
        const uint32_t wdst = lds_w + (uint32_t)(((it + 1) & 1) * SLAB_BYTES);
        const uint8_t* wnext = wsrc + (long long)s_next * SLAB_BYTES;
        const uint8_t* slab = my_slab + (it & 1) * SLAB_BYTES;
        const uint8_t* slab_next = my_slab + ((it + 1) & 1) * SLAB_BYTES;
        __builtin_amdgcn_sched_barrier(0);
        static_for<0, 64>([&](auto SIDX) XQ_INLINE_LAMBDA {
            constexpr int sidx = decltype(SIDX)::value;
            constexpr int ks = sidx >> 3, m = sidx & 7;
            constexpr int hs = sidx & 31, hf = sidx >> 5;            // slot inside the half slab, which half
            acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                __builtin_bit_cast(bf16x8, af[m]), __builtin_bit_cast(bf16x8, bd[hf][ks & 3]), acc[m], 0, 0, 0);
            // next slab's weights: 4 DMA steps per half slab, one every other slot
            if constexpr (hs < 8 && (hs & 1) == 0)
                dma_b128(wnext + (hf * 4 + (hs >> 1)) * 8192, dma_voff, wdst + (hf * 4 + (hs >> 1)) * 8192);
            // token rows: outstanding behind the DMA of the next half are this half's 4 weight steps
            if constexpr (hs == 16) {
                asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
                take_x(bd[hf ^ 1]);
            }
            if constexpr (hs == 20) {
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                issue_x(2 * it + hf + 2);
            }
            // the next slab's weights have landed for everyone (its buffer was last read one slab
            // ago); the newest 4 DMAs, the token rows just issued, may still be in flight
            if constexpr (ks == SLAB_KSTEPS - 1 && m == 1) {
                asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
                __syncthreads();
            }
            if constexpr (sidx + 7 < 64) af[(sidx + 7) & 7] = *reinterpret_cast<const uint4*>(slab + (sidx + 7) * 1024);
            else if (more_main) af[(sidx + 7) & 7] = *reinterpret_cast<const uint4*>(slab_next + (sidx + 7 - 64) * 1024);
            __builtin_amdgcn_sched_barrier(0);
        });
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // nothing may still be writing this workgroup's LDS
    if constexpr (DMODE == DENSE_PREFILL) {
        __syncthreads();                                  // ... including the other waves' staging copies
        prefill_epilogue(p, c, acc, lds);
    } else if constexpr (DMODE == DENSE_STORE) {
        if (c.tok < c.len) {
            float* row = p.kv_out + (((long long)c.b * p.pc_blocks_cap + c.tok) * p.grid_heads + c.hk) * 256 + c.half * 4;
#pragma unroll
            for (int nb = 0; nb < 8; ++nb)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    float4 v = {0.0f, 0.0f, 0.0f, 0.0f};
                    if (p.store_add) v = *reinterpret_cast<const float4*>(row + nb * 32 + i4 * 8);
                    v.x = __builtin_fmaf(p.store_scale, acc[nb][i4 * 4], v.x);
                    v.y = __builtin_fmaf(p.store_scale, acc[nb][i4 * 4 + 1], v.y);
                    v.z = __builtin_fmaf(p.store_scale, acc[nb][i4 * 4 + 2], v.z);
                    v.w = __builtin_fmaf(p.store_scale, acc[nb][i4 * 4 + 3], v.w);
                    *reinterpret_cast<float4*>(row + nb * 32 + i4 * 8) = v;
                }
        }
    } else if constexpr (DMODE == DENSE_SCORES) {
        scores_epilogue(p, c, acc);
    } else {
        attention_epilogue(p, c, acc);
    }
}

// ---- pre-pass of the coded kernel: effective scales e = 2^(bits+14) * scale (1 for a zero scale)
// as bf16, laid out [sequence][tile][group (+1 pad)][256 tokens] so that a tile's scales of
// one group are contiguous (tokens past len repeat the last row).
__global__ __launch_bounds__(256) void scale_transpose_kernel(const uint16_t* __restrict__ scale,
                                                              uint16_t* __restrict__ eT, int cap, int ng,
                                                              int ng_row, int tiles_per_seq, int bits, BatchI32 len)
{
    const int tile = blockIdx.x, b = blockIdx.y, t = threadIdx.x;
    const int L = len.v[b];
    if (tile * TILE_TOKENS >= L) return;
    const long long row = (long long)b * cap + min(tile * TILE_TOKENS + t, L - 1);
    uint16_t* dst = eT + ((long long)b * tiles_per_seq + tile) * (long long)(ng + 1) * TILE_TOKENS + t;
    for (int g = 0; g < ng; ++g) {
        const uint32_t sb = scale[row * ng_row + g];
        const uint32_t e = sb ? sb + ((uint32_t)(bits + F16_SUBNORMAL_EXP - F16_MANT_BITS) << 7) : 0x3F80u;
        dst[(long long)g * TILE_TOKENS] = (uint16_t)e;
    }
    dst[(long long)ng * TILE_TOKENS] = 0x3F80u;       // pad group (fetched, never used)
}

// ---- split-context combine: out[b][h][:] = sum_c w_c o_c / sum_c w_c l_c, w_c = 2^(m_c - M).
// One workgroup per (sequence, query head): COMBINE_GROUPS groups of 128 threads (one per output
// column) each take every COMBINE_GROUPS-th chunk, so the loads of a group's chunks are
// independent and overlap; the groups' sums are added in fixed order (deterministic result).
constexpr int COMBINE_GROUPS = 8;
__global__ __launch_bounds__(128 * COMBINE_GROUPS) void combine_kernel(const float* __restrict__ part_o,
                                                                       const float* __restrict__ part_ml,
                                                                       float* __restrict__ out, int Hq,
                                                                       int chunks_per_seq, BatchI32 len, int rows_per_seq,
                                                                       int chunk_tokens)
{
    __shared__ float sm[COMBINE_GROUPS];
    __shared__ float sl[COMBINE_GROUPS];
    __shared__ float so[COMBINE_GROUPS][128];
    const int h = blockIdx.x, b = blockIdx.y, n = threadIdx.x & 127, grp = threadIdx.x >> 7;
    // b runs over sequences x rows_per_seq (the queries of a prefill chunk; 1 at decode)
    const int nchunks = (len.v[b / rows_per_seq] + chunk_tokens - 1) / chunk_tokens;
    const long long base = ((long long)b * Hq + h) * chunks_per_seq;
    float m_g = -INFINITY;
    for (int c = grp; c < nchunks; c += COMBINE_GROUPS) m_g = fmaxf(m_g, part_ml[(base + c) * 2]);
    if (n == 0) sm[grp] = m_g;
    __syncthreads();
    float M = sm[0];
#pragma unroll
    for (int g = 1; g < COMBINE_GROUPS; ++g) M = fmaxf(M, sm[g]);
    float L = 0.0f, o = 0.0f;
#pragma unroll 4
    for (int c = grp; c < nchunks; c += COMBINE_GROUPS) {
        const float w = __builtin_amdgcn_exp2f(part_ml[(base + c) * 2] - M);
        L = __builtin_fmaf(w, part_ml[(base + c) * 2 + 1], L);
        o = __builtin_fmaf(w, part_o[(base + c) * 128 + n], o);
    }
    so[grp][n] = o;
    if (n == 0) sl[grp] = L;
    __syncthreads();
    if (grp == 0) {
        float Lt = sl[0], ot = so[0][n];
#pragma unroll
        for (int g = 1; g < COMBINE_GROUPS; ++g) { Lt += sl[g]; ot += so[g][n]; }
        out[((long long)b * Hq + h) * 128 + n] = ot / Lt;
    }
}

template <typename K>
static hipError_t launch_with_lds(K kernel, int lds_bytes, const RematParams& p, int grid, hipStream_t s)
{
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    kernel<<<dim3(grid), dim3(512), lds_bytes, s>>>(p);
    return hipGetLastError();
}

size_t remat_workspace_bytes(int B, int Hq, int max_len, int d, int group, bool coded)
{
    const size_t tiles = ((size_t)max_len + TILE_TOKENS - 1) / TILE_TOKENS;
    const size_t chunks = tiles * (TILE_TOKENS / CHUNK_TOKENS);
    size_t bytes = (size_t)B * Hq * chunks * (128 + 2) * sizeof(float);
    if (coded) {
        bytes += (size_t)B * tiles * (size_t)(d / group + 1) * TILE_TOKENS * sizeof(uint16_t);   // eT
    }
    return bytes;
}

// latent cache of rank r: partials, effective scales of the K half and of the V half, scores
size_t remat_latent_workspace_bytes(int B, int Hq, int max_len, int r, int group)
{
    const size_t tiles = ((size_t)max_len + TILE_TOKENS - 1) / TILE_TOKENS;
    return remat_workspace_bytes(B, Hq, max_len, r, group, true) +
           (size_t)B * tiles * (size_t)(r / group + 1) * TILE_TOKENS * sizeof(uint16_t) +
           (size_t)B * Hq * tiles * TILE_TOKENS * sizeof(float);
}

// the prefill epilogue lays its own images over the whole LDS once the contraction is done
template <int MODE>
constexpr int lds_for_mode(int bits)
{
    return MODE == MODE_PREFILL && LDS_PREFILL_TOTAL > lds_coded_total(bits) ? LDS_PREFILL_TOTAL : lds_coded_total(bits);
}

template <int MODE>
static hipError_t launch_coded(int bits, int G, const RematParams& p, int grid, hipStream_t s)
{
    switch (bits * 1000 + G) {
        case 2064: return launch_with_lds(remat_attn_coded_kernel<2, 64, MODE>, lds_for_mode<MODE>(2), p, grid, s);
        case 2128: return launch_with_lds(remat_attn_coded_kernel<2, 128, MODE>, lds_for_mode<MODE>(2), p, grid, s);
        case 3064: return launch_with_lds(remat_attn_coded_kernel<3, 64, MODE>, lds_for_mode<MODE>(3), p, grid, s);
        case 3128: return launch_with_lds(remat_attn_coded_kernel<3, 128, MODE>, lds_for_mode<MODE>(3), p, grid, s);
        case 4064: return launch_with_lds(remat_attn_coded_kernel<4, 64, MODE>, lds_for_mode<MODE>(4), p, grid, s);
        case 4128: return launch_with_lds(remat_attn_coded_kernel<4, 128, MODE>, lds_for_mode<MODE>(4), p, grid, s);
    }
    return hipErrorInvalidValue;
}

static void fill_common(RematParams& p, const xq_attn_t* a, const uint16_t* q, int B, int cap, const BatchI32& len,
                        int max_len, void* ws)
{
    p.q = q;
    p.B = B; p.cap = cap; p.Hq = a->n_q_heads; p.Hkv = a->n_kv_heads;
    p.tiles_per_seq = (max_len + TILE_TOKENS - 1) / TILE_TOKENS;
    p.chunks_per_seq = p.tiles_per_seq * (TILE_TOKENS / CHUNK_TOKENS);
    p.scale_log2e = a->softmax_scale * 1.44269504088896340736f;
    p.len = len;
    p.part_o = static_cast<float*>(ws);
    p.part_ml = p.part_o + (size_t)B * p.Hq * p.chunks_per_seq * 128;
}

hipError_t run_remat_attn_prefill(const xq_attn_t* a, const uint16_t* q, int T, const xq_cache_t* xc,
                                  const uint16_t* acc, int B, int cap, int d, const void* wprep,
                                  const BatchI32& len, int max_len, float* out, void* ws,
                                  const float* rope, const BatchI32* pos0, hipStream_t s);

// query heads per KV head from which the decode step goes through the matrix-core epilogue (the
// per-query-head vector epilogue runs that many times per tile; measured break-even is about 4)
constexpr int DECODE_MFMA_EPILOGUE_MIN_GROUP = 4;

hipError_t run_remat_attn_decode(const xq_attn_t* a, const uint16_t* q, const xq_cache_t* xc,
                                 const uint16_t* acc, int B, int cap, int d, const void* wprep,
                                 const BatchI32& len, int max_len, float* out, void* ws,
                                 const float* rope, const BatchI32* pos0, hipStream_t s)
{
    if (a->n_q_heads / a->n_kv_heads >= DECODE_MFMA_EPILOGUE_MIN_GROUP)     // same layouts and workspace at T = 1
        return run_remat_attn_prefill(a, q, 1, xc, acc, B, cap, d, wprep, len, max_len, out, ws, rope, pos0, s);
    const int bits = xc ? xc->fmt.bits : 16;
    const int G = xc ? xc->fmt.group : 128;
    const WPrepLayout L = make_wprep_layout(d, G, bits, a->n_kv_heads);
    RematParams p{};
    fill_common(p, a, q, B, cap, len, max_len, ws);
    p.codes = xc ? xc->codes : nullptr;
    p.zero = xc ? xc->zero : nullptr;
    p.acc = acc;
    p.wprep = static_cast<const uint8_t*>(wprep);
    p.d = d; p.row_d = d; p.grid_heads = p.Hkv;
    p.n_main_slabs = L.n_main_slabs; p.n_corr_ksteps = L.n_corr_ksteps; p.ng = L.ng; p.ng_pad = L.ng_pad;
    p.ng_row = L.ng;
    p.head_bytes = (long long)L.head_bytes;
    p.rope = rope;
    if (rope) p.pos0 = *pos0;
    uint16_t* eT = reinterpret_cast<uint16_t*>(p.part_ml + (size_t)B * p.Hq * p.chunks_per_seq * 2);
    p.eT = eT;

    const int grid = p.Hkv * p.B * p.tiles_per_seq;
    hipError_t e = hipErrorInvalidValue;
    if (xc) {
        scale_transpose_kernel<<<dim3(p.tiles_per_seq, B), dim3(TILE_TOKENS), 0, s>>>(
            xc->scale, eT, cap, L.ng, L.ng, p.tiles_per_seq, bits, len);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        e = launch_coded<MODE_ATTENTION>(bits, G, p, grid, s);
    } else {
        e = launch_with_lds(remat_attn_dense_kernel<DENSE_ATTENTION>, LDS_DENSE_TOTAL, p, grid, s);
    }
    if (e != hipSuccess) return e;
    combine_kernel<<<dim3(p.Hq, p.B), dim3(128 * COMBINE_GROUPS), 0, s>>>(p.part_o, p.part_ml, out, p.Hq, p.chunks_per_seq, p.len, 1, CHUNK_TOKENS);
    return hipGetLastError();
}

// Causal attention of the T newest tokens of every sequence (chunked prefill): the decode launch
// with T query rows per sequence in the partial buffers and the matrix-core epilogue.
size_t remat_prefill_workspace_bytes(int B, int T, int Hq, int max_len, int d, int group, bool coded)
{
    const size_t tiles = ((size_t)max_len + TILE_TOKENS - 1) / TILE_TOKENS;
    size_t bytes = ((size_t)B * T * Hq * tiles + 7) / 8 * 8 * (128 + 2) * sizeof(float);    // one partial per tile
    if (coded) bytes += (size_t)B * tiles * (size_t)(d / group + 1) * TILE_TOKENS * sizeof(uint16_t);
    return bytes;
}

hipError_t run_remat_attn_prefill(const xq_attn_t* a, const uint16_t* q, int T, const xq_cache_t* xc,
                                  const uint16_t* acc, int B, int cap, int d, const void* wprep,
                                  const BatchI32& len, int max_len, float* out, void* ws,
                                  const float* rope, const BatchI32* pos0, hipStream_t s)
{
    const int bits = xc ? xc->fmt.bits : 16;
    const int G = xc ? xc->fmt.group : 128;
    const WPrepLayout L = make_wprep_layout(d, G, bits, a->n_kv_heads);
    RematParams p{};
    p.q = q; p.Tq = T;
    p.B = B; p.cap = cap; p.Hq = a->n_q_heads; p.Hkv = a->n_kv_heads;
    p.tiles_per_seq = (max_len + TILE_TOKENS - 1) / TILE_TOKENS;
    p.chunks_per_seq = p.tiles_per_seq;                  // the epilogue merges a tile's chunks: one partial per tile
    p.scale_log2e = a->softmax_scale * 1.44269504088896340736f;
    p.len = len;
    const size_t rows = ((size_t)B * T * p.Hq * p.tiles_per_seq + 7) / 8 * 8;   // (keeps the scale copy 16-byte aligned)
    p.part_o = static_cast<float*>(ws);
    p.part_ml = p.part_o + rows * 128;
    p.eT = reinterpret_cast<uint16_t*>(p.part_ml + rows * 2);
    p.codes = xc ? xc->codes : nullptr;
    p.zero = xc ? xc->zero : nullptr;
    p.acc = acc;
    p.wprep = static_cast<const uint8_t*>(wprep);
    p.d = d; p.row_d = d; p.grid_heads = p.Hkv;
    p.n_main_slabs = L.n_main_slabs; p.n_corr_ksteps = L.n_corr_ksteps; p.ng = L.ng; p.ng_pad = L.ng_pad;
    p.ng_row = L.ng;
    p.head_bytes = (long long)L.head_bytes;
    p.rope = rope;
    if (rope) p.pos0 = *pos0;
    const int grid = p.Hkv * p.B * p.tiles_per_seq;
    hipError_t e;
    if (xc) {
        scale_transpose_kernel<<<dim3(p.tiles_per_seq, B), dim3(TILE_TOKENS), 0, s>>>(
            xc->scale, const_cast<uint16_t*>(p.eT), cap, L.ng, L.ng, p.tiles_per_seq, bits, len);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        e = launch_coded<MODE_PREFILL>(bits, G, p, grid, s);
    } else {
        e = launch_with_lds(remat_attn_dense_kernel<DENSE_PREFILL>, LDS_DENSE_TOTAL, p, grid, s);
    }
    if (e != hipSuccess) return e;
    combine_kernel<<<dim3(p.Hq, p.B * T), dim3(128 * COMBINE_GROUPS), 0, s>>>(p.part_o, p.part_ml, out, p.Hq,
                                                                            p.chunks_per_seq, p.len, T, TILE_TOKENS);
    return hipGetLastError();
}

// Latent cache [X Uk | X Uv] of rank r (Sec. 3.3.1): two passes of the same contraction kernel over
// the two halves of the cache rows, each with all 256 columns in use -- pass 1 rematerialises the
// keys of a pair of KV heads from the first r channels and stores the scaled scores, pass 2 the
// values of the pair from the last r channels and turns scores into softmax partials.
hipError_t run_remat_attn_decode_latent(const xq_attn_t* a, const uint16_t* q, const xq_cache_t* xc,
                                        const void* wprep, const BatchI32& len, int max_len, float* out, void* ws,
                                        hipStream_t s)
{
    const int bits = xc->fmt.bits, G = xc->fmt.group, r = xc->fmt.d / 2, B = xc->B, cap = xc->cap;
    const int pairs = a->n_kv_heads / 2;
    const WPrepLayout L = make_wprep_layout(r, G, bits, pairs);          // one stream per half, "head" = pair
    RematParams p{};
    fill_common(p, a, q, B, cap, len, max_len, ws);
    p.d = r; p.row_d = 2 * r; p.grid_heads = pairs;
    p.n_main_slabs = L.n_main_slabs; p.n_corr_ksteps = L.n_corr_ksteps; p.ng = L.ng; p.ng_pad = L.ng_pad;
    p.ng_row = 2 * L.ng;
    p.head_bytes = (long long)L.head_bytes;
    const size_t et_elems = (size_t)B * p.tiles_per_seq * (size_t)(L.ng + 1) * TILE_TOKENS;
    uint16_t* eT_k = reinterpret_cast<uint16_t*>(p.part_ml + (size_t)B * p.Hq * p.chunks_per_seq * 2);
    uint16_t* eT_v = eT_k + et_elems;
    p.scores = reinterpret_cast<float*>(eT_v + et_elems);
    p.score_stride = p.tiles_per_seq * TILE_TOKENS;
    const int grid = pairs * B * p.tiles_per_seq;

    scale_transpose_kernel<<<dim3(p.tiles_per_seq, B), dim3(TILE_TOKENS), 0, s>>>(
        xc->scale, eT_k, cap, L.ng, 2 * L.ng, p.tiles_per_seq, bits, len);
    scale_transpose_kernel<<<dim3(p.tiles_per_seq, B), dim3(TILE_TOKENS), 0, s>>>(
        xc->scale + L.ng, eT_v, cap, L.ng, 2 * L.ng, p.tiles_per_seq, bits, len);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // pass 1: keys
    p.codes = xc->codes; p.zero = xc->zero; p.eT = eT_k;
    p.wprep = static_cast<const uint8_t*>(wprep);
    e = launch_coded<MODE_SCORES>(bits, G, p, grid, s);
    if (e != hipSuccess) return e;
    // pass 2: values
    p.codes = xc->codes + (size_t)r * bits / 8; p.zero = xc->zero + L.ng; p.eT = eT_v;
    p.wprep = static_cast<const uint8_t*>(wprep) + L.total_bytes;
    e = launch_coded<MODE_WEIGHTED_SUM>(bits, G, p, grid, s);
    if (e != hipSuccess) return e;
    combine_kernel<<<dim3(p.Hq, p.B), dim3(128 * COMBINE_GROUPS), 0, s>>>(p.part_o, p.part_ml, out, p.Hq, p.chunks_per_seq, p.len, 1, CHUNK_TOKENS);
    return hipGetLastError();
}

// Sec. 3.3.2: acc[b][t][:] += dequant(latent delta cache row) U_kv^T for t < len[b], with the
// contraction kernel laid over d / 256 column blocks of the hidden size.  ws holds the effective
// scales only.
size_t upproject_workspace_bytes(int B, int max_len, int n_lat, int group)
{
    const size_t tiles = ((size_t)max_len + TILE_TOKENS - 1) / TILE_TOKENS;
    return (size_t)B * tiles * (size_t)(n_lat / group + 1) * TILE_TOKENS * sizeof(uint16_t);
}

hipError_t run_cl_accumulate_latent(uint16_t* acc, const xq_cache_t* xc, int d, const void* uprep,
                                    const BatchI32& len, int max_len, void* ws, hipStream_t s)
{
    const int bits = xc->fmt.bits, G = xc->fmt.group, n_lat = xc->fmt.d, B = xc->B;
    const int blocks = d / 256;
    const WPrepLayout L = make_wprep_layout(n_lat, G, bits, blocks);
    RematParams p{};
    p.B = B; p.cap = xc->cap; p.Hq = p.Hkv = blocks; p.grid_heads = blocks;
    p.tiles_per_seq = (max_len + TILE_TOKENS - 1) / TILE_TOKENS;
    p.chunks_per_seq = p.tiles_per_seq * (TILE_TOKENS / CHUNK_TOKENS);
    p.len = len;
    p.codes = xc->codes; p.zero = xc->zero;
    p.wprep = static_cast<const uint8_t*>(uprep);
    p.d = n_lat; p.row_d = n_lat;
    p.n_main_slabs = L.n_main_slabs; p.n_corr_ksteps = L.n_corr_ksteps; p.ng = L.ng; p.ng_pad = L.ng_pad;
    p.ng_row = L.ng;
    p.head_bytes = (long long)L.head_bytes;
    p.eT = static_cast<uint16_t*>(ws);
    p.acc_out = acc; p.d_out = d;
    scale_transpose_kernel<<<dim3(p.tiles_per_seq, B), dim3(TILE_TOKENS), 0, s>>>(
        xc->scale, static_cast<uint16_t*>(ws), xc->cap, L.ng, L.ng, p.tiles_per_seq, bits, len);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_coded<MODE_ACCUMULATE>(bits, G, p, blocks * B * p.tiles_per_seq, s);
}

// ---- per-channel cache (Sec. 3.3.1) ----------------------------------------------------------
// Pre-pass 1: per block, E = exponent with max_c scale < 2^E, and the block's final factor
// 2^(E + bits - 1) (the operand factors are scale * 2^(15 - E), the prepared weights carry 2^(-14 - bits)
// relative to the code bits).  One workgroup per (block, sequence).
__global__ __launch_bounds__(256) void pc_block_exponent_kernel(const uint16_t* __restrict__ scale, float* __restrict__ fscale,
                                                                int* __restrict__ eblk, int d, int blocks_cap,
                                                                int blocks_ws, int bits, BatchI32 nblk)
{
    __shared__ uint32_t red[256];
    const int blk = blockIdx.x, b = blockIdx.y;
    if (blk >= nblk.v[b]) return;
    const uint16_t* row = scale + ((long long)b * blocks_cap + blk) * d;
    uint32_t mx = 0;
    for (int c = threadIdx.x; c < d; c += 256) mx = max(mx, (uint32_t)row[c]);    // non-negative bf16: ordered as integers
    red[threadIdx.x] = mx;
    __syncthreads();
    for (int st = 128; st > 0; st >>= 1) {
        if ((int)threadIdx.x < st) red[threadIdx.x] = max(red[threadIdx.x], red[threadIdx.x + st]);
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const int e8 = (int)(red[0] >> 7);                                          // biased exponent of the largest scale
        const int E = red[0] ? e8 - 126 : 0;                                        // largest scale < 2^E
        eblk[(long long)b * blocks_ws + blk] = E;                                   // (workspace rows per sequence)
        fscale[(long long)b * blocks_ws + blk] = ldexpf(1.0f, E + bits - 1);
    }
}

// Pre-pass 2: the factor images, [sequence][tile][slab (+1 pad)][block of the tile][k-step][lane half][8] fp16, in
// the order the unpacked operand dwords hold their channels (the unpack table gives the code of each slot).
// Blocks past the sequence's last one repeat it (their tokens are masked, but must stay finite).
struct PcImageArgs {
    const uint16_t* scale;
    const int* eblk;
    uint16_t* img;
    int d, blocks_cap, blocks_ws, block, tiles_per_seq, n_slabs, G;   // blocks per sequence in the cache / in eblk
    BatchI32 nblk;
    UnpackTable tab;
};
__global__ __launch_bounds__(256) void pc_factor_image_kernel(PcImageArgs a)
{
    const int slab = blockIdx.x, tile = blockIdx.y, b = blockIdx.z;
    const int bpt = TILE_TOKENS / a.block;                       // blocks per tile
    if (tile * bpt >= a.nblk.v[b]) return;
    uint16_t* out = a.img + (((long long)b * a.tiles_per_seq + tile) * (a.n_slabs + 1) + slab) * (LDS_SCALES_BYTES / 2);
    const int ksg_n = a.G / 16;
    for (int e = threadIdx.x; e < bpt * 128; e += 256) {
        const int i = e & 7, half = (e >> 3) & 1, ks = (e >> 4) & 7, bt = e >> 7;
        const int blk = min(tile * bpt + bt, a.nblk.v[b] - 1);
        const int gi = ks / ksg_n, ksg = ks % ksg_n;
        const int c = slab * 128 + gi * a.G + half * (a.G / 2) + (ksg >> 2) * 32 + a.tab.code_of_slot[ksg & 3][i];
        const float sc = bf16_bits_to_f32(a.scale[((long long)b * a.blocks_cap + blk) * a.d + c]);
        const float f = ldexpf(sc, 15 - a.eblk[(long long)b * a.blocks_ws + blk]);
        out[e] = __builtin_bit_cast(uint16_t, (_Float16)f);
    }
}

bool unpack_table_for(int bits, UnpackTable* t);

size_t remat_pc_workspace_bytes(int B, int Hq, int Hkv, int max_len, int d, int block)
{
    const size_t tiles = ((size_t)max_len + TILE_TOKENS - 1) / TILE_TOKENS;
    const size_t chunks = (tiles + 1) * (TILE_TOKENS / CHUNK_TOKENS);
    const size_t blocks = (size_t)max_len / block + 1;
    return (size_t)B * Hq * chunks * (128 + 2) * sizeof(float)                    // partials
         + (size_t)B * tiles * (size_t)(d / 128 + 1) * LDS_SCALES_BYTES           // factor images
         + (size_t)B * blocks * (size_t)Hkv * 256 * sizeof(float)                 // z W rows
         + (size_t)B * blocks * 2 * sizeof(float) + 256;                          // block factors and exponents
}

// Decode attention from a per-channel cache plus the bf16 residual window of the newest len % block tokens.
hipError_t run_remat_attn_decode_pc(const xq_attn_t* a, const uint16_t* q, const xq_cache_t* xc, const uint16_t* tail,
                                    const void* wprep_coded, const void* wprep_dense, const BatchI32& len, int max_len,
                                    float* out, void* ws, hipStream_t s)
{
    const int bits = xc->fmt.bits, blockT = xc->fmt.group, d = xc->fmt.d, B = xc->B, cap = xc->cap;
    const int blocks_cap = cap / blockT;
    const WPrepLayout Lc = make_wprep_layout(d, 128, bits, a->n_kv_heads);
    const WPrepLayout Ld = make_wprep_layout(d, 128, 16, a->n_kv_heads);
    UnpackTable tab;
    if (!unpack_table_for(bits, &tab)) return hipErrorInvalidValue;
    BatchI32 nblk{}, len_coded{}, len_tail{}, chunk0{};
    int max_coded = 0, max_nblk = 0, any_tail = 0;
    for (int b = 0; b < B; ++b) {
        nblk.v[b] = len.v[b] / blockT;
        len_coded.v[b] = nblk.v[b] * blockT;
        len_tail.v[b] = len.v[b] - len_coded.v[b];
        chunk0.v[b] = len_coded.v[b] / CHUNK_TOKENS;
        max_coded = len_coded.v[b] > max_coded ? len_coded.v[b] : max_coded;
        max_nblk = nblk.v[b] > max_nblk ? nblk.v[b] : max_nblk;
        any_tail |= len_tail.v[b];
    }
    const int tiles_all = (max_len + TILE_TOKENS - 1) / TILE_TOKENS;
    const int tiles_coded = (max_coded + TILE_TOKENS - 1) / TILE_TOKENS;
    const int chunks_stride = (tiles_all + 1) * (TILE_TOKENS / CHUNK_TOKENS);
    // workspace carve-up (sizes as in remat_pc_workspace_bytes)
    float* part_o = static_cast<float*>(ws);
    float* part_ml = part_o + (size_t)B * a->n_q_heads * chunks_stride * 128;
    uint8_t* img = reinterpret_cast<uint8_t*>(part_ml + (size_t)B * a->n_q_heads * chunks_stride * 2);
    float* zw = reinterpret_cast<float*>(img + (size_t)B * tiles_all * (size_t)(d / 128 + 1) * LDS_SCALES_BYTES);
    const size_t blocks_ws = (size_t)max_len / blockT + 1;
    float* fscale = zw + (size_t)B * blocks_ws * a->n_kv_heads * 256;
    int* eblk = reinterpret_cast<int*>(fscale + (size_t)B * blocks_ws);

    RematParams p{};
    p.q = q;
    p.B = B; p.Hq = a->n_q_heads; p.Hkv = a->n_kv_heads; p.grid_heads = p.Hkv;
    p.scale_log2e = a->softmax_scale * 1.44269504088896340736f;
    p.part_o = part_o; p.part_ml = part_ml; p.chunks_per_seq = chunks_stride;
    p.d = d; p.row_d = d;
    hipError_t e = hipSuccess;
    if (max_nblk > 0) {
        // block exponents, factor images
        pc_block_exponent_kernel<<<dim3(max_nblk, B), dim3(256), 0, s>>>(xc->scale, fscale, eblk, d, blocks_cap, (int)blocks_ws, bits, nblk);
        PcImageArgs ia{xc->scale, eblk, reinterpret_cast<uint16_t*>(img), d, blocks_cap, (int)blocks_ws, blockT, tiles_coded, Lc.n_main_slabs, 128,
                       nblk, tab};
        pc_factor_image_kernel<<<dim3(Lc.n_main_slabs, tiles_coded, B), dim3(256), 0, s>>>(ia);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        // z_blk [Wk | Wv]: the dense contraction over the zero-point rows, stored
        RematParams z = p;
        z.acc = xc->zero; z.cap = blocks_cap; z.len = nblk;                  // source rows: one per block
        z.tiles_per_seq = (max_nblk + TILE_TOKENS - 1) / TILE_TOKENS;
        z.wprep = static_cast<const uint8_t*>(wprep_dense);
        z.n_main_slabs = Ld.n_main_slabs; z.head_bytes = (long long)Ld.head_bytes;
        z.kv_out = zw; z.pc_blocks_cap = (int)blocks_ws;                     // destination rows per sequence
        z.store_scale = 1.0f; z.store_add = 0;
        e = launch_with_lds(remat_attn_dense_kernel<DENSE_STORE>, LDS_DENSE_TOTAL, z, p.Hkv * B * z.tiles_per_seq, s);
        if (e == hipSuccess && bits == 4) {                                  // + 8 s_blk [Wk | Wv]: the codes enter as code - 8
            z.acc = xc->scale; z.store_scale = 8.0f; z.store_add = 1;
            e = launch_with_lds(remat_attn_dense_kernel<DENSE_STORE>, LDS_DENSE_TOTAL, z, p.Hkv * B * z.tiles_per_seq, s);
        }
        if (e != hipSuccess) return e;
        // the coded blocks
        RematParams m = p;
        m.codes = xc->codes; m.eT = reinterpret_cast<const uint16_t*>(img);
        m.cap = cap; m.len = len_coded; m.tiles_per_seq = tiles_coded;
        m.wprep = static_cast<const uint8_t*>(wprep_coded);
        m.n_main_slabs = Lc.n_main_slabs; m.n_corr_ksteps = Lc.n_corr_ksteps; m.ng = Lc.ng; m.ng_pad = Lc.ng_pad; m.ng_row = Lc.ng;
        m.head_bytes = (long long)Lc.head_bytes;
        m.pc_fscale = fscale; m.pc_zw = zw; m.pc_block = blockT; m.pc_blocks_cap = (int)blocks_ws;
        const int grid = p.Hkv * B * tiles_coded;
        switch (bits) {
            case 2: e = launch_with_lds(remat_attn_coded_kernel<2, 128, MODE_ATTENTION_PC>, lds_coded_total(2), m, grid, s); break;
            case 3: e = launch_with_lds(remat_attn_coded_kernel<3, 128, MODE_ATTENTION_PC>, lds_coded_total(3), m, grid, s); break;
            case 4: e = launch_with_lds(remat_attn_coded_kernel<4, 128, MODE_ATTENTION_PC>, lds_coded_total(4), m, grid, s); break;
            default: e = hipErrorInvalidValue;
        }
        if (e != hipSuccess) return e;
    }
    if (any_tail) {
        // the residual window: bf16 rows, dense-source kernel, partial chunks placed after the coded ones
        RematParams t = p;
        t.acc = tail; t.cap = blockT; t.len = len_tail; t.tiles_per_seq = 1; t.chunk0 = chunk0;
        t.wprep = static_cast<const uint8_t*>(wprep_dense);
        t.n_main_slabs = Ld.n_main_slabs; t.head_bytes = (long long)Ld.head_bytes;
        e = launch_with_lds(remat_attn_dense_kernel<DENSE_ATTENTION>, LDS_DENSE_TOTAL, t, p.Hkv * B, s);
        if (e != hipSuccess) return e;
    }
    combine_kernel<<<dim3(p.Hq, B), dim3(128 * COMBINE_GROUPS), 0, s>>>(part_o, part_ml, out, p.Hq, chunks_stride, len, 1,
                                                                      CHUNK_TOKENS);
    return hipGetLastError();
}

// ---- the paper's setting for grouped-query models (Sec. 3.3.1): X Uk per channel with a residual
// window, X Uv per token.  Two passes as in run_remat_attn_decode_latent: pass 1 rematerialises the keys of a
// head pair from the per-channel K cache (coded blocks, then the window rows through the dense kernel) and
// stores the scaled scores; pass 2 is the unchanged value pass over the per-token V cache.
size_t remat_latent_pc_workspace_bytes(int B, int Hq, int Hkv, int max_len, int r, int block, int v_group)
{
    const size_t tiles = ((size_t)max_len + TILE_TOKENS - 1) / TILE_TOKENS;
    const size_t chunks = tiles * (TILE_TOKENS / CHUNK_TOKENS);
    const size_t blocks = (size_t)max_len / block + 1;
    return (size_t)B * Hq * chunks * (128 + 2) * sizeof(float)                          // partials
         + (size_t)B * Hq * (tiles + 1) * TILE_TOKENS * sizeof(float)                   // scores
         + (size_t)B * tiles * (size_t)(r / 128 + 1) * LDS_SCALES_BYTES                 // K factor images
         + (size_t)B * blocks * (size_t)(Hkv / 2) * 256 * sizeof(float)                 // z W rows of the head pairs
         + (size_t)B * tiles * (size_t)(r / v_group + 1) * TILE_TOKENS * sizeof(uint16_t)    // V effective scales
         + (size_t)B * blocks * 2 * sizeof(float) + 256;                                // block factors and exponents
}

hipError_t run_remat_attn_decode_latent_pc(const xq_attn_t* a, const uint16_t* q, const xq_cache_t* kc,
                                           const uint16_t* ktail, const xq_cache_t* vc, const void* wk_coded,
                                           const void* wk_dense, const void* wv_coded, const BatchI32& len, int max_len,
                                           float* out, void* ws, hipStream_t s)
{
    const int kbits = kc->fmt.bits, blockT = kc->fmt.group, r = kc->fmt.d, B = kc->B;
    const int vbits = vc->fmt.bits, vG = vc->fmt.group;
    const int pairs = a->n_kv_heads / 2;
    const int blocks_cap = kc->cap / blockT;
    const WPrepLayout Lk = make_wprep_layout(r, 128, kbits, pairs);
    const WPrepLayout Ld = make_wprep_layout(r, 128, 16, pairs);
    const WPrepLayout Lv = make_wprep_layout(r, vG, vbits, pairs);
    UnpackTable tab;
    if (!unpack_table_for(kbits, &tab)) return hipErrorInvalidValue;
    BatchI32 nblk{}, len_coded{}, len_tail{};
    int max_coded = 0, max_nblk = 0, any_tail = 0;
    for (int b = 0; b < B; ++b) {
        nblk.v[b] = len.v[b] / blockT;
        len_coded.v[b] = nblk.v[b] * blockT;
        len_tail.v[b] = len.v[b] - len_coded.v[b];
        max_coded = len_coded.v[b] > max_coded ? len_coded.v[b] : max_coded;
        max_nblk = nblk.v[b] > max_nblk ? nblk.v[b] : max_nblk;
        any_tail |= len_tail.v[b];
    }
    const int tiles_all = (max_len + TILE_TOKENS - 1) / TILE_TOKENS;
    const int tiles_coded = (max_coded + TILE_TOKENS - 1) / TILE_TOKENS;
    const int chunks = tiles_all * (TILE_TOKENS / CHUNK_TOKENS);
    const size_t blocks_ws = (size_t)max_len / blockT + 1;
    // workspace carve-up (sizes as in remat_latent_pc_workspace_bytes)
    float* part_o = static_cast<float*>(ws);
    float* part_ml = part_o + (size_t)B * a->n_q_heads * chunks * 128;
    float* scores = part_ml + (size_t)B * a->n_q_heads * chunks * 2;
    const int score_stride = (tiles_all + 1) * TILE_TOKENS;
    uint8_t* img = reinterpret_cast<uint8_t*>(scores + (size_t)B * a->n_q_heads * score_stride);
    float* zw = reinterpret_cast<float*>(img + (size_t)B * tiles_all * (size_t)(r / 128 + 1) * LDS_SCALES_BYTES);
    uint16_t* eT_v = reinterpret_cast<uint16_t*>(zw + (size_t)B * blocks_ws * pairs * 256);      // (16-byte aligned: a DMA source)
    float* fscale = reinterpret_cast<float*>(eT_v + (size_t)B * tiles_all * (size_t)(r / vG + 1) * TILE_TOKENS);
    int* eblk = reinterpret_cast<int*>(fscale + (size_t)B * blocks_ws);

    RematParams p{};
    p.q = q;
    p.B = B; p.Hq = a->n_q_heads; p.Hkv = a->n_kv_heads; p.grid_heads = pairs;
    p.scale_log2e = a->softmax_scale * 1.44269504088896340736f;
    p.part_o = part_o; p.part_ml = part_ml; p.chunks_per_seq = chunks;
    p.scores = scores; p.score_stride = score_stride;
    p.d = r; p.row_d = r;
    hipError_t e = hipSuccess;
    if (max_nblk > 0) {
        pc_block_exponent_kernel<<<dim3(max_nblk, B), dim3(256), 0, s>>>(kc->scale, fscale, eblk, r, blocks_cap, (int)blocks_ws, kbits, nblk);
        PcImageArgs ia{kc->scale, eblk, reinterpret_cast<uint16_t*>(img), r, blocks_cap, (int)blocks_ws, blockT, tiles_coded,
                       Lk.n_main_slabs, 128, nblk, tab};
        pc_factor_image_kernel<<<dim3(Lk.n_main_slabs, tiles_coded, B), dim3(256), 0, s>>>(ia);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        RematParams z = p;                                                   // z_blk (Sk Bk^T) of every head pair
        z.acc = kc->zero; z.cap = blocks_cap; z.len = nblk;
        z.tiles_per_seq = (max_nblk + TILE_TOKENS - 1) / TILE_TOKENS;
        z.wprep = static_cast<const uint8_t*>(wk_dense);
        z.n_main_slabs = Ld.n_main_slabs; z.head_bytes = (long long)Ld.head_bytes;
        z.kv_out = zw; z.pc_blocks_cap = (int)blocks_ws;
        z.store_scale = 1.0f; z.store_add = 0;
        e = launch_with_lds(remat_attn_dense_kernel<DENSE_STORE>, LDS_DENSE_TOTAL, z, pairs * B * z.tiles_per_seq, s);
        if (e == hipSuccess && kbits == 4) {                                 // + 8 s_blk (Sk Bk^T): the codes enter as code - 8
            z.acc = kc->scale; z.store_scale = 8.0f; z.store_add = 1;
            e = launch_with_lds(remat_attn_dense_kernel<DENSE_STORE>, LDS_DENSE_TOTAL, z, pairs * B * z.tiles_per_seq, s);
        }
        if (e != hipSuccess) return e;
        RematParams m = p;                                                   // pass 1, coded blocks
        m.codes = kc->codes; m.eT = reinterpret_cast<const uint16_t*>(img);
        m.cap = kc->cap; m.len = len_coded; m.tiles_per_seq = tiles_coded;
        m.wprep = static_cast<const uint8_t*>(wk_coded);
        m.n_main_slabs = Lk.n_main_slabs; m.n_corr_ksteps = Lk.n_corr_ksteps; m.ng = Lk.ng; m.ng_pad = Lk.ng_pad; m.ng_row = Lk.ng;
        m.head_bytes = (long long)Lk.head_bytes;
        m.pc_fscale = fscale; m.pc_zw = zw; m.pc_block = blockT; m.pc_blocks_cap = (int)blocks_ws;
        const int grid = pairs * B * tiles_coded;
        switch (kbits) {
            case 2: e = launch_with_lds(remat_attn_coded_kernel<2, 128, MODE_SCORES_PC>, lds_coded_total(2), m, grid, s); break;
            case 3: e = launch_with_lds(remat_attn_coded_kernel<3, 128, MODE_SCORES_PC>, lds_coded_total(3), m, grid, s); break;
            case 4: e = launch_with_lds(remat_attn_coded_kernel<4, 128, MODE_SCORES_PC>, lds_coded_total(4), m, grid, s); break;
            default: e = hipErrorInvalidValue;
        }
        if (e != hipSuccess) return e;
    }
    if (any_tail) {                                                          // pass 1, window rows
        RematParams t = p;
        t.acc = ktail; t.cap = blockT; t.len = len_tail; t.tiles_per_seq = 1; t.tok0 = len_coded;
        t.wprep = static_cast<const uint8_t*>(wk_dense);
        t.n_main_slabs = Ld.n_main_slabs; t.head_bytes = (long long)Ld.head_bytes;
        e = launch_with_lds(remat_attn_dense_kernel<DENSE_SCORES>, LDS_DENSE_TOTAL, t, pairs * B, s);
        if (e != hipSuccess) return e;
    }
    // pass 2: values from the per-token cache
    scale_transpose_kernel<<<dim3(tiles_all, B), dim3(TILE_TOKENS), 0, s>>>(vc->scale, eT_v, vc->cap, Lv.ng, Lv.ng, tiles_all, vbits, len);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    RematParams v = p;
    v.codes = vc->codes; v.zero = vc->zero; v.eT = eT_v;
    v.cap = vc->cap; v.len = len; v.tiles_per_seq = tiles_all;
    v.wprep = static_cast<const uint8_t*>(wv_coded);
    v.n_main_slabs = Lv.n_main_slabs; v.n_corr_ksteps = Lv.n_corr_ksteps; v.ng = Lv.ng; v.ng_pad = Lv.ng_pad; v.ng_row = Lv.ng;
    v.head_bytes = (long long)Lv.head_bytes;
    e = launch_coded<MODE_WEIGHTED_SUM>(vbits, vG, v, pairs * B * tiles_all, s);
    if (e != hipSuccess) return e;
    combine_kernel<<<dim3(p.Hq, B), dim3(128 * COMBINE_GROUPS), 0, s>>>(part_o, part_ml, out, p.Hq, chunks, len, 1, CHUNK_TOKENS);
    return hipGetLastError();
}

}  // namespace xq
