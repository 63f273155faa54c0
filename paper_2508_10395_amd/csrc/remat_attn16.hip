// Attention over a per-token X cache with groups of 128 codes (2-bit: also 64), over the complete blocks of a
// per-channel X cache, or over the bf16 cross-layer accumulator, built on v_mfma_f32_16x16x32: decode (one query row
// per head) and, through a matrix-core epilogue, prefill chunks and decode with many query heads per KV head
// (Sec. 3.1, Sec. 3.2, Sec. 3.3.1, App. A and the cost model of Sec. 3.4 in arxiv 2508.10395).  Same mathematics, same partials and the same
// workgroup shape as remat_attn_coded_kernel<BITS, 128, MODE_ATTENTION> in remat_attn.hip -- eight waves, a
// wave owns 32 tokens and all 256 columns of [Wk_h | Wv_h], codes enter the fp16 MFMA as subnormals, one
// accumulator carried through the groups by Horner rescaling, zero-points through a few bf16 k-steps -- but
// the 32 x 256 block of a wave is cut into 2 x 16 accumulator tiles of 16 x 16 and every MFMA contracts 32
// indices.  The matrix pipe does the same multiply-adds with half the accumulator updates, and on this chip
// that is what counts: the kernel's time is set by the clock the chip can hold under the matrix cores' power
// draw, and a register-resident loop of 16x16x32 MFMAs sustains about 97 % of the nominal rate on these
// operands (3-bit codes against 8-bit significands) where 32x32x16 sustains about 82 %.
//
// Lane l of a wave: c16 = l % 16, quarter q = l / 16.  It holds the tokens 32 wave + 16 s + c16, s = 0, 1, and
// of every accumulator tile (s, ct) the four columns 16 ct + 4 q + [0, 4) of its token.  Of a slab's 128
// codes per token it unpacks unit q (codes [32 q, 32 q + 32)), whose four k-steps are the slab's four ticks.
// The weights come from the second prepared stream (16-column fragments, remat_layout.hpp), tile ct running
// 3 - ct / 4 ticks behind the walk so that every tick rescales four tiles.
#include <mutex>

#include "remat_common.hpp"

namespace xq {

typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

__device__ __forceinline__ float row16_max(float v)      // all-reduce over each row of 16 lanes
{
    v = fmaxf(v, dpp_f32<DPP_QUAD_XOR1>(v));
    v = fmaxf(v, dpp_f32<DPP_QUAD_XOR2>(v));
    v = fmaxf(v, dpp_f32<DPP_ROW_HALF_MIRROR>(v));
    v = fmaxf(v, dpp_f32<DPP_ROW_MIRROR>(v));
    return v;
}
__device__ __forceinline__ float row16_sum(float v)
{
    v += dpp_f32<DPP_QUAD_XOR1>(v);
    v += dpp_f32<DPP_QUAD_XOR2>(v);
    v += dpp_f32<DPP_ROW_HALF_MIRROR>(v);
    v += dpp_f32<DPP_ROW_MIRROR>(v);
    return v;
}

// rotary embedding of the rematerialised keys (tiles 0-7): column n < 64 pairs with n + 64, i.e. tile ct with tile
// ct + 4, same element; the table row is the token's position
__device__ __forceinline__ void rope_rotate16(const RematParams& p, const TileCtx& c, f32x4 (&acc)[2][16])
{
    const int tok_base = c.tile * TILE_TOKENS + c.wave * CHUNK_TOKENS;
    const int c16 = c.lane & 15, q = c.lane >> 4;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const int tok = min(tok_base + 16 * s + c16, c.len - 1);
        const float* tab = p.rope + (long long)(p.pos0.v[c.b] + tok) * 128;
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) {
            const float* cs = tab + 2 * (16 * ct + 4 * q);
            const float4 cs0 = *reinterpret_cast<const float4*>(cs);
            const float4 cs1 = *reinterpret_cast<const float4*>(cs + 4);
            const float co[4] = {cs0.x, cs0.z, cs1.x, cs1.z}, si[4] = {cs0.y, cs0.w, cs1.y, cs1.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float a = acc[s][ct][k], b = acc[s][ct + 4][k];
                acc[s][ct][k] = __builtin_fmaf(a, co[k], -b * si[k]);
                acc[s][ct + 4][k] = __builtin_fmaf(b, co[k], a * si[k]);
            }
        }
    }
}

// ---- attention on the rematerialised chunk, accumulator layout of the 16 x 16 tiles: tiles 0-7 are K, 8-15 V;
// element i of tile (s, ct) is column 16 (ct % 8) + 4 q + i of token 32 wave + 16 s + c16.  Scores, softmax
// weights and the weighted sum of V stay inside the wave; one partial (m, l, o[128]) per query head.
__device__ __forceinline__ void attention_epilogue16(const RematParams& p, const TileCtx& c, f32x4 (&acc)[2][16])
{
    const int tok_base = c.tile * TILE_TOKENS + c.wave * CHUNK_TOKENS;
    if (tok_base >= c.len) return;                                         // chunk entirely past len
    const int c16 = c.lane & 15, q = c.lane >> 4;
    if (p.rope) rope_rotate16(p, c, acc);
    const int gq = p.Hq / p.Hkv;
    const int chunk = p.chunk0.v[c.b] + c.tile * (TILE_TOKENS / CHUNK_TOKENS) + c.wave;
    for (int j = 0; j < gq; ++j) {
        const int hq = c.hk * gq + j;
        const uint16_t* qv = p.q + ((long long)c.b * p.Hq + hq) * 128 + 4 * q;
        float dot[2] = {0.0f, 0.0f};
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) {
            const uint2 qq = *reinterpret_cast<const uint2*>(qv + 16 * ct);
            const float q0 = bf16_lo_to_f32(qq.x), q1 = bf16_hi_to_f32(qq.x), q2 = bf16_lo_to_f32(qq.y), q3 = bf16_hi_to_f32(qq.y);
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                dot[s] = __builtin_fmaf(q0, acc[s][ct][0], dot[s]);
                dot[s] = __builtin_fmaf(q1, acc[s][ct][1], dot[s]);
                dot[s] = __builtin_fmaf(q2, acc[s][ct][2], dot[s]);
                dot[s] = __builtin_fmaf(q3, acc[s][ct][3], dot[s]);
            }
        }
        float sc[2];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            float d = dot[s] + __shfl_xor(dot[s], 16);                    // the four quarters hold 32 columns each
            d += __shfl_xor(d, 32);
            sc[s] = tok_base + 16 * s + c16 < c.len ? d * p.scale_log2e : -INFINITY;
        }
        const float m = row16_max(fmaxf(sc[0], sc[1]));                    // (every row holds all 32 tokens)
        const float p0 = __builtin_amdgcn_exp2f(sc[0] - m), p1 = __builtin_amdgcn_exp2f(sc[1] - m);
        const float l = row16_sum(p0 + p1);
        const long long pidx = ((long long)c.b * p.Hq + hq) * p.chunks_per_seq + chunk;
        float* po = p.part_o + pidx * 128 + 4 * q;
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) {
            float o[4];
#pragma unroll
            for (int k = 0; k < 4; ++k)   // masked tokens have weight 0 and their rows are clamped copies: finite
                o[k] = row16_sum(__builtin_fmaf(p0, acc[0][8 + ct][k], p1 * acc[1][8 + ct][k]));
            if (c16 == 0) {
                float4 w; w.x = o[0]; w.y = o[1]; w.z = o[2]; w.w = o[3];
                *reinterpret_cast<float4*>(po + 16 * ct) = w;
            }
        }
        if (c.lane == 0) {
            p.part_ml[pidx * 2] = m;
            p.part_ml[pidx * 2 + 1] = l;
        }
    }
}

// =====================================================================================
// Attention for many query rows (chunked prefill, App. A; decode with four or more query heads per KV head) on the
// matrix cores, for the 16 x 16 tile layout.  Query rows (a query token and one of the KV head's query heads) are
// taken 16 at a time:
//   S^T[token][query] = K Q^T : A = the wave's K tiles straight from the accumulator registers -- the 8 values a lane
//       holds of two adjacent tiles are 8 contraction indices in a fixed permuted order, which the Q fragment loads
//       mirror -- split into bf16 hi + lo (8 MFMAs per token half).  The result has lane = (query c16, tokens
//       16 s + 4 q + [0, 4)): mask, max, exp2 and sum are per-lane loops plus exchanges between the four quarters.
//   The eight waves exchange their maxima through LDS (barrier), so every wave forms its softmax weights against the
//   tile's maximum, and writes them (bf16 hi + lo) to LDS exactly as its lanes hold them: 16 bytes per lane, which
//   is one lane's share of an A fragment of P (query rows x 32 tokens).  Barrier.
//   O[query][n] = P V : wave w owns the 16 value columns 16 w + [0, 16) and contracts over all 256 tokens of the
//       tile: per 32-token chunk one P fragment (from LDS, as written) against the chunk's V read column-wise, for
//       which every wave has transposed its V once per tile into bf16 hi and lo images [n][32 tokens] in LDS
//       (64-byte rows whose 8-byte pieces are XOR-swizzled by the row: conflict-free fragment reads);
//       hi*hi + lo*hi + hi*lo, the lo*lo term (2^-16 relative) is dropped.  Each wave stores its 16 columns of the
//       partial (m, l, o[128]) per (query row, 256-token tile): no sum over waves is left.
// Two workgroup barriers per 16 query rows, and P V of one group overlaps the scores of the next.  LDS: 8 x 16 KiB of V images over the dead slab buffers, 16 KiB of
// softmax weights, 1 KiB of maxima and sums.  Called by all eight waves; nothing else may touch the LDS any more.
// =====================================================================================
constexpr int PF16_VT_IMAGE_BYTES = 128 * 64;
constexpr int PF16_VT_WAVE_BYTES = 2 * PF16_VT_IMAGE_BYTES;
constexpr int PF16_P_OFF = 8 * PF16_VT_WAVE_BYTES;
constexpr int PF16_P_BYTES = 2 * 8 * 1024;             // hi and lo, [chunk 8][lane 64][16 B]
constexpr int PF16_M_OFF = PF16_P_OFF + PF16_P_BYTES;   // float [8 waves][16 queries] maxima, then sums
constexpr int PF16_TOTAL = PF16_M_OFF + 2 * 8 * 16 * 4;

// byte offset of the 8-byte piece (4 tokens) `piece` of row n inside a V image
__device__ __forceinline__ int vt16_offset(int n, int piece) { return n * 64 + ((piece ^ (2 * ((n >> 2) & 3))) << 3); }

__device__ __forceinline__ void split_hi_lo(const float (&v)[8], uint4& hi, uint4& lo)
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

__device__ __forceinline__ f32x4 mfma16_bf16(const uint4& a, const uint4& b, const f32x4& c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

__device__ __forceinline__ void prefill_epilogue16(const RematParams& p, const TileCtx& c, f32x4 (&acc)[2][16], uint8_t* lds)
{
    const int tok0 = c.tile * TILE_TOKENS + c.wave * CHUNK_TOKENS;
    const bool active = tok0 < c.len;                                      // wave-uniform: chunk not entirely past len
    // (the lane index passes through an empty asm statement: the addresses derived from it below are then not
    // computed ahead of the contraction loop, where they would cost registers the loop does not have)
    int lane_here = c.lane;
    asm volatile("" : "+v"(lane_here));
    const int c16 = lane_here & 15, q = lane_here >> 4;
    __syncthreads();                                                       // every wave is done with the slab buffers
    uint4 khi[2][4], klo[2][4];
    if (active) {
        if (p.rope) rope_rotate16(p, c, acc);
        // V^T images of the wave's 32 tokens: element i of tile (s, 8 + ct) is V[token 16 s + c16][n = 16 ct + 4 q + i]
        uint8_t* vt = lds + c.wave * PF16_VT_WAVE_BYTES;
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int ct = 0; ct < 8; ++ct)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int n = 16 * ct + 4 * q + i, t = 16 * s + c16;
                    const float v = acc[s][8 + ct][i];
                    const uint32_t h = pack_bf16x2_rne(v, 0.0f);
                    uint8_t* dst = vt + vt16_offset(n, t >> 2) + (t & 3) * 2;
                    *reinterpret_cast<uint16_t*>(dst) = (uint16_t)h;
                    *reinterpret_cast<uint16_t*>(dst + PF16_VT_IMAGE_BYTES) = (uint16_t)pack_bf16x2_rne(v - bf16_lo_to_f32(h), 0.0f);
                }
        // K fragments: contraction block kb covers columns [32 kb, 32 kb + 32) = tiles 2 kb, 2 kb + 1; this lane's 8
        // of them are 32 kb + 4 q + [0, 4) and 32 kb + 16 + 4 q + [0, 4)
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) {
                float v[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) v[k] = acc[s][2 * kb + (k >> 2)][k & 3];
                split_hi_lo(v, khi[s][kb], klo[s][kb]);
            }
    } else {
        // a chunk entirely past len contributes nothing: zero V images (and zero weights below) let every wave
        // contract over all eight chunks without a branch
        uint8_t* vt = lds + c.wave * PF16_VT_WAVE_BYTES;
#pragma unroll
        for (int k = 0; k < PF16_VT_WAVE_BYTES / 1024; ++k)
            *reinterpret_cast<uint4*>(vt + k * 1024 + c.lane * 16) = make_uint4(0u, 0u, 0u, 0u);
    }

    const int gq = p.Hq / p.Hkv, NQ = p.Tq * gq;
    float* mbuf = reinterpret_cast<float*>(lds + PF16_M_OFF);             // [wave][16 queries]
    float* lbuf = mbuf + 8 * 16;
    uint8_t* pbuf = lds + PF16_P_OFF;
    // query row qi = (query token tq, head j of the KV head's gq): qi / gq by a multiply (exact while qi gq < 2^32;
    // the host admits no more than 65535 query tokens per launch)
    const uint32_t gq_magic = 0xFFFFFFFFu / (uint32_t)gq + 1u;
    auto token_of = [&](int qi) -> int { return gq == 1 ? qi : (int)__umulhi((uint32_t)qi, gq_magic); };
    auto part_row = [&](int qi) -> long long {
        const int tq = token_of(qi);
        return ((long long)c.b * p.Tq + tq) * p.Hq + c.hk * gq + (qi - tq * gq);
    };
    const int ncol = 16 * c.wave + c16;                                    // the value column this lane reads and stores
    // Where a group of 16 rows is a whole number of query tokens (1, 2, 4, 8 or 16 heads per KV head), the rows of
    // consecutive groups are a fixed stride apart, and the addresses of a group follow from those of the previous one by
    // an addition: the 64-bit multiplies of part_row (quarter-rate instructions, six uses per group) were a third of the
    // group loop's issue time.  load_q and scores are called for the groups in order, which the running values rely on.
    const bool lin = 16 % gq == 0;
    const int tok_per_group = lin ? 16 / gq : 0;
    const long long rows_per_group = (long long)tok_per_group * p.Hq;
    const uint16_t* q_run = p.q + part_row(c16) * 128 + 4 * q;            // this lane's query row of the next group to load
    int tq_run = token_of(c16);                                            // ... its query token, of the next group to score
    float* po_run = p.part_o + (part_row(4 * q) * p.chunks_per_seq + c.tile) * 128 + ncol;   // row 4 q of the group to store
    float* pml_run = p.part_ml + (part_row(c16) * p.chunks_per_seq + c.tile) * 2;
    long long po_step[4];                                                  // rows 4 q + i against row 4 q: the same for every lane
#pragma unroll
    for (int i = 0; i < 4; ++i) po_step[i] = (gq >= 4 ? i : (long long)(i / gq) * p.Hq + i % gq) * p.chunks_per_seq * 128;
    // Q fragments of the group that starts at query row q0, for this lane's query row of it (rows past NQ repeat the
    // last one and are not stored)
    auto load_q = [&](int q0, uint4 (&qf)[4]) XQ_INLINE_LAMBDA {
        const uint16_t* qv;
        if (lin && q0 + 16 <= NQ) {
            qv = q_run;
            q_run += rows_per_group * 128;
        } else {
            qv = p.q + part_row(min(q0 + c16, NQ - 1)) * 128 + 4 * q;
        }
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) {
            const uint2 a = *reinterpret_cast<const uint2*>(qv + 32 * kb);
            const uint2 b = *reinterpret_cast<const uint2*>(qv + 32 * kb + 16);
            qf[kb] = make_uint4(a.x, a.y, b.x, b.y);
        }
    };
    // scores of the wave's 32 tokens against the group's 16 query rows, masked and scaled; their maximum per query row
    // goes to mbuf
    auto scores = [&](int q0, const uint4 (&qf)[4], f32x4 (&S)[2]) XQ_INLINE_LAMBDA {
        float m = -INFINITY;
        if (active) {
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int i = 0; i < 4; ++i) S[s][i] = 0.0f;
#pragma unroll
            for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    S[s] = mfma16_bf16(khi[s][kb], qf[kb], S[s]);
                    S[s] = mfma16_bf16(klo[s][kb], qf[kb], S[s]);
                }
            // element i of S[s] <-> token tok0 + 16 s + 4 q + i; visible up to the query's own row
            // (rows past NQ, which are not stored, take whatever token the running value names)
            const int tq = lin ? tq_run : token_of(min(q0 + c16, NQ - 1));
            const int limit = c.len - p.Tq + tq - tok0;
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int rel = 16 * s + 4 * q + i;
                    S[s][i] = rel <= limit ? S[s][i] * p.scale_log2e : -INFINITY;
                    m = fmaxf(m, S[s][i]);
                }
            m = fmaxf(m, __shfl_xor(m, 16));
            m = fmaxf(m, __shfl_xor(m, 32));
        }
        tq_run += tok_per_group;
        if (q == 0) mbuf[c.wave * 16 + c16] = m;
    };

    // Software pipeline over the groups: between the two barriers of group g the softmax weights are formed; after
    // the second one P V of group g runs alongside the scores of group g + 1 (independent work: the matrix pipe and
    // the LDS latencies of one hide behind the other), and the queries of group g + 2 are already on their way --
    // the barriers wait for this wave's LDS accesses only, not for its global loads and stores.
    auto lds_barrier = [&]() XQ_INLINE_LAMBDA { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
    uint4 qf[4];
    f32x4 S[2];
    uint4 vh[8], vl[8];
    load_q(0, qf);
    scores(0, qf, S);
    if (16 < NQ) load_q(16, qf);
    for (int q0 = 0; q0 < NQ; q0 += 16) {
        lds_barrier();                                                     // the group's maxima are in mbuf
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < 8; ++w) M = fmaxf(M, mbuf[w * 16 + c16]);
        const float Mu = M == -INFINITY ? 0.0f : M;                        // nothing visible: all weights 0
        float l = 0.0f;
        uint4 phi = make_uint4(0u, 0u, 0u, 0u), plo = phi;
        if (active) {
            float pr[8];
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    pr[4 * s + i] = __builtin_amdgcn_exp2f(S[s][i] - Mu);
                    l += pr[4 * s + i];
                }
            l += __shfl_xor(l, 16);
            l += __shfl_xor(l, 32);
            split_hi_lo(pr, phi, plo);
        }
        *reinterpret_cast<uint4*>(pbuf + (c.wave * 64 + c.lane) * 16) = phi;
        *reinterpret_cast<uint4*>(pbuf + PF16_P_BYTES / 2 + (c.wave * 64 + c.lane) * 16) = plo;
        if (q == 0) lbuf[c.wave * 16 + c16] = l;
        lds_barrier();                                                     // weights and sums of all eight chunks are in LDS
        // operands of P V, four chunks ahead: contraction index (quarter q', element 4 s + i) of chunk cw <-> its
        // token 16 s + 4 q' + i, for the P fragment as written above and for the V pieces q' and 4 + q' alike
        uint4 ph[4], pl[4];
        auto load_chunk = [&](auto CW) XQ_INLINE_LAMBDA {
            constexpr int cw = decltype(CW)::value, k = cw & 3;
            ph[k] = *reinterpret_cast<const uint4*>(pbuf + (cw * 64 + c.lane) * 16);
            pl[k] = *reinterpret_cast<const uint4*>(pbuf + PF16_P_BYTES / 2 + (cw * 64 + c.lane) * 16);
        };
        static_for<0, 4>(load_chunk);
        // the V fragments of this wave's 16 columns are the same for every group of query rows: they are taken out of
        // the images once and stay in registers (the accumulator's are free by now)
        if (q0 == 0) {
            static_for<0, 8>([&](auto CW) XQ_INLINE_LAMBDA {
                constexpr int cw = decltype(CW)::value;
                const uint8_t* v0 = lds + cw * PF16_VT_WAVE_BYTES + vt16_offset(ncol, q);
                const uint8_t* v1 = lds + cw * PF16_VT_WAVE_BYTES + vt16_offset(ncol, 4 + q);
                const uint2 h0 = *reinterpret_cast<const uint2*>(v0), h1 = *reinterpret_cast<const uint2*>(v1);
                const uint2 l0 = *reinterpret_cast<const uint2*>(v0 + PF16_VT_IMAGE_BYTES);
                const uint2 l1 = *reinterpret_cast<const uint2*>(v1 + PF16_VT_IMAGE_BYTES);
                vh[cw] = make_uint4(h0.x, h0.y, h1.x, h1.y);
                vl[cw] = make_uint4(l0.x, l0.y, l1.x, l1.y);
            });
        }
        float Lt = 0.0f;
        if (c.wave == 0 && q == 0) {
#pragma unroll
            for (int w = 0; w < 8; ++w) Lt += lbuf[w * 16 + c16];
        }
        // the next group's scores (its maxima go to mbuf, which nobody reads any more before the next barrier), then
        // the queries of the group after it
        if (q0 + 16 < NQ) {
            scores(q0 + 16, qf, S);
            if (q0 + 32 < NQ) load_q(q0 + 32, qf);
        }
        f32x4 O0 = {0.0f, 0.0f, 0.0f, 0.0f}, O1 = O0, O2 = O0;             // hi*hi, lo*hi, hi*lo: three independent chains
        static_for<0, 8>([&](auto CW) XQ_INLINE_LAMBDA {
            constexpr int cw = decltype(CW)::value, k = cw & 3;
            O0 = mfma16_bf16(ph[k], vh[cw], O0);
            O1 = mfma16_bf16(pl[k], vh[cw], O1);
            O2 = mfma16_bf16(ph[k], vl[cw], O2);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (cw + 4 < 8) load_chunk(std::integral_constant<int, cw + 4>{});
            __builtin_amdgcn_sched_barrier(0);
        });
        if (c.wave == 0 && q == 0 && q0 + c16 < NQ) {
            float* ml = lin ? pml_run : p.part_ml + (part_row(q0 + c16) * p.chunks_per_seq + c.tile) * 2;
            ml[0] = M;
            ml[1] = Lt;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int qr = q0 + 4 * q + i;
            float* o = lin ? po_run + po_step[i] : p.part_o + (part_row(qr) * p.chunks_per_seq + c.tile) * 128 + ncol;
            if (qr < NQ) *o = (O1[i] + O2[i]) + O0[i];
        }
        po_run += rows_per_group * p.chunks_per_seq * 128;
        pml_run += rows_per_group * p.chunks_per_seq * 2;
    }
}

// ---- latent cache (Sec. 3.3.1), pass 2 on the 16 x 16 tiles (pass 1, the scores, stays with the 32x32x16 kernel: its
// loop is as fast on the eight slabs of a latent half and its epilogue is lighter; measured 273 against 296 us on
// config 4).  tiles 0-7 / 8-15 hold the values of the pair's two KV heads.  One head after the other goes through the second
// half of the matrix-core epilogue above: the wave writes the head's V images, turns the stored scores of the head's
// query heads (lane = query head c16, eight of the wave's tokens: 16 s + 4 q + [0, 4)) into softmax weights against the
// tile's maximum, and contracts its 16 value columns over the tile's 256 tokens: one partial (m, l, o[128]) per query
// head and tile.  Called by all eight waves; nothing else may touch the LDS any more.  At most 16 query heads per KV head.
__device__ __forceinline__ void weighted_sum_epilogue16(const RematParams& p, const TileCtx& c, f32x4 (&acc)[2][16], uint8_t* lds)
{
    const int tok0 = c.tile * TILE_TOKENS + c.wave * CHUNK_TOKENS;
    const bool active = tok0 < c.len;                                      // wave-uniform: chunk not entirely past len
    const int c16 = c.lane & 15, q = c.lane >> 4;
    const int gq = p.Hq / p.Hkv;
    const long long srow = p.score_stride;
    float* mbuf = reinterpret_cast<float*>(lds + PF16_M_OFF);             // [wave][16 queries]
    float* lbuf = mbuf + 8 * 16;
    uint8_t* pbuf = lds + PF16_P_OFF;
    uint8_t* vt = lds + c.wave * PF16_VT_WAVE_BYTES;
    const int ncol = 16 * c.wave + c16;                                    // the value column this lane reads and stores
    auto lds_barrier = [&]() XQ_INLINE_LAMBDA { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
    // the stored scores of both heads, masked (rows past the head's query heads repeat the last one and are not stored)
    float S[2][8];
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
        if (active) {
            const float* sp = p.scores + ((long long)c.b * p.Hq + (2 * c.hk + hh) * gq + min(c16, gq - 1)) * srow + tok0 + 4 * q;
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const float4 s4 = *reinterpret_cast<const float4*>(sp + 16 * s);      // past len: other rows' or stale values
                const float sv[4] = {s4.x, s4.y, s4.z, s4.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) S[hh][4 * s + i] = tok0 + 16 * s + 4 * q + i < c.len ? sv[i] : -INFINITY;
            }
        }
    }
    __syncthreads();                                                       // every wave is done with the slab buffers
    static_for<0, 2>([&](auto HH) XQ_INLINE_LAMBDA {       // (compile-time: the accumulator must stay in registers)
        constexpr int hh = decltype(HH)::value;
        const int hq0 = (2 * c.hk + hh) * gq;
        if constexpr (hh == 1) lds_barrier();                              // the first head's images and weights have been read
        float m = -INFINITY;
        if (active) {
            // V^T images: element i of tile (s, 8 hh + ct) is V[token 16 s + c16][n = 16 ct + 4 q + i]
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int ct = 0; ct < 8; ++ct)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int n = 16 * ct + 4 * q + i, t = 16 * s + c16;
                        const float v = acc[s][8 * hh + ct][i];
                        const uint32_t h = pack_bf16x2_rne(v, 0.0f);
                        uint8_t* dst = vt + vt16_offset(n, t >> 2) + (t & 3) * 2;
                        *reinterpret_cast<uint16_t*>(dst) = (uint16_t)h;
                        *reinterpret_cast<uint16_t*>(dst + PF16_VT_IMAGE_BYTES) = (uint16_t)pack_bf16x2_rne(v - bf16_lo_to_f32(h), 0.0f);
                    }
#pragma unroll
            for (int k = 0; k < 8; ++k) m = fmaxf(m, S[hh][k]);
            m = fmaxf(m, __shfl_xor(m, 16));
            m = fmaxf(m, __shfl_xor(m, 32));
        } else {
            // a chunk entirely past len contributes nothing: zero images and zero weights
#pragma unroll
            for (int k = 0; k < PF16_VT_WAVE_BYTES / 1024; ++k)
                *reinterpret_cast<uint4*>(vt + k * 1024 + c.lane * 16) = make_uint4(0u, 0u, 0u, 0u);
        }
        if (q == 0) mbuf[c.wave * 16 + c16] = m;
        lds_barrier();                                                     // the maxima are in mbuf
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < 8; ++w) M = fmaxf(M, mbuf[w * 16 + c16]);
        const float Mu = M == -INFINITY ? 0.0f : M;
        float l = 0.0f;
        uint4 phi = make_uint4(0u, 0u, 0u, 0u), plo = phi;
        if (active) {
            float pr[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                pr[k] = __builtin_amdgcn_exp2f(S[hh][k] - Mu);
                l += pr[k];
            }
            l += __shfl_xor(l, 16);
            l += __shfl_xor(l, 32);
            split_hi_lo(pr, phi, plo);
        }
        *reinterpret_cast<uint4*>(pbuf + (c.wave * 64 + c.lane) * 16) = phi;
        *reinterpret_cast<uint4*>(pbuf + PF16_P_BYTES / 2 + (c.wave * 64 + c.lane) * 16) = plo;
        if (q == 0) lbuf[c.wave * 16 + c16] = l;
        lds_barrier();                                                     // images, weights and sums of all eight chunks are in LDS
        float Lt = 0.0f;
        if (c.wave == 0 && q == 0) {
#pragma unroll
            for (int w = 0; w < 8; ++w) Lt += lbuf[w * 16 + c16];
        }
        f32x4 O0 = {0.0f, 0.0f, 0.0f, 0.0f}, O1 = O0, O2 = O0;             // hi*hi, lo*hi, hi*lo: three independent chains
        static_for<0, 8>([&](auto CW) XQ_INLINE_LAMBDA {
            constexpr int cw = decltype(CW)::value;
            const uint4 ph = *reinterpret_cast<const uint4*>(pbuf + (cw * 64 + c.lane) * 16);
            const uint4 pl = *reinterpret_cast<const uint4*>(pbuf + PF16_P_BYTES / 2 + (cw * 64 + c.lane) * 16);
            const uint8_t* v0 = lds + cw * PF16_VT_WAVE_BYTES + vt16_offset(ncol, q);
            const uint8_t* v1 = lds + cw * PF16_VT_WAVE_BYTES + vt16_offset(ncol, 4 + q);
            const uint2 h0 = *reinterpret_cast<const uint2*>(v0), h1 = *reinterpret_cast<const uint2*>(v1);
            const uint2 l0 = *reinterpret_cast<const uint2*>(v0 + PF16_VT_IMAGE_BYTES);
            const uint2 l1 = *reinterpret_cast<const uint2*>(v1 + PF16_VT_IMAGE_BYTES);
            const uint4 vh = make_uint4(h0.x, h0.y, h1.x, h1.y), vl = make_uint4(l0.x, l0.y, l1.x, l1.y);
            O0 = mfma16_bf16(ph, vh, O0);
            O1 = mfma16_bf16(pl, vh, O1);
            O2 = mfma16_bf16(ph, vl, O2);
        });
        if (c.wave == 0 && q == 0 && c16 < gq) {
            const long long pidx = ((long long)c.b * p.Hq + hq0 + c16) * p.chunks_per_seq + c.tile;
            p.part_ml[pidx * 2] = M;
            p.part_ml[pidx * 2 + 1] = Lt;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int qr = 4 * q + i;
            if (qr < gq) p.part_o[(((long long)c.b * p.Hq + hq0 + qr) * p.chunks_per_seq + c.tile) * 128 + ncol] = (O1[i] + O2[i]) + O0[i];
        }
    });
}

// G = 64 (2-bit codes only): "scales on the token operand".  With groups of 64 a tile would meet two group boundaries
// per slab, and rescaling 128 accumulator registers twice per slab makes the loop wait for vector-instruction issue
// (measured: no faster than the 32x32x16 kernel).  Instead the group's scale goes into the token fragment: tick j takes
// the 32 codes of unit j of the slab (quarter q its k-step q, so that a tick lies inside one group; possible because the
// 2-bit k-steps differ by a rotation only), and every operand dword is multiplied, right after the unpack, by the packed
// fp16 factor f = 2^15 e_group / N_token, N_token = the power of two at or above the token's largest effective scale
// (the pre-pass leaves it in the spare group row of the transposed scales).  A 2-bit code times an 8-bit significand is
// exact in fp16, and a group 2^11 below the token's largest reaches the subnormal grid with an absolute error of 2^-24
// of the largest: no Horner pass, no scale state in the loop, one scaling by N_token 2^-15 at the end.
//
// MODE_ATTENTION_PC (per-channel cache, Sec. 3.3.1: one scale and zero-point per channel and block of 64 or 128
// tokens; codes packed per token row as in a per-token cache, walked in the layout of groups of 128).  The scale
// varies along the contraction, so it too goes to the token operand: every unpacked operand dword is multiplied
// (packed fp16) by the block's factors scale 2^(15 - E_blk) of its two channels -- exact for codes of at most 3 bits;
// 4-bit codes enter as code - 8, whose products are exact too, and the block-constant 8 scale W term joins the
// zero-point term.  A wave's 32 tokens lie in one block, so all lanes of a quarter read the same factors from a 1 KiB
// image per slab that the scale DMA brings into three rotating buffers.  No Horner pass, no correction phase: the
// epilogue scales by the block's power of two and adds z_blk [Wk_h | Wv_h], which a pre-pass has left in memory.
template <int BITS, int G, int MODE>
__global__ __launch_bounds__(512) void remat_attn_tile16_kernel(const RematParams p)
{
    static_assert(G == 128 || (G == 64 && BITS == 2), "group size");
    constexpr bool PC = MODE == MODE_ATTENTION_PC;     // per-channel source: block factors on the token operand
    static_assert(!PC || G == 128, "the per-channel source unpacks like groups of 128");
    constexpr int GPS = 128 / G;                       // groups per slab
    constexpr int NCUR = G == 64 ? 4 : BITS;           // dwords of packed codes a lane keeps per slab and token half
    constexpr int ROW_SLAB_BYTES = 16 * BITS;          // packed bytes of 128 channels of one token
    constexpr int UNIT_BYTES = 4 * BITS;               // ... of a unit of 32 codes
    constexpr int NCI = 4 * BITS;                      // code-DMA wave instructions per slab per workgroup
    constexpr int IMG_BYTES = code_image_bytes(BITS);
    constexpr int NIMG = n_code_images(BITS);
    constexpr int LDS_SCALES_OFF = lds_scales_off(BITS);
    constexpr int NT = TILE16_TICKS;                   // ticks (k32-steps) per slab
    // slots between the LDS read of a weight fragment and its use (one fewer where the epilogue keeps more alive)
    constexpr int AHEAD = (MODE == MODE_PREFILL || MODE == MODE_WEIGHTED_SUM) ? 4 : 5;
    constexpr int NRING = 8;                           // (divides 64: the ring runs on from slab to slab)

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    TileCtx c;
    if (!locate_tile(p, c)) return;
    const int lane = c.lane, wave = c.wave;
    const int c16 = lane & 15, q = lane >> 4;

    // (n_corr_ksteps counts ticks here; the per-channel source has no correction phase: its zero-point term
    // comes from a pre-pass)
    const int n_corr_slabs = PC ? 0 : (p.n_corr_ksteps + NT - 1) / NT;
    const int head_shift = p.head_shift[c.hk];         // the head's stream holds its weights times 2^head_shift
    const uint8_t* wsrc = p.wprep + (long long)c.hk * p.head_bytes + wave * 1024;   // this wave's DMA share
    const uint32_t dma_voff = (uint32_t)lane * 16u;
    const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) uint8_t*)lds;
    const uint32_t lds_w = lds_base + wave * 1024;
    const uint8_t* my_slab = lds + lane * 16;          // + buffer * SLAB_BYTES + (tick * 16 + tile) * 1024

    // ---- token-side sources
    const long long seq_row0 = (long long)c.b * p.cap;
    const uint32_t row_bytes = (uint32_t)(p.row_d * BITS / 8);
    const uint8_t* cbase = p.codes + seq_row0 * row_bytes;
    const uint16_t* zbase = p.zero + seq_row0 * p.ng_row;
    // per-token source: effective scales, GPS * 512 bytes per slab; per-channel: one 1 KiB factor image per slab
    constexpr int E_SLAB_BYTES = PC ? LDS_SCALES_BYTES : 512 * GPS;
    const uint8_t* ebase = reinterpret_cast<const uint8_t*>(p.eT) +
                           (PC ? ((long long)c.b * p.tiles_per_seq + c.tile) * (long long)(p.n_main_slabs + 1) * LDS_SCALES_BYTES
                               : ((long long)c.b * p.tiles_per_seq + c.tile) * (long long)(p.ng + 1) * 512);
    int my_row[2];
    uint32_t moff[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        my_row[s] = wave * CHUNK_TOKENS + 16 * s + c16;
        moff[s] = (uint32_t)min(c.tile * TILE_TOKENS + my_row[s], c.len - 1) * (uint32_t)p.ng_row;
    }
    // this lane's codes and scales in the LDS images, for its first token; the second one sits 16 rows further on (one
    // base each, so that the loop keeps one register per pointer).  Groups of 128: unit q; groups of 64: of every unit j
    // the dword that holds its k-step q (2 bits: dword q / 2)
    const uint8_t* my_codes0 = lds + LDS_CODES_OFF + my_row[0] * ROW_SLAB_BYTES + (G == 128 ? q * UNIT_BYTES : (q >> 1) * 4);
    const uint16_t* my_scale0 = reinterpret_cast<const uint16_t*>(lds + LDS_SCALES_OFF) + my_row[0];
    // code DMA: 16-byte piece pc of the tile's slab image = (row pc / BITS, part pc % BITS);
    // wave instruction i covers pieces [64 i, 64 i + 64); this wave issues i = wave and wave + 8
    uint32_t cvoff[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int pc = (wave + 8 * k) * 64 + lane;
        const int rl = pc / BITS, prt = pc % BITS;
        cvoff[k] = (uint32_t)min(c.tile * TILE_TOKENS + rl, c.len - 1) * row_bytes + prt * 16;
    }

    f32x4 acc[2][16];                    // [token half][column tile]: tiles 0-7 K, 8-15 V
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int ct = 0; ct < 16; ++ct)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[s][ct][i] = 0.0f;

    uint4 af[8];                         // weight fragments, ring over slots (loaded AHEAD slots ahead)
    uint32_t ub[2][NT][4];               // token fragments, ring over ticks
    uint32_t cur[2][NCUR];               // packed codes of the current slab, per token half
    float E_prev[2], E_cur[2];           // groups of 128: effective scales of the previous and the current slab's group
    float hr[2];                         // ... and the Horner factors E_prev / E_cur of the boundaries seen this slab
    // groups of 64: packed fp16 factors (f, f) of the slab's two groups per token half, for the slab whose codes are in
    // cur; the token's normaliser and 2^15 / normaliser
    uint32_t fac[2][2];
    float tok_norm[2], tok_inv15[2];
    // 2-bit codes, groups of 64: k-step q of a unit is its dword q / 2 rotated left by 6 and 2 (q even) or by 30 and
    // 26 (q odd: a right shift by 2 and 6; what the rotation brings in falls outside the masks)
    const int rot_a = (q & 1) ? 30 : 6, rot_b = (q & 1) ? 26 : 2;
    // per-channel source: the block's factors scale 2^(15 - E_blk) of this quarter's channels, in the order the operand
    // dwords hold them, from the slab's image in a scale buffer ([block of the tile][tick][quarter][8 fp16]: every lane
    // of a quarter reads the same 16 bytes); pcf = those of the tick whose fragments are made next
    const uint8_t* my_factors = lds + LDS_SCALES_OFF + (PC ? ((wave * CHUNK_TOKENS) / p.pc_block) * 256 + q * 16 : 0);
    uint4 pcf = {0u, 0u, 0u, 0u};
    auto fetch_tick_factors = [&](int sbuf, int j) XQ_INLINE_LAMBDA {
        pcf = *reinterpret_cast<const uint4*>(my_factors + sbuf * LDS_SCALES_BYTES + j * 64);
    };

    auto fetch_scales = [&](int sbuf, float (&e)[2]) XQ_INLINE_LAMBDA {
#pragma unroll
        for (int s = 0; s < 2; ++s) e[s] = __uint_as_float((uint32_t)my_scale0[16 * s + sbuf * (LDS_SCALES_BYTES / 2)] << 16);
    };
    // groups of 64: the factors of the slab whose scales are in buffer sbuf
    auto fetch_factors = [&](int sbuf, uint32_t (&f)[2][2]) XQ_INLINE_LAMBDA {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const float e = __uint_as_float((uint32_t)my_scale0[16 * s + sbuf * (LDS_SCALES_BYTES / 2) + g * TILE_TOKENS] << 16);
                const _Float16 h = (_Float16)(e * tok_inv15[s]);            // exact: 8-bit significand, at most 2^15
                const xq_f16x2 hh = {h, h};
                f[s][g] = __builtin_bit_cast(uint32_t, hh);
            }
    };
    auto fetch_tokens = [&](int img) XQ_INLINE_LAMBDA {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const uint8_t* src = my_codes0 + s * 16 * ROW_SLAB_BYTES + img * IMG_BYTES;
            if constexpr (G == 64) {
#pragma unroll
                for (int j = 0; j < 4; ++j) cur[s][j] = *reinterpret_cast<const uint32_t*>(src + j * UNIT_BYTES);
            } else if constexpr (BITS == 4) {
                const uint4 v = *reinterpret_cast<const uint4*>(src);
                cur[s][0] = v.x; cur[s][1] = v.y; cur[s][2] = v.z; cur[s][3] = v.w;
            } else if constexpr (BITS == 2) {
                const uint2 v = *reinterpret_cast<const uint2*>(src);
                cur[s][0] = v.x; cur[s][1] = v.y;
            } else {
#pragma unroll
                for (int i = 0; i < BITS; ++i) cur[s][i] = reinterpret_cast<const uint32_t*>(src)[i];
            }
        }
    };
    // the 4 operand dwords of tick j of the slab whose codes are in cur (groups of 64: times the group's factor)
    auto unpack_tick = [&](int s, int j, uint32_t (&t)[4]) XQ_INLINE_LAMBDA {
        if constexpr (PC) {
            unpack_kstep<BITS>(&cur[s][0], j, t);
            if constexpr (BITS == 4) {
                // a 4-bit code times an 8-bit significand needs 12 bits; (code - 8) times it needs 11 and is exact in
                // fp16.  All 4-bit fields sit at mantissa offset 6, so 8 is the subnormal 2^-15 in both halves; the
                // 8 * scale * W that this takes out is the same for every token of the block and comes back with
                // the zero-point term.
                constexpr uint32_t MINUS_EIGHT = 0x82008200u;
#pragma unroll
                for (int i = 0; i < 4; ++i) t[i] = pk_add_f16(t[i], MINUS_EIGHT);
            }
            t[0] = pk_mul_f16(t[0], pcf.x); t[1] = pk_mul_f16(t[1], pcf.y);
            t[2] = pk_mul_f16(t[2], pcf.z); t[3] = pk_mul_f16(t[3], pcf.w);
        } else if constexpr (G == 128) {
            unpack_kstep<BITS>(&cur[s][0], j, t);
        } else {
            const uint32_t d = cur[s][j];
            const uint32_t a = __builtin_amdgcn_alignbit(d, d, 32 - rot_a), b = __builtin_amdgcn_alignbit(d, d, 32 - rot_b);
            const uint32_t f = fac[s][j >> 1];
            t[0] = pk_mul_f16(a & 0x00C000C0u, f); t[1] = pk_mul_f16(a & 0x03000300u, f);
            t[2] = pk_mul_f16(b & 0x00C000C0u, f); t[3] = pk_mul_f16(b & 0x03000300u, f);
        }
    };
    auto make_fragment = [&](auto S, auto J) XQ_INLINE_LAMBDA {
        constexpr int s = decltype(S)::value, j = decltype(J)::value;
        unpack_tick(s, j, ub[s][j]);
    };
    auto make_half_fragment = [&](auto S, auto J, auto H) XQ_INLINE_LAMBDA {   // operand dwords 2 H, 2 H + 1 of it
        constexpr int s = decltype(S)::value, j = decltype(J)::value, h = decltype(H)::value;
        uint32_t t[4];
        unpack_tick(s, j, t);
        ub[s][j][2 * h] = t[2 * h];
        ub[s][j][2 * h + 1] = t[2 * h + 1];
    };
    // one piece of the DMA that brings in main slab `slab` (weights to `wdst`): steps 0,1 this wave's
    // code pieces (to code image `img`), 2 scales (wave 7; of slab `slab2`, into scale buffer `sbuf`),
    // 3..10 the weight chunks
    auto dma_step = [&](int step, int slab, int img, int slab2, bool with_scales2, int sbuf, uint32_t wdst) XQ_INLINE_LAMBDA {
        if (step < 2) {
            if (wave + 8 * step < NCI)
                dma_b128(cbase + slab * ROW_SLAB_BYTES, cvoff[step],
                         lds_base + LDS_CODES_OFF + (uint32_t)(img * IMG_BYTES) + (wave + 8 * step) * 1024);
        } else if (step == 2) {
            if (with_scales2 && wave == 7)
                dma_b128(ebase + (long long)slab2 * E_SLAB_BYTES, dma_voff, lds_base + LDS_SCALES_OFF + (uint32_t)(sbuf * LDS_SCALES_BYTES));
        } else {
            dma_b128(wsrc + (long long)slab * SLAB_BYTES + (step - 3) * 8192, dma_voff, wdst + (step - 3) * 8192);
        }
    };

    // ==== phase 1: the zero-point correction (scale 1): bf16 ticks whose token-side operands are the stored
    // zero-points of 8 groups per lane.  The codes and scales of the slab that cyclically precedes the first
    // one arrive meanwhile: the lagging tiles start inside it.
    const bool vec_meta = (p.ng & 7) == 0 && (p.ng_row & 7) == 0 && ((size_t)zbase & 15) == 0 && p.meta_shift == 0;
    auto load_meta = [&](int s, int kk) -> uint4 {
        const int kappa0 = kk * 32 + q * 8;
        const int term = kappa0 / p.ng_pad, g0 = kappa0 % p.ng_pad;
        uint4 v = {0u, 0u, 0u, 0u};
        if (kk < p.n_corr_ksteps && term < N_CORR_TERMS) {
            if (vec_meta) {
                v = *reinterpret_cast<const uint4*>(zbase + moff[s] + g0);
            } else {
                uint32_t h[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int g = g0 + i;
                    const uint32_t x = zbase[moff[s] + (min(g, p.ng - 1) >> p.meta_shift)];
                    h[i] = g < p.ng ? x : 0u;               // padding groups contribute nothing
                }
                v.x = h[0] | (h[1] << 16); v.y = h[2] | (h[3] << 16);
                v.z = h[4] | (h[5] << 16); v.w = h[6] | (h[7] << 16);
            }
        }
        return v;
    };
    const int slab_prev = p.n_main_slabs - 1;           // the walk is cyclic: the slab "before" slab 0
    if constexpr (G == 64) {
        // the tokens' normalisers (powers of two): the spare group row of the transposed scales
        const uint16_t* nrm = reinterpret_cast<const uint16_t*>(ebase + (long long)p.ng * 512);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const uint32_t nb = (uint32_t)nrm[my_row[s]] << 16;
            tok_norm[s] = __uint_as_float(nb);
            tok_inv15[s] = __uint_as_float(0x7F000000u - nb + (15u << 23));   // 2^15 / normaliser, exactly
        }
    }
    if constexpr (PC) issue_slab(wsrc, lds_w, dma_voff);                               // the first main slab -> buffer 0
    else issue_slab_chunks(wsrc + (long long)p.n_main_slabs * SLAB_BYTES, lds_w, dma_voff,   // correction slab 0 -> buffer 0
                           2 * min(NT, p.n_corr_ksteps));                                    // (a tick is two chunks)
    dma_step(0, slab_prev, NIMG - 1, 0, false, 0, 0);                                  // predecessor codes -> last image
    dma_step(1, slab_prev, NIMG - 1, 0, false, 0, 0);
    dma_step(2, 0, 0, slab_prev, true, 2, 0);                                          // its scales -> scale buffer 2
    dma_step(2, 0, 0, 0, true, 0, 0);                                                  // first slab's scales -> buffer 0
    if (p.n_main_slabs > 1) dma_step(2, 0, 0, 1, true, 1, 0);                          // second slab's -> buffer 1
    if constexpr (NIMG == 2) {                                                         // first slab's codes -> image 0
        dma_step(0, 0, 0, 0, false, 0, 0);
        dma_step(1, 0, 0, 0, false, 0, 0);
    }
    uint4 mfr[2][NT];
    if constexpr (PC) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        fetch_tokens(NIMG - 1);
        if constexpr (NIMG == 1) {
            // every wave now holds its predecessor codes in registers: the first slab's codes may overwrite the only image
            __syncthreads();
            dma_step(0, 0, 0, 0, false, 0, 0);
            dma_step(1, 0, 0, 0, false, 0, 0);
        }
    } else {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int j = 0; j < NT; ++j) mfr[s][j] = load_meta(s, j);
    }
    for (int cs = 0; cs < n_corr_slabs; ++cs) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        // The zero-points have arrived with that wait, but the compiler counts only its own loads, not the DMA: left
        // alone it waits for them at their first use, with vmcnt(0), behind the DMA issued next, and the correction
        // would start only after that slab has landed.  Using the registers here puts its wait here, where it is free.
#pragma unroll
        for (int ss = 0; ss < 2; ++ss)
            asm volatile("" :: "v"(mfr[ss][0].x), "v"(mfr[ss][0].y), "v"(mfr[ss][0].z), "v"(mfr[ss][0].w),
                               "v"(mfr[ss][1].x), "v"(mfr[ss][1].y), "v"(mfr[ss][1].z), "v"(mfr[ss][1].w),
                               "v"(mfr[ss][2].x), "v"(mfr[ss][2].y), "v"(mfr[ss][2].z), "v"(mfr[ss][2].w),
                               "v"(mfr[ss][3].x), "v"(mfr[ss][3].y), "v"(mfr[ss][3].z), "v"(mfr[ss][3].w));
        const uint32_t wdst = lds_w + (uint32_t)(((cs + 1) & 1) * SLAB_BYTES);
        if (cs + 1 < n_corr_slabs)
            issue_slab_chunks(wsrc + (long long)(p.n_main_slabs + cs + 1) * SLAB_BYTES, wdst, dma_voff,
                              2 * min(NT, p.n_corr_ksteps - (cs + 1) * NT));
        else issue_slab(wsrc, wdst, dma_voff);                                                   // the first main slab
        if (cs == 0) {
            fetch_tokens(NIMG - 1);
            if constexpr (G == 64) fetch_factors(2, fac);
            else fetch_scales(2, E_prev);
        }
        const uint8_t* slab = my_slab + (cs & 1) * SLAB_BYTES;
        const int nj = min(NT, p.n_corr_ksteps - cs * NT);
#pragma unroll
        for (int sl = 0; sl < AHEAD; ++sl) af[sl] = *reinterpret_cast<const uint4*>(slab + sl * 1024);
        static_for<0, NT * 16>([&](auto SIDX) XQ_INLINE_LAMBDA {
            constexpr int sidx = decltype(SIDX)::value, j = sidx >> 4, ct = sidx & 15;
            if (j < nj) {
                acc[0][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, af[sidx & 7]),
                                                                     __builtin_bit_cast(bf16x8, mfr[0][j]), acc[0][ct], 0, 0, 0);
                acc[1][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, af[sidx & 7]),
                                                                     __builtin_bit_cast(bf16x8, mfr[1][j]), acc[1][ct], 0, 0, 0);
            }
            if constexpr (sidx + AHEAD < NT * 16) af[(sidx + AHEAD) & 7] = *reinterpret_cast<const uint4*>(slab + (sidx + AHEAD) * 1024);
            if constexpr (NIMG == 1) {
                if constexpr (sidx == 0) {
                    if (cs == 0) {
                        // every wave now holds its predecessor codes in registers: the first slab's
                        // codes may overwrite the only image
                        __syncthreads();
                        dma_step(0, 0, 0, 0, false, 0, 0);
                        dma_step(1, 0, 0, 0, false, 0, 0);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        if (cs + 1 < n_corr_slabs) {
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int j = 0; j < NT; ++j) mfr[s][j] = load_meta(s, (cs + 1) * NT + j);
        }
    }

    // ==== phase 2: the d x 256 contraction, a cyclic walk over the d/32 ticks that starts at slab 0.  Tile ct
    // runs lag(ct) = 3 - ct / 4 ticks behind: at tick tau it multiplies the weights of tick tau - lag (the
    // stream is laid out in this order) with the token fragment unpacked lag ticks ago, which waits in a 4-deep
    // ring.  A tile enters the current slab's group at tick lag(ct); its 8 accumulator registers are rescaled
    // in the slots before that, so every tick rescales four tiles: eight slots of a tick multiply four registers
    // each, four others unpack half a token fragment each, and no slot carries more than five such instructions.
    //
    // Set-up: the ring's lagging fragments are ticks 1..3 of the predecessor slab, in whose group the lagging
    // tiles start; the accumulators (holding the correction in units of 1) are brought to those scales.
    static_for<1, NT>([&](auto J) XQ_INLINE_LAMBDA {
        if constexpr (PC) fetch_tick_factors(2, decltype(J)::value);       // (the predecessor slab's factors wait in buffer 2)
        make_fragment(std::integral_constant<int, 0>{}, J);
        make_fragment(std::integral_constant<int, 1>{}, J);
    });
    const int par0 = n_corr_slabs & 1;                 // weight buffer of main iteration 0
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    fetch_tokens(0);
    if constexpr (PC) fetch_tick_factors(0, 0);
    else if constexpr (G == 64) fetch_factors(0, fac);
    else fetch_scales(0, E_cur);
    {
        const uint8_t* slab0 = my_slab + par0 * SLAB_BYTES;
#pragma unroll
        for (int sl = 0; sl < AHEAD; ++sl) af[sl] = *reinterpret_cast<const uint4*>(slab0 + sl * 1024);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            // (every tile starts in the predecessor's units: those without lag are rescaled at tick 0 like the others
            // later; groups of 64: in the token's own units, 2^15 / normaliser, for the whole walk)
            if constexpr (!PC) {
                const float r_prev = G == 64 ? ldexpf(tok_inv15[s], head_shift) : ldexpf(__builtin_amdgcn_rcpf(E_prev[s]), head_shift);
#pragma unroll
                for (int ct = 0; ct < 16; ++ct) acc[s][ct] *= r_prev;
                if constexpr (G == 128) hr[s] = E_prev[s] * __builtin_amdgcn_rcpf(E_cur[s]);
            }
        }
    }

    for (int it = 0; it < p.n_main_slabs; ++it) {
        // With a single code image, everyone must have taken the previous slab's codes out of it before
        // this slab's DMA refills it; iteration 0 keeps a barrier for the scale buffer the set-up has just read.
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
        float e_nxt[2] = {1.0f, 1.0f};                       // scales of the next slab (landed one slab ago)
        float hr_n[2] = {1.0f, 1.0f};                        // boundary factors of the next iteration
        // scale buffers: per-token source, slab s in buffer s & 1 (its scales are taken into registers one slab ahead);
        // per-channel source, slab s in buffer s % 3 (its factors are read all through its own iteration)
        const int sb_dma = PC ? (it + 2) % 3 : (it & 1);
        const int sb_cur = it % 3, sb_nxt = (it + 1) % 3;
        __builtin_amdgcn_sched_barrier(0);

        static_for<0, NT * 16>([&](auto SIDX) XQ_INLINE_LAMBDA {
            constexpr int sidx = decltype(SIDX)::value;
            constexpr int j = sidx >> 4, ct = sidx & 15;
            constexpr int ring = (j - tile16_lag(ct)) & (NT - 1);
            acc[0][ct] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                __builtin_bit_cast(f16x8, af[sidx % NRING]), as_frag(ub[0][ring][0], ub[0][ring][1], ub[0][ring][2], ub[0][ring][3]),
                acc[0][ct], 0, 0, 0);
            acc[1][ct] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                __builtin_bit_cast(f16x8, af[sidx % NRING]), as_frag(ub[1][ring][0], ub[1][ring][1], ub[1][ring][2], ub[1][ring][3]),
                acc[1][ct], 0, 0, 0);

            // DMA of the next slab: 11 steps per wave, one every other slot
            if constexpr ((sidx >> 1) < 11 && (sidx & 1) == 0)
                dma_step(sidx >> 1, s_next, img_next, s_next2, true, sb_dma, wdst);
            // the old codes are no longer needed: wait until the next slab has landed for everyone,
            // then take the next slab's codes
            if constexpr (sidx == 64 - AHEAD) {               // (after the last read of this slab's weights, before the first of the next's)
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                __syncthreads();
                if (more_main) fetch_tokens(img_next);
            }
            // weight fragment of the slot AHEAD ahead (the last slots of a slab read the next slab, which has landed by then)
            if constexpr (sidx + AHEAD < 64) af[(sidx + AHEAD) % NRING] = *reinterpret_cast<const uint4*>(slab + (sidx + AHEAD) * 1024);
            else if (more_main) af[(sidx + AHEAD) % NRING] = *reinterpret_cast<const uint4*>(slab_next + (sidx + AHEAD - 64) * 1024);
            // token fragments, half a fragment (two operand dwords) per slot in the four slots of every tick that
            // rescale nothing.  Tick j + 1's ring entry was last read by tick j's tiles 0-3 (lag 3) and is first
            // read by tick j + 1's tiles 12-15; tick 0's is made in the slab's first four slots, from the codes
            // taken out of LDS at the end of the previous slab.
            // (per-channel source: the tick's factors come out of LDS four slots before its first half fragment)
            if constexpr (PC && j + 1 < NT && ct == 8 - 4 * j) fetch_tick_factors(sb_cur, j + 1);
            if constexpr (PC && sidx == 61) fetch_tick_factors(sb_nxt, 0);
            if constexpr (sidx < 4) make_half_fragment(std::integral_constant<int, (sidx >> 1)>{}, std::integral_constant<int, 0>{}, std::integral_constant<int, (sidx & 1)>{});
            if constexpr (j + 1 < NT && ct >= 12 - 4 * j && ct < 16 - 4 * j)
                make_half_fragment(std::integral_constant<int, ((ct - (12 - 4 * j)) >> 1)>{}, std::integral_constant<int, j + 1>{}, std::integral_constant<int, ((ct - (12 - 4 * j)) & 1)>{});
            // the next slab's scales are in LDS since the previous slab
            if constexpr (!PC && sidx == 40) {
                if (more_main) {
                    // (groups of 64: the slab's last fragment was made in slot 39, the factors may be replaced)
                    if constexpr (G == 64) fetch_factors((it + 1) & 1, fac);
                    else fetch_scales((it + 1) & 1, e_nxt);
                }
            }
            if constexpr (G == 128 && !PC && sidx == 58) {
                if (more_main) { hr_n[0] = E_cur[0] * __builtin_amdgcn_rcpf(e_nxt[0]); hr_n[1] = E_cur[1] * __builtin_amdgcn_rcpf(e_nxt[1]); }
            }
            // Horner: the four tiles that enter this slab's group at tick jj (tiles 4 (3 - jj) + i) are rescaled half
            // a tile per slot in the eight slots 12 jj + 4 + [0, 8): after the tile's MFMAs of the previous tick
            // have long retired, before its slot of tick jj, and in none of the slots that unpack codes
            if constexpr (G == 128 && !PC) {
                constexpr int r = sidx - 4, jj = r / 12, o = r % 12;
                if constexpr (sidx >= 4 && jj < NT && o < 8) {
                    constexpr int s = o & 1, ct2 = 4 * (3 - jj) + (o >> 1);
                    static_assert(tile16_lag(ct2) == jj && sidx < 16 * jj + ct2 && sidx + 16 > 16 * jj + ct2 + 2, "Horner slot outside the tile's window");
                    float x0 = acc[s][ct2][0] * hr[s], x1 = acc[s][ct2][1] * hr[s], x2 = acc[s][ct2][2] * hr[s], x3 = acc[s][ct2][3] * hr[s];
                    asm volatile("" :: "v"(x0), "v"(x1), "v"(x2), "v"(x3));
                    acc[s][ct2][0] = x0; acc[s][ct2][1] = x1; acc[s][ct2][2] = x2; acc[s][ct2][3] = x3;
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        if (more_main && !PC) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                if constexpr (G == 128) { E_prev[s] = E_cur[s]; E_cur[s] = e_nxt[s]; hr[s] = hr_n[s]; }
            }
        }
    }
    // every tile has ended in the last slab's group (groups of 64: the token's units all along); leave that scale:
    // the accumulator is K | V
    if constexpr (PC) {
        // K | V = accumulator * 2^(E_blk + bits - 1) + z_blk [Wk_h | Wv_h]; waves past len take the last block's
        const int blk = min((c.tile * TILE_TOKENS + wave * CHUNK_TOKENS) / p.pc_block, (c.len - 1) / p.pc_block);
        const long long brow = (long long)c.b * p.pc_blocks_cap + blk;
        const float fs = ldexpf(p.pc_fscale[brow], -head_shift);
        const float* zw = p.pc_zw + (brow * p.grid_heads + c.hk) * 256 + 4 * q;
#pragma unroll
        for (int ct = 0; ct < 16; ++ct) {
            const float4 z = *reinterpret_cast<const float4*>(zw + 16 * ct);
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                acc[s][ct][0] = __builtin_fmaf(acc[s][ct][0], fs, z.x);
                acc[s][ct][1] = __builtin_fmaf(acc[s][ct][1], fs, z.y);
                acc[s][ct][2] = __builtin_fmaf(acc[s][ct][2], fs, z.z);
                acc[s][ct][3] = __builtin_fmaf(acc[s][ct][3], fs, z.w);
            }
        }
    } else {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const float f = G == 64 ? ldexpf(tok_norm[s], -head_shift - 15) : ldexpf(E_cur[s], -head_shift);
#pragma unroll
            for (int ct = 0; ct < 16; ++ct) acc[s][ct] *= f;
        }
    }
    // (after the last barrier of the walk nothing reads or writes the slab buffers any more)
    if constexpr (MODE == MODE_PREFILL) prefill_epilogue16(p, c, acc, lds);
    else if constexpr (MODE == MODE_WEIGHTED_SUM) weighted_sum_epilogue16(p, c, acc, lds);
    else attention_epilogue16(p, c, acc);
}

// =====================================================================================
// Dense source (the bf16 accumulator of XQuant-CL, Sec. 3.2) on the same 16 x 16 tiles: no codes, no scales,
// no lag -- slab s, tick j multiplies channels 128 s + 32 j + [0, 32) for every tile.  A wave needs, per half
// slab (2 ticks = 64 channels), 128 contiguous bytes of each of its 32 token rows: 4 LDS-DMA instructions
// fetch 8 rows x 128 B each into a 4 KiB staging area private to the wave (the hand-over needs s_waitcnt, no
// barrier), and 4 ds_read_b128 per lane bring the fragments into registers -- lane (c16, q) takes, of token
// 16 s + c16, the 16 bytes of quarter q of tick jj.  The 16-byte piece p of row r of block j (tokens 8 j ..
// 8 j + 7) sits in slot 8 (r % 8) + (p ^ f), f = ((r % 8) >> 1) | ((j & 1) << 2), which keeps both the
// DMA's linear LDS write and the fragment read free of bank conflicts.
// Per half slab (32 slots): slot 16 takes the fragments of the next half out of staging, slot 20 issues the
// DMA of the half after it.
// =====================================================================================
constexpr int LDS_DENSE16_STAGE_OFF = 2 * SLAB_BYTES;
constexpr int LDS_DENSE16_STAGE_BYTES = 4096;          // per wave
constexpr int LDS_DENSE16_TOTAL = LDS_DENSE16_STAGE_OFF + 8 * LDS_DENSE16_STAGE_BYTES;
static_assert(LDS_DENSE16_TOTAL <= LDS_MAX, "dense kernel LDS");

template <int MODE>
__global__ __launch_bounds__(512) void remat_attn_dense16_kernel(const RematParams p)
{
    constexpr int AHEAD = 5;                           // slots between the LDS read of a weight fragment and its use
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    TileCtx c;
    if (!locate_tile(p, c)) return;
    const int lane = c.lane, wave = c.wave;
    const int c16 = lane & 15, q = lane >> 4;

    const uint8_t* wsrc = p.wprep + (long long)c.hk * p.head_bytes + wave * 1024;
    const uint32_t dma_voff = (uint32_t)lane * 16u;
    const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) uint8_t*)lds;
    const uint32_t lds_w = lds_base + wave * 1024;
    const uint8_t* my_slab = lds + lane * 16;
    const uint8_t* cbase = reinterpret_cast<const uint8_t*>(p.acc) + (long long)c.b * p.cap * p.d * 2;
    const uint32_t row_bytes = (uint32_t)p.d * 2u;
    const int n_halves = 2 * p.n_main_slabs;

    // DMA side: lane = (row r8 of the block, slot column); block j covers the wave's tokens 8 j .. 8 j + 7
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
    const uint32_t stage = lds_base + LDS_DENSE16_STAGE_OFF + wave * LDS_DENSE16_STAGE_BYTES;
    // fragment side: token 16 s + c16 is row c16 % 8 of block 2 s + c16 / 8; piece 4 jj + q
    const uint8_t* my_stage = lds + LDS_DENSE16_STAGE_OFF + wave * LDS_DENSE16_STAGE_BYTES + (c16 >> 3) * 1024 + (c16 & 7) * 128;
    const int fx = ((c16 & 7) >> 1) | ((c16 >> 3) << 2);
    auto issue_x = [&](int h) {                           // token rows of half slab h -> staging
        const int hc = min(h, n_halves - 1);              // (past the end: a harmless repeat)
        const uint8_t* src = cbase + (long long)hc * 128;
#pragma unroll
        for (int j = 0; j < 4; ++j) dma_b128(src, xvoff[j], stage + j * 1024);
    };
    auto take_x = [&](uint4 (&dst)[2][2]) {               // [token half s][tick jj of the half slab]
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
                dst[s][jj] = *reinterpret_cast<const uint4*>(my_stage + s * 2048 + (((4 * jj + q) ^ fx) * 16));
    };

    f32x4 acc[2][16];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int ct = 0; ct < 16; ++ct)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[s][ct][i] = 0.0f;

    uint4 af[8];                         // weight fragments, ring over slots (loaded AHEAD slots ahead)
    uint4 bd[2][2][2];                   // token fragments of the two halves of a slab

    issue_slab(wsrc, lds_w, dma_voff);
    issue_x(0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    take_x(bd[0]);
#pragma unroll
    for (int sl = 0; sl < AHEAD; ++sl) af[sl] = *reinterpret_cast<const uint4*>(my_slab + sl * 1024);
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
            constexpr int j = sidx >> 4, ct = sidx & 15;
            constexpr int hs = sidx & 31, hf = sidx >> 5;            // slot inside the half slab, which half
            acc[0][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                __builtin_bit_cast(bf16x8, af[sidx & 7]), __builtin_bit_cast(bf16x8, bd[hf][0][j & 1]), acc[0][ct], 0, 0, 0);
            acc[1][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                __builtin_bit_cast(bf16x8, af[sidx & 7]), __builtin_bit_cast(bf16x8, bd[hf][1][j & 1]), acc[1][ct], 0, 0, 0);
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
            // the next slab's weights have landed for everyone (its buffer was last read one slab ago, and this
            // slab's last fragment has been read in the slot before); the newest 4 DMAs, the token rows just
            // issued, may still be in flight
            if constexpr (sidx == 64 - AHEAD) {
                asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
                __syncthreads();
            }
            if constexpr (sidx + AHEAD < 64) af[(sidx + AHEAD) & 7] = *reinterpret_cast<const uint4*>(slab + (sidx + AHEAD) * 1024);
            else if (more_main) af[(sidx + AHEAD) & 7] = *reinterpret_cast<const uint4*>(slab_next + (sidx + AHEAD - 64) * 1024);
            __builtin_amdgcn_sched_barrier(0);
        });
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // nothing may still be writing this workgroup's LDS
    if constexpr (MODE == MODE_PREFILL) prefill_epilogue16(p, c, acc, lds);   // (starts with a workgroup barrier)
    else attention_epilogue16(p, c, acc);
}

static hipError_t allow_lds_once(const void* k, int lds_bytes, int slot)
{
    static std::mutex mu;
    static bool done[64][24];                     // [device][kernel: 4 format + mode; 16, 17: dense; 18-20: per-channel]
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!done[dev][slot]) {
        e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        done[dev][slot] = true;
    }
    return hipSuccess;
}

static_assert(PF16_TOTAL <= lds_coded_total(2) && PF16_TOTAL <= lds_coded_total(3) && PF16_TOTAL <= lds_coded_total(4) &&
              PF16_TOTAL <= LDS_DENSE16_TOTAL, "the matrix-core epilogue fits the LDS the contraction loop has");

// prefill: the matrix-core epilogue (many query rows) instead of the per-query-head vector epilogue
hipError_t launch_tile16_dense(const RematParams& p, int grid, hipStream_t s, bool prefill)
{
    typedef void (*Kernel)(const RematParams);
    const Kernel k = prefill ? remat_attn_dense16_kernel<MODE_PREFILL> : remat_attn_dense16_kernel<MODE_ATTENTION>;
    hipError_t e = allow_lds_once(reinterpret_cast<const void*>(k), LDS_DENSE16_TOTAL, prefill ? 17 : 16);
    if (e != hipSuccess) return e;
    k<<<dim3(grid), dim3(512), LDS_DENSE16_TOTAL, s>>>(p);
    return hipGetLastError();
}

typedef void (*Tile16Kernel)(const RematParams);
template <int BITS, int G>
static Tile16Kernel tile16_kernel_for(int mode)
{
    switch (mode) {
        case MODE_ATTENTION: return remat_attn_tile16_kernel<BITS, G, MODE_ATTENTION>;
        case MODE_PREFILL: return remat_attn_tile16_kernel<BITS, G, MODE_PREFILL>;
        case MODE_WEIGHTED_SUM: return remat_attn_tile16_kernel<BITS, G, MODE_WEIGHTED_SUM>;
    }
    return nullptr;
}

// mode: MODE_ATTENTION (decode, vector epilogue), MODE_PREFILL (matrix-core epilogue for many query rows),
// MODE_WEIGHTED_SUM (the second pass over a latent cache)
hipError_t launch_tile16(int bits, int G, const RematParams& p, int grid, hipStream_t s, int mode)
{
    Tile16Kernel k = nullptr;
    int format = -1;
    switch (bits * 1000 + G) {
        case 2128: k = tile16_kernel_for<2, 128>(mode); format = 0; break;
        case 3128: k = tile16_kernel_for<3, 128>(mode); format = 1; break;
        case 4128: k = tile16_kernel_for<4, 128>(mode); format = 2; break;
        case 2064: k = tile16_kernel_for<2, 64>(mode); format = 3; break;
    }
    if (!k) return hipErrorInvalidValue;
    const int mode_slot = mode == MODE_ATTENTION ? 0 : mode == MODE_PREFILL ? 1 : 2;
    const int lds_bytes = lds_coded_total(bits);
    const hipError_t e = allow_lds_once(reinterpret_cast<const void*>(k), lds_bytes, 4 * format + mode_slot);
    if (e != hipSuccess) return e;
    k<<<dim3(grid), dim3(512), lds_bytes, s>>>(p);
    return hipGetLastError();
}

// decode attention over the complete blocks of a per-channel cache (Sec. 3.3.1); the stream is that of groups of 128
hipError_t launch_tile16_per_channel(int bits, const RematParams& p, int grid, hipStream_t s)
{
    typedef void (*Kernel)(const RematParams);
    Kernel k = nullptr;
    switch (bits) {
        case 2: k = remat_attn_tile16_kernel<2, 128, MODE_ATTENTION_PC>; break;
        case 3: k = remat_attn_tile16_kernel<3, 128, MODE_ATTENTION_PC>; break;
        case 4: k = remat_attn_tile16_kernel<4, 128, MODE_ATTENTION_PC>; break;
        default: return hipErrorInvalidValue;
    }
    const int lds_bytes = lds_coded_total(bits);
    const hipError_t e = allow_lds_once(reinterpret_cast<const void*>(k), lds_bytes, 16 + bits);
    if (e != hipSuccess) return e;
    k<<<dim3(grid), dim3(512), lds_bytes, s>>>(p);
    return hipGetLastError();
}

}  // namespace xq
