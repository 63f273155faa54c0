// What a wave does with the 256 rematerialised columns of its 32 tokens once the contraction is done:
// decode attention (vector epilogue), attention for many query rows through the matrix cores (prefill),
// the two passes of the latent cache, the up-projecting accumulate of Sec. 3.3.2.
#pragma once
#include "remat_common.hpp"

namespace xq {

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

// V^T images of the wave's 32 tokens from four accumulator blocks: element i of block nb is V[token tl][n],
// n = 32 nb + 8 (i/4) + 4 half + i%4
__device__ __forceinline__ void write_v_images(uint8_t* vt, const TileCtx& c, const f32x16& v0, const f32x16& v1,
                                               const f32x16& v2, const f32x16& v3)
{
    const f32x16* blocks[4] = {&v0, &v1, &v2, &v3};
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int n = nb * 32 + (i >> 2) * 8 + c.half * 4 + (i & 3);
            const float v = (*blocks[nb])[i];
            const uint32_t h = pack_bf16x2_rne(v, 0.0f);
            uint8_t* dst = vt + vt_offset(n, c.tl >> 2) + (c.tl & 3) * 2;
            *reinterpret_cast<uint16_t*>(dst) = (uint16_t)h;
            *reinterpret_cast<uint16_t*>(dst + VT_IMAGE_BYTES) = (uint16_t)pack_bf16x2_rne(v - bf16_lo_to_f32(h), 0.0f);
        }
}

// Second half of the matrix-core epilogue for one group of up to 32 query rows (row q0 + lane % 32 in this
// lane): given the wave's chunk maximum m, sum l and weights pr (register r <-> token 8 (r/4) + 4 half + r%4,
// relative to m) it forms P V against the wave's V images, merges the eight waves of the workgroup (maxima and
// sums through LDS, rescaled O blocks summed in fixed wave order through the staging area) and stores one
// partial per query row and tile.  part_row(query index) gives the row's index in the partial buffers; rows at
// or past n_rows are not stored.  Called by all eight waves (workgroup barriers inside).
template <class PartRow>
__device__ __forceinline__ void pv_merge_store(const RematParams& p, const TileCtx& c, uint8_t* lds, const uint8_t* vt,
                                               bool active, float m, float l, const float (&pr)[16], int q0, int n_rows,
                                               PartRow part_row)
{
    const int jq = c.tl;
    float* mbuf = reinterpret_cast<float*>(lds + PF_STAGE_OFF);            // [wave][32 queries]
    float* lbuf = mbuf + 8 * 32;
    float* stage = reinterpret_cast<float*>(lds + PF_STAGE_OFF);           // [wave][16][64]
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
    const float f = __builtin_amdgcn_exp2f(m - Mu);                        // per lane-query
    __syncthreads();                                                       // mbuf / lbuf are reused as staging
    if (c.wave == 0 && c.half == 0 && q0 + jq < n_rows) {
        const long long pidx = part_row(q0 + jq) * p.chunks_per_seq + c.tile;
        p.part_ml[pidx * 2] = M;
        p.part_ml[pidx * 2 + 1] = Lt;
    }
    uint4 phi[2], plo[2];
    float fr[16];                                                          // the factor of register r's query
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
            if (qr < n_rows) p.part_o[(part_row(qr) * p.chunks_per_seq + c.tile) * 128 + nb * 32 + jq] = sum;
        }
        __syncthreads();
    }
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
        write_v_images(vt, c, acc[4], acc[5], acc[6], acc[7]);
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
    auto part_row = [&](int qi) -> long long {
        const int tq = qi / gq;
        return ((long long)c.b * p.Tq + tq) * p.Hq + c.hk * gq + (qi - tq * gq);
    };
    for (int q0 = 0; q0 < NQ; q0 += 32) {
        // this lane's query row of the group (rows past NQ repeat the last one and are not stored)
        const int qi = min(q0 + jq, NQ - 1);
        const int tq = qi / gq;
        const long long qrow = part_row(qi);
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
        pv_merge_store(p, c, lds, vt, active, m, l, pr, q0, NQ, part_row);
    }
}

// ---- latent cache (Sec. 3.3.1), pass 1: the wave holds the keys of two KV heads of its 32 tokens
// (blocks 0-3: head 2 pair, blocks 4-7: head 2 pair + 1) and stores the scaled scores of their
// query heads; pass 2 turns them into softmax partials against the values.
// The epilogue is bound by vector-instruction issue (all eight waves are in it at once), so the query vectors of the
// pair's heads (contiguous in q) are first converted to fp32 and put into LDS -- `qstage`, a region of qstage_bytes
// that only this wave touches any more: a head then costs 16 ds_read_b128 and 64 fma per lane, without the
// conversions and without one memory latency per head.  Pairs with more query heads than fit read q from memory.
__device__ __forceinline__ void scores_epilogue(const RematParams& p, const TileCtx& c, f32x16 (&acc)[8], uint8_t* qstage,
                                                int qstage_bytes)
{
    if (c.tile * TILE_TOKENS + c.wave * CHUNK_TOKENS >= c.len) return;
    const int gq = p.Hq / p.Hkv;
    const long long srow = p.score_stride;
    const int tok_out = p.tok0.v[c.b] + c.tok;
    const uint16_t* qpair = p.q + ((long long)c.b * p.Hq + 2 * c.hk * gq) * 128;     // 2 gq heads x 128 bf16
    const int n_q = 2 * gq * 128;
    const bool staged = n_q * 4 <= qstage_bytes && (reinterpret_cast<size_t>(p.q) & 15) == 0;   // (wave-uniform)
    float* qf = reinterpret_cast<float*>(qstage);
    if (staged) {
        for (int i0 = c.lane * 8; i0 < n_q; i0 += 512) {
            const uint4 v = *reinterpret_cast<const uint4*>(qpair + i0);
            float4 lo, hi;
            lo.x = bf16_lo_to_f32(v.x); lo.y = bf16_hi_to_f32(v.x); lo.z = bf16_lo_to_f32(v.y); lo.w = bf16_hi_to_f32(v.y);
            hi.x = bf16_lo_to_f32(v.z); hi.y = bf16_hi_to_f32(v.z); hi.z = bf16_lo_to_f32(v.w); hi.w = bf16_hi_to_f32(v.w);
            *reinterpret_cast<float4*>(qf + i0) = lo;
            *reinterpret_cast<float4*>(qf + i0 + 4) = hi;
        }
        __builtin_amdgcn_wave_barrier();
    }
    static_for<0, 2>([&](auto HH) XQ_INLINE_LAMBDA {       // (compile-time: the accumulator must stay in registers)
        constexpr int hh = decltype(HH)::value;
        for (int j = 0; j < gq; ++j) {
            const int hq = (2 * c.hk + hh) * gq + j;
            float dot = 0.0f;
            if (staged) {
                const float* qv = qf + (hh * gq + j) * 128 + c.half * 4;
#pragma unroll
                for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                    for (int i4 = 0; i4 < 4; ++i4) {
                        const float4 qq = *reinterpret_cast<const float4*>(qv + nb * 32 + i4 * 8);
                        const f32x16& a = acc[4 * hh + nb];
                        dot = __builtin_fmaf(qq.x, a[i4 * 4 + 0], dot);
                        dot = __builtin_fmaf(qq.y, a[i4 * 4 + 1], dot);
                        dot = __builtin_fmaf(qq.z, a[i4 * 4 + 2], dot);
                        dot = __builtin_fmaf(qq.w, a[i4 * 4 + 3], dot);
                    }
            } else {
                const uint16_t* qv = p.q + ((long long)c.b * p.Hq + hq) * 128;
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
            }
            const float sc = (dot + __shfl_xor(dot, 32)) * p.scale_log2e;
            if (c.half == 0 && c.tok < c.len) p.scores[((long long)c.b * p.Hq + hq) * srow + tok_out] = sc;
        }
    });
}

// pass 2: blocks 0-3 / 4-7 hold the values of the two KV heads.  Per head, the stored scores of its query
// heads (lane = query head, registers = 16 of the wave's 32 tokens) become softmax weights and go through the
// second half of the matrix-core epilogue: one partial (m, l, o[128]) per query head and tile.
// Called by all eight waves of the workgroup.
__device__ __forceinline__ void weighted_sum_epilogue(const RematParams& p, const TileCtx& c, f32x16 (&acc)[8], uint8_t* lds)
{
    const int tok0 = c.tile * TILE_TOKENS + c.wave * CHUNK_TOKENS;
    const bool active = tok0 < c.len;
    uint8_t* vt = lds + c.wave * VT_WAVE_BYTES;
    const int gq = p.Hq / p.Hkv;
    const long long srow = p.score_stride;
    static_for<0, 2>([&](auto HH) XQ_INLINE_LAMBDA {       // (compile-time: the accumulator must stay in registers)
        constexpr int hh = decltype(HH)::value;
        const int hq0 = (2 * c.hk + hh) * gq;
        if (active) write_v_images(vt, c, acc[4 * hh], acc[4 * hh + 1], acc[4 * hh + 2], acc[4 * hh + 3]);
        __builtin_amdgcn_wave_barrier();
        auto part_row = [&](int qi) -> long long { return (long long)c.b * p.Hq + hq0 + qi; };
        float m = -INFINITY, l = 0.0f;
        float pr[16];
        if (active) {
            const float* sp = p.scores + ((long long)c.b * p.Hq + hq0 + min(c.tl, gq - 1)) * srow + tok0 + c.half * 4;
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                // tokens tok0 + 8 i4 + 4 half + [0, 4): 16 bytes; past len the buffer holds other rows' or stale values
                const float4 s4 = *reinterpret_cast<const float4*>(sp + 8 * i4);
                const float sv[4] = {s4.x, s4.y, s4.z, s4.w};
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int tok = tok0 + 8 * i4 + 4 * c.half + k;
                    pr[4 * i4 + k] = tok < c.len ? sv[k] : -INFINITY;
                    m = fmaxf(m, pr[4 * i4 + k]);
                }
            }
            m = fmaxf(m, __shfl_xor(m, 32));
            const float mu = m == -INFINITY ? 0.0f : m;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                pr[r] = __builtin_amdgcn_exp2f(pr[r] - mu);
                l += pr[r];
            }
            l += __shfl_xor(l, 32);
        }
        pv_merge_store(p, c, lds, vt, active, m, l, pr, 0, gq, part_row);
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

}  // namespace xq
