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
#include "remat_common.hpp"
#include "remat_epilogues.hpp"

namespace xq {

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
// MODE_SCORES_PC (pass 1 of the latent path with per-channel keys; the decode attention over a per-channel X
// cache, MODE_ATTENTION_PC, runs the same scheme on the 16 x 16 tiles of remat_attn16.hip) reads a per-channel
// cache (Sec. 3.3.1: one scale and zero-point per channel and block of 64 or 128 tokens).  The scale now varies along the contraction, so it moves to the token
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
    const int head_shift = p.head_shift[c.hk];         // the head's stream holds its weights times 2^head_shift
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
    const bool vec_meta = (p.ng & 7) == 0 && (p.ng_row & 7) == 0 && ((size_t)zbase & 15) == 0 && p.meta_shift == 0;
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
                    const uint32_t x = mbase[moff + (min(g, p.ng - 1) >> p.meta_shift)];
                    h[i] = g < p.ng ? x : 0u;               // padding groups contribute nothing
                }
                v.x = h[0] | (h[1] << 16); v.y = h[2] | (h[3] << 16);
                v.z = h[4] | (h[5] << 16); v.w = h[6] | (h[7] << 16);
            }
        }
        return v;
    };
    const int slab_prev = p.n_main_slabs - 1;           // the walk is cyclic: the slab "before" slab 0
    issue_slab_chunks(wsrc + (long long)p.n_main_slabs * SLAB_BYTES, lds_w, dma_voff,  // correction slab 0 -> buffer 0
                      min(SLAB_KSTEPS, p.n_corr_ksteps));                              // (a chunk is a k-step)
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
        // The zero-points have arrived with that wait, but the compiler counts only its own loads, not the DMA: left
        // alone it waits for them at their first use, with vmcnt(0), behind the DMA issued next, and the correction
        // would start only after that slab has landed.  Using the registers here puts its wait here, where it is free.
        if constexpr (!PC) {
#pragma unroll
            for (int kh = 0; kh < 2; ++kh)
                asm volatile("" :: "v"(mfr[4 * kh].x), "v"(mfr[4 * kh].y), "v"(mfr[4 * kh].z), "v"(mfr[4 * kh].w),
                                   "v"(mfr[4 * kh + 1].x), "v"(mfr[4 * kh + 1].y), "v"(mfr[4 * kh + 1].z), "v"(mfr[4 * kh + 1].w),
                                   "v"(mfr[4 * kh + 2].x), "v"(mfr[4 * kh + 2].y), "v"(mfr[4 * kh + 2].z), "v"(mfr[4 * kh + 2].w),
                                   "v"(mfr[4 * kh + 3].x), "v"(mfr[4 * kh + 3].y), "v"(mfr[4 * kh + 3].z), "v"(mfr[4 * kh + 3].w));
        }
        const uint32_t wdst = lds_w + (uint32_t)(((cs + 1) & 1) * SLAB_BYTES);
        if (cs + 1 < n_corr_slabs)
            issue_slab_chunks(wsrc + (long long)(p.n_main_slabs + cs + 1) * SLAB_BYTES, wdst, dma_voff,
                              min(SLAB_KSTEPS, p.n_corr_ksteps - (cs + 1) * SLAB_KSTEPS));
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
                const float r0 = ldexpf(__builtin_amdgcn_rcpf(E[floordiv_c(j - 8, KSG) + GPS]), head_shift);
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
        const float fs = ldexpf(p.pc_fscale[brow], -head_shift);
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
        for (int j = 0; j < 8; ++j) acc[j] *= ldexpf(E[GPS + j / KSG], -head_shift);
    }
    // (after the last barrier of the walk nothing reads or writes the slab buffers any more)
    if constexpr (MODE == MODE_SCORES || MODE == MODE_SCORES_PC) scores_epilogue(p, c, acc, lds + wave * 8192, 8192);
    else if constexpr (MODE == MODE_WEIGHTED_SUM) weighted_sum_epilogue(p, c, acc, lds);
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
// pair of KV heads) for the rows of a residual window, 4 store the rows as bf16 (a plain GEMM: the bulk
// projection into the latent space)
constexpr int DENSE_ATTENTION = 0, DENSE_PREFILL = 1, DENSE_STORE = 2, DENSE_SCORES = 3, DENSE_STORE_BF16 = 4;
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
    // second source of the bf16 store mode (rows of another tensor, subtracted): its row offsets and base
    uint32_t xvoff2[4] = {0u, 0u, 0u, 0u};
    const uint8_t* cbase2 = nullptr;
    int split_halves = 0x7FFFFFFF;                        // first half slab that reads the second source
    if constexpr (DMODE == DENSE_STORE_BF16) {
        if (p.acc2) {
            cbase2 = reinterpret_cast<const uint8_t*>(p.acc2);
            split_halves = 2 * p.w_slabs;
            const int r8 = lane >> 3, sc = lane & 7;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int piece = sc ^ ((r8 >> 1) | ((j & 1) << 2));
                const int tok = min(c.tile * TILE_TOKENS + wave * CHUNK_TOKENS + 8 * j + r8, c.len - 1);
                const int sb = tok / p.Tq, st = tok - sb * p.Tq;
                const uint32_t row2 = (uint32_t)sb * (uint32_t)p.cap2 + (uint32_t)(p.tok0.v[sb] + st);
                xvoff2[j] = row2 * row_bytes + (uint32_t)piece * 16u;
            }
        }
    }
    const uint32_t stage = lds_base + LDS_DENSE_STAGE_OFF + wave * LDS_DENSE_STAGE_BYTES;
    // fragment side: this lane's token tl, k-step kk of the half slab -> piece 2 kk + half
    const uint8_t* my_stage = lds + LDS_DENSE_STAGE_OFF + wave * LDS_DENSE_STAGE_BYTES + (tl >> 3) * 1024 + (tl & 7) * 128;
    const int fx = ((tl & 7) >> 1) | (((tl >> 3) & 1) << 2);
    auto issue_x = [&](int h) {                           // token rows of half slab h -> staging
        const int hc = min(h, n_halves - 1);              // (past the end: a harmless repeat)
        if (DMODE == DENSE_STORE_BF16 && hc >= split_halves) {
            const uint8_t* src = cbase2 + (long long)(hc - split_halves) * 128;
#pragma unroll
            for (int j = 0; j < 4; ++j) dma_b128(src, xvoff2[j], stage + j * 1024);
        } else {
            const uint8_t* src = cbase + (long long)hc * 128;
#pragma unroll
            for (int j = 0; j < 4; ++j) dma_b128(src, xvoff[j], stage + j * 1024);
        }
    };
    auto take_x = [&](uint4 (&dst)[4], int h) {           // h: the half slab these rows belong to
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            dst[kk] = *reinterpret_cast<const uint4*>(my_stage + (((2 * kk + half) ^ fx) * 16));
        if (DMODE == DENSE_STORE_BF16 && h >= split_halves) {          // the second source is subtracted
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                dst[kk].x ^= 0x80008000u; dst[kk].y ^= 0x80008000u; dst[kk].z ^= 0x80008000u; dst[kk].w ^= 0x80008000u;
            }
        }
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
    take_x(bd[0], 0);
#pragma unroll
    for (int sl = 0; sl < 7; ++sl) af[sl] = *reinterpret_cast<const uint4*>(my_slab + sl * 1024);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // staging has been read: it may be refilled
    issue_x(1);

    for (int it = 0; it < p.n_main_slabs; ++it) {
        const bool more_main = it + 1 < p.n_main_slabs;
        const int s_next = more_main ? it + 1 : it;       // (the last iteration repeats itself into unused buffers)
        const uint32_t wdst = lds_w + (uint32_t)(((it + 1) & 1) * SLAB_BYTES);
        // (bf16 store mode with a second source: the weight stream is walked a second time)
        const int s_w = (DMODE == DENSE_STORE_BF16 && s_next >= p.w_slabs) ? s_next - p.w_slabs : s_next;
        const uint8_t* wnext = wsrc + (long long)s_w * SLAB_BYTES;
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
                take_x(bd[hf ^ 1], 2 * it + hf + 1);
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
    } else if constexpr (DMODE == DENSE_STORE_BF16) {
        // a plain bf16 GEMM row block: out[token][256 hk + column], one RNE rounding (the bulk projection X U)
        if (c.tok < c.len) {
            uint16_t* row = p.rows_out + ((long long)c.tok * p.grid_heads + c.hk) * 256 + c.half * 4;
#pragma unroll
            for (int nb = 0; nb < 8; ++nb)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    uint2 v;
                    v.x = pack_bf16x2_rne(acc[nb][i4 * 4], acc[nb][i4 * 4 + 1]);
                    v.y = pack_bf16x2_rne(acc[nb][i4 * 4 + 2], acc[nb][i4 * 4 + 3]);
                    *reinterpret_cast<uint2*>(row + nb * 32 + i4 * 8) = v;
                }
        }
    } else if constexpr (DMODE == DENSE_SCORES) {
        scores_epilogue(p, c, acc, lds + LDS_DENSE_STAGE_OFF + wave * LDS_DENSE_STAGE_BYTES, LDS_DENSE_STAGE_BYTES);   // (the wave's own, idle now)
    } else {
        attention_epilogue(p, c, acc);
    }
}

// ---- pre-pass of the coded kernel: effective scales e = 2^(bits+14) * scale (1 for a zero scale)
// as bf16, laid out [sequence][tile][group (+1 pad)][256 tokens] so that a tile's scales of
// one group are contiguous (tokens past len repeat the last row).
__global__ __launch_bounds__(256) void scale_transpose_kernel(const uint16_t* __restrict__ scale,
                                                              uint16_t* __restrict__ eT, int cap, int ng,
                                                              int ng_row, int tiles_per_seq, int bits, BatchI32 len,
                                                              int meta_shift = 0, bool with_normaliser = false)
{
    const int tile = blockIdx.x, b = blockIdx.y, t = threadIdx.x;
    const int L = len.v[b];
    if (tile * TILE_TOKENS >= L) return;
    const long long row = (long long)b * cap + min(tile * TILE_TOKENS + t, L - 1);
    uint16_t* dst = eT + ((long long)b * tiles_per_seq + tile) * (long long)(ng + 1) * TILE_TOKENS + t;
    uint32_t emax = 0;                                // (positive bf16 bit patterns order as integers)
    for (int g = 0; g < ng; ++g) {
        const uint32_t sb = scale[row * ng_row + (g >> meta_shift)];
        const uint32_t e = sb ? sb + ((uint32_t)(bits + F16_SUBNORMAL_EXP - F16_MANT_BITS) << 7) : 0x3F80u;
        dst[(long long)g * TILE_TOKENS] = (uint16_t)e;
        emax = max(emax, e);
    }
    // spare group row (fetched with the last slab's scales, not used as a scale): 1, or on request the token's
    // normaliser, the power of two at or above its largest effective scale
    const uint32_t norm = (emax & 0x7F80u) + ((emax & 0x7Fu) ? 0x80u : 0u);
    dst[(long long)ng * TILE_TOKENS] = with_normaliser ? (uint16_t)norm : (uint16_t)0x3F80u;
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

// The same merge for partials that come one per 256-token tile (the matrix-core epilogue: prefill chunks, decode with
// many query heads per KV head): few per row but many rows.  One wave per row (query token, head), two output columns
// per lane, four rows per workgroup, no LDS; the tiles are summed in order (deterministic).
__global__ __launch_bounds__(256) void combine_rows_kernel(const float* __restrict__ part_o,
                                                           const float* __restrict__ part_ml,
                                                           float* __restrict__ out, int Hq, int chunks_per_seq,
                                                           BatchI32 len, int rows_per_seq, int chunk_tokens, int n_rows)
{
    const int row = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
    const int lane = threadIdx.x & 63;
    if (row >= n_rows) return;
    const int seq = row / (Hq * rows_per_seq);
    const int nchunks = (len.v[seq] + chunk_tokens - 1) / chunk_tokens;
    const long long base = (long long)row * chunks_per_seq;
    float M = -INFINITY;
    for (int c = 0; c < nchunks; ++c) M = fmaxf(M, part_ml[(base + c) * 2]);
    float L = 0.0f, ox = 0.0f, oy = 0.0f;
#pragma unroll 4
    for (int c = 0; c < nchunks; ++c) {
        const float w = __builtin_amdgcn_exp2f(part_ml[(base + c) * 2] - M);
        const float2 o = *reinterpret_cast<const float2*>(part_o + (base + c) * 128 + 2 * lane);
        L = __builtin_fmaf(w, part_ml[(base + c) * 2 + 1], L);
        ox = __builtin_fmaf(w, o.x, ox);
        oy = __builtin_fmaf(w, o.y, oy);
    }
    float2 r; r.x = ox / L; r.y = oy / L;
    *reinterpret_cast<float2*>(out + (long long)row * 128 + 2 * lane) = r;
}

}  // namespace xq

#include "remat_launch.hpp"
