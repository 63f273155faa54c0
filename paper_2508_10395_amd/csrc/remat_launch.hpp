// Host side of the rematerialisation kernels: workspace sizes, kernel parameters, launches.  Included at the
// end of remat_attn.hip (the kernels are templates of that translation unit).
#pragma once
#include <mutex>
#include <vector>

namespace xq {

// the per-head shift array of a prepared stream (after the slabs and the column sums)
static const int32_t* stream_shifts(const void* wprep, const WPrepLayout& L)
{
    return reinterpret_cast<const int32_t*>(static_cast<const uint8_t*>(wprep) + L.stream_bytes + L.colsum_bytes);
}

// Kernels that use more than 64 KiB of LDS must be told so once (per device); remember which have been.
static hipError_t allow_large_lds(const void* kernel, int lds_bytes)
{
    struct Done { const void* kernel; int device; int bytes; };
    static std::mutex mu;
    static std::vector<Done> done;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    for (const Done& d : done)
        if (d.kernel == kernel && d.device == dev && d.bytes >= lds_bytes) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e == hipSuccess) done.push_back({kernel, dev, lds_bytes});
    return e;
}

template <typename K>
static hipError_t launch_with_lds(K kernel, int lds_bytes, const RematParams& p, int grid, hipStream_t s)
{
    hipError_t e = allow_large_lds(reinterpret_cast<const void*>(kernel), lds_bytes);
    if (e != hipSuccess) return e;
    kernel<<<dim3(grid), dim3(512), lds_bytes, s>>>(p);
    return hipGetLastError();
}

// (d, group): of the walk -- for an 8-bit cache twice the hidden size and 128, see make_wprep_layout_for_cache
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

// the matrix-core epilogues lay their own images over the whole LDS once the contraction is done
template <int MODE>
constexpr int lds_for_mode(int bits)
{
    return (MODE == MODE_PREFILL || MODE == MODE_WEIGHTED_SUM) && LDS_PREFILL_TOTAL > lds_coded_total(bits)
               ? LDS_PREFILL_TOTAL : lds_coded_total(bits);
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

// the kernels on 16 x 16 x 32 MFMAs (remat_attn16.hip): groups of 128 codes (2-bit: also 64) or the dense source;
// mode = MODE_ATTENTION, MODE_PREFILL (the matrix-core epilogue for many query rows instead of the per-query-head
// vector epilogue) or MODE_WEIGHTED_SUM (the second pass over a latent cache)
hipError_t launch_tile16(int bits, int G, const RematParams& p, int grid, hipStream_t s, int mode);
hipError_t launch_tile16_dense(const RematParams& p, int grid, hipStream_t s, bool prefill);
hipError_t launch_tile16_per_channel(int bits, const RematParams& p, int grid, hipStream_t s);

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
    const int cache_bits = xc ? xc->fmt.bits : 16;
    const int bits = cache_bits == 8 ? 4 : cache_bits;                   // (an 8-bit cache is walked nibble by nibble)
    const int G = cache_bits == 8 ? 128 : xc ? xc->fmt.group : 128;
    const WPrepLayout L = make_wprep_layout_for_cache(d, xc ? xc->fmt.group : 128, cache_bits, a->n_kv_heads);
    RematParams p{};
    fill_common(p, a, q, B, cap, len, max_len, ws);
    p.codes = xc ? xc->codes : nullptr;
    p.zero = xc ? xc->zero : nullptr;
    p.acc = acc;
    p.wprep = static_cast<const uint8_t*>(wprep);
    p.head_shift = stream_shifts(wprep, L);
    p.d = L.d; p.row_d = L.d; p.grid_heads = p.Hkv;
    p.n_main_slabs = L.n_main_slabs; p.n_corr_ksteps = L.n_corr_ksteps; p.ng = L.ng; p.ng_pad = L.ng_pad;
    p.ng_row = xc ? d / xc->fmt.group : 0;
    p.meta_shift = (cache_bits == 8 && xc->fmt.group == 128) ? 1 : 0;
    p.head_bytes = (long long)L.head_bytes;
    p.rope = rope;
    if (rope) p.pos0 = *pos0;
    uint16_t* eT = reinterpret_cast<uint16_t*>(p.part_ml + (size_t)B * p.Hq * p.chunks_per_seq * 2);
    p.eT = eT;

    const int grid = p.Hkv * p.B * p.tiles_per_seq;
    hipError_t e = hipErrorInvalidValue;
    if (xc) {
        scale_transpose_kernel<<<dim3(p.tiles_per_seq, B), dim3(TILE_TOKENS), 0, s>>>(
            xc->scale, eT, cap, L.ng, p.ng_row, p.tiles_per_seq, bits, len, p.meta_shift, L.t16_bytes && G == 64);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        if (L.t16_bytes) {                                   // the stream of 16-column fragments and its kernel
            p.wprep += L.t16_offset;
            p.head_bytes = (long long)L.t16_head_bytes;
            p.n_corr_ksteps = L.t16_n_corr_ticks;
            e = launch_tile16(bits, G, p, grid, s, MODE_ATTENTION);
        } else {
            e = launch_coded<MODE_ATTENTION>(bits, G, p, grid, s);
        }
    } else {
        // bf16 token rows are 5 times the bytes of 3-bit codes and every head reads them: let the heads of an
        // XCD take the same tile side by side, so that its L2 serves all but the first (measured: 1.80 -> 1.66 ms
        // on the Llama-2-7B shape; the coded kernel gains nothing from it)
        p.tile_major = 1;
        if (L.t16_bytes) {
            p.wprep += L.t16_offset;
            p.head_bytes = (long long)L.t16_head_bytes;
            e = launch_tile16_dense(p, grid, s, false);
        } else {
            e = launch_with_lds(remat_attn_dense_kernel<DENSE_ATTENTION>, LDS_DENSE_TOTAL, p, grid, s);
        }
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
    const int cache_bits = xc ? xc->fmt.bits : 16;
    const int bits = cache_bits == 8 ? 4 : cache_bits;                   // (an 8-bit cache is walked nibble by nibble)
    const int G = cache_bits == 8 ? 128 : xc ? xc->fmt.group : 128;
    const WPrepLayout L = make_wprep_layout_for_cache(d, xc ? xc->fmt.group : 128, cache_bits, a->n_kv_heads);
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
    p.head_shift = stream_shifts(wprep, L);
    p.d = L.d; p.row_d = L.d; p.grid_heads = p.Hkv;
    p.n_main_slabs = L.n_main_slabs; p.n_corr_ksteps = L.n_corr_ksteps; p.ng = L.ng; p.ng_pad = L.ng_pad;
    p.ng_row = xc ? d / xc->fmt.group : 0;
    p.meta_shift = (cache_bits == 8 && xc->fmt.group == 128) ? 1 : 0;
    p.head_bytes = (long long)L.head_bytes;
    p.rope = rope;
    if (rope) p.pos0 = *pos0;
    const int grid = p.Hkv * p.B * p.tiles_per_seq;
    hipError_t e;
    if (xc) {
        scale_transpose_kernel<<<dim3(p.tiles_per_seq, B), dim3(TILE_TOKENS), 0, s>>>(
            xc->scale, const_cast<uint16_t*>(p.eT), cap, L.ng, p.ng_row, p.tiles_per_seq, bits, len, p.meta_shift,
            L.t16_bytes && G == 64);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        if (L.t16_bytes) {                                   // the stream of 16-column fragments and its kernel
            p.wprep += L.t16_offset;
            p.head_bytes = (long long)L.t16_head_bytes;
            p.n_corr_ksteps = L.t16_n_corr_ticks;
            e = launch_tile16(bits, G, p, grid, s, MODE_PREFILL);
        } else {
            e = launch_coded<MODE_PREFILL>(bits, G, p, grid, s);
        }
    } else {
        p.tile_major = 1;                                    // (as in the decode launch)
        if (L.t16_bytes) {
            p.wprep += L.t16_offset;
            p.head_bytes = (long long)L.t16_head_bytes;
            e = launch_tile16_dense(p, grid, s, true);
        } else {
            e = launch_with_lds(remat_attn_dense_kernel<DENSE_PREFILL>, LDS_DENSE_TOTAL, p, grid, s);
        }
    }
    if (e != hipSuccess) return e;
    const int n_rows = p.B * T * p.Hq;
    combine_rows_kernel<<<dim3((n_rows + 3) / 4), dim3(256), 0, s>>>(p.part_o, p.part_ml, out, p.Hq, p.chunks_per_seq, p.len, T,
                                                                    TILE_TOKENS, n_rows);
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
    const WPrepLayout L = make_wprep_layout_for_cache(r, G, bits, pairs);          // one stream per half, "head" = pair
    // pass 2 runs on the 16-column fragments where the format has them (that epilogue takes 16 query rows per KV head,
    // which is the most an attention descriptor may ask for)
    const bool t16 = L.t16_bytes != 0 && a->n_q_heads / a->n_kv_heads <= 16;
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

    const bool normaliser = t16 && G == 64;                 // (the scaled-operand loop wants the tokens' normalisers)
    scale_transpose_kernel<<<dim3(p.tiles_per_seq, B), dim3(TILE_TOKENS), 0, s>>>(
        xc->scale, eT_k, cap, L.ng, 2 * L.ng, p.tiles_per_seq, bits, len);
    scale_transpose_kernel<<<dim3(p.tiles_per_seq, B), dim3(TILE_TOKENS), 0, s>>>(
        xc->scale + L.ng, eT_v, cap, L.ng, 2 * L.ng, p.tiles_per_seq, bits, len, 0, normaliser);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // pass 1: keys
    p.codes = xc->codes; p.zero = xc->zero; p.eT = eT_k;
    p.wprep = static_cast<const uint8_t*>(wprep);
    p.head_shift = stream_shifts(p.wprep, L);
    e = launch_coded<MODE_SCORES>(bits, G, p, grid, s);
    if (e != hipSuccess) return e;
    // pass 2: values; its epilogue merges the eight chunks of a tile: one partial per tile
    p.codes = xc->codes + (size_t)r * bits / 8; p.zero = xc->zero + L.ng; p.eT = eT_v;
    p.wprep = static_cast<const uint8_t*>(wprep) + L.total_bytes;
    p.head_shift = stream_shifts(p.wprep, L);
    p.chunks_per_seq = p.tiles_per_seq;
    if (t16) {
        p.wprep += L.t16_offset;
        p.head_bytes = (long long)L.t16_head_bytes;
        p.n_corr_ksteps = L.t16_n_corr_ticks;
        e = launch_tile16(bits, G, p, grid, s, MODE_WEIGHTED_SUM);
    } else {
        e = launch_coded<MODE_WEIGHTED_SUM>(bits, G, p, grid, s);
    }
    if (e != hipSuccess) return e;
    combine_kernel<<<dim3(p.Hq, p.B), dim3(128 * COMBINE_GROUPS), 0, s>>>(p.part_o, p.part_ml, out, p.Hq, p.tiles_per_seq, p.len, 1, TILE_TOKENS);
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
    p.head_shift = stream_shifts(uprep, L);
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

// Pre-pass 2: the factor images, [sequence][tile][slab (+1 pad)][block of the tile][k-step][lane half][8] fp16 (for the
// kernels on 16-column fragments: ...[block of the tile][tick][lane quarter][8], quarter q = unit q of the slab), in
// the order the unpacked operand dwords hold their channels (the unpack table gives the code of each slot).
// Blocks past the sequence's last one repeat it (their tokens are masked, but must stay finite).
struct PcImageArgs {
    const uint16_t* scale;
    const int* eblk;
    uint16_t* img;
    int d, blocks_cap, blocks_ws, block, tiles_per_seq, n_slabs, G;   // blocks per sequence in the cache / in eblk
    int tile16;                                                       // the order of the 16-column-fragment kernels
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
        int c = slab * 128 + gi * a.G + half * (a.G / 2) + (ksg >> 2) * 32 + a.tab.code_of_slot[ksg & 3][i];
        if (a.tile16) c = slab * 128 + ((e >> 3) & 3) * 32 + a.tab.code_of_slot[(e >> 5) & 3][i];   // [tick][quarter][8]
        const float sc = bf16_bits_to_f32(a.scale[((long long)b * a.blocks_cap + blk) * a.d + c]);
        const float f = ldexpf(sc, 15 - a.eblk[(long long)b * a.blocks_ws + blk]);
        out[e] = __builtin_bit_cast(uint16_t, (_Float16)f);
    }
}

bool unpack_table_for(int bits, UnpackTable* t);

// The per-block terms of a per-channel cache (factor images, z W rows, block factors and exponents) depend on the
// complete blocks only, so a caller may keep them in a buffer of its own between decode steps and have them
// recomputed only after a block was completed.  That buffer is laid out for the cache's capacity, so that the
// positions do not move while the sequences grow; col_blocks = 256-column blocks of the prepared weights.
struct PcTerms {
    uint8_t* img;
    float* zw;
    float* fscale;
    int* eblk;
    size_t blocks_ws;      // rows per sequence of zw, fscale, eblk
};

size_t pc_terms_bytes(int B, int cap, int d, int block, int col_blocks)
{
    const size_t tiles = ((size_t)cap + TILE_TOKENS - 1) / TILE_TOKENS;
    const size_t blocks = (size_t)cap / block + 1;
    return (size_t)B * tiles * (size_t)(d / 128 + 1) * LDS_SCALES_BYTES + (size_t)B * blocks * (size_t)col_blocks * 256 * sizeof(float)
         + (size_t)B * blocks * 2 * sizeof(float) + 256;
}

static PcTerms carve_pc_terms(void* base, int B, int cap, int d, int block, int col_blocks)
{
    const size_t tiles = ((size_t)cap + TILE_TOKENS - 1) / TILE_TOKENS;
    PcTerms t{};
    t.blocks_ws = (size_t)cap / block + 1;
    t.img = static_cast<uint8_t*>(base);
    t.zw = reinterpret_cast<float*>(t.img + (size_t)B * tiles * (size_t)(d / 128 + 1) * LDS_SCALES_BYTES);
    t.fscale = t.zw + (size_t)B * t.blocks_ws * col_blocks * 256;
    t.eblk = reinterpret_cast<int*>(t.fscale + (size_t)B * t.blocks_ws);
    return t;
}

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
                                    void* terms, bool terms_valid, float* out, void* ws, hipStream_t s)
{
    const int bits = xc->fmt.bits, blockT = xc->fmt.group, d = xc->fmt.d, B = xc->B, cap = xc->cap;
    const int blocks_cap = cap / blockT;
    const WPrepLayout Lc = make_wprep_layout_for_cache(d, 128, bits, a->n_kv_heads);    // (has the 16-column fragments)
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
    size_t blocks_ws = (size_t)max_len / blockT + 1;
    float* fscale = zw + (size_t)B * blocks_ws * a->n_kv_heads * 256;
    int* eblk = reinterpret_cast<int*>(fscale + (size_t)B * blocks_ws);
    if (terms) {                                                             // the caller's own buffer for the per-block terms
        const PcTerms t = carve_pc_terms(terms, B, cap, d, blockT, a->n_kv_heads);
        img = t.img; zw = t.zw; fscale = t.fscale; eblk = t.eblk; blocks_ws = t.blocks_ws;
    }
    const bool compute_terms = !(terms && terms_valid);

    RematParams p{};
    p.q = q;
    p.B = B; p.Hq = a->n_q_heads; p.Hkv = a->n_kv_heads; p.grid_heads = p.Hkv;
    p.scale_log2e = a->softmax_scale * 1.44269504088896340736f;
    p.part_o = part_o; p.part_ml = part_ml; p.chunks_per_seq = chunks_stride;
    p.d = d; p.row_d = d;
    hipError_t e = hipSuccess;
    if (max_nblk > 0 && compute_terms) {
        // block exponents, factor images
        pc_block_exponent_kernel<<<dim3(max_nblk, B), dim3(256), 0, s>>>(xc->scale, fscale, eblk, d, blocks_cap, (int)blocks_ws, bits, nblk);
        PcImageArgs ia{xc->scale, eblk, reinterpret_cast<uint16_t*>(img), d, blocks_cap, (int)blocks_ws, blockT, tiles_coded, Lc.n_main_slabs, 128,
                       1, nblk, tab};
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
    }
    if (max_nblk > 0) {
        // the coded blocks
        RematParams m = p;
        m.codes = xc->codes; m.eT = reinterpret_cast<const uint16_t*>(img);
        m.cap = cap; m.len = len_coded; m.tiles_per_seq = tiles_coded;
        m.wprep = static_cast<const uint8_t*>(wprep_coded);
        m.head_shift = stream_shifts(wprep_coded, Lc);
        m.n_main_slabs = Lc.n_main_slabs; m.n_corr_ksteps = Lc.n_corr_ksteps; m.ng = Lc.ng; m.ng_pad = Lc.ng_pad; m.ng_row = Lc.ng;
        m.wprep += Lc.t16_offset;                                            // the stream of 16-column fragments
        m.head_bytes = (long long)Lc.t16_head_bytes;
        m.pc_fscale = fscale; m.pc_zw = zw; m.pc_block = blockT; m.pc_blocks_cap = (int)blocks_ws;
        e = launch_tile16_per_channel(bits, m, p.Hkv * B * tiles_coded, s);
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

// App. B: the first channel of X Uk, which collects the outliers, kept in fp16 instead of being quantised.  Its share
// of the keys is the rank-1 term k0[t] * W[0][:], so its share of a query head's score is k0[t] * (q . W[0][columns of
// the head]); this kernel adds it to the stored scores between the two passes (the prepared key streams carry a zero
// row 0, so nothing else of that channel reaches the keys).  Grid (token chunks, query heads, sequences).
__global__ __launch_bounds__(256) void outlier_scores_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ w_row0,
                                                             const uint16_t* __restrict__ k0, long long k0_stride,
                                                             float* __restrict__ scores, long long score_stride, int Hq,
                                                             int Hkv, float scale_log2e, BatchI32 len)
{
    const int hq = blockIdx.y, b = blockIdx.z;
    const int hk = hq / (Hq / Hkv);
    const int lane = threadIdx.x & 63;
    const uint16_t* qv = q + ((long long)b * Hq + hq) * 128;
    const uint16_t* wv = w_row0 + hk * 128;
    float dot = bf16_bits_to_f32(qv[lane]) * bf16_bits_to_f32(wv[lane]);
    dot = __builtin_fmaf(bf16_bits_to_f32(qv[lane + 64]), bf16_bits_to_f32(wv[lane + 64]), dot);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) dot += __shfl_xor(dot, off);          // every wave holds the whole sum
    const float f = dot * scale_log2e;
    float* srow = scores + ((long long)b * Hq + hq) * score_stride;
    const uint16_t* krow = k0 + (long long)b * k0_stride;
    const int n = len.v[b];
    for (int t = blockIdx.x * 256 + threadIdx.x; t < n; t += gridDim.x * 256)
        srow[t] = __builtin_fmaf((float)__builtin_bit_cast(_Float16, krow[t]), f, srow[t]);
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
                                           const uint16_t* k0_f16, long long k0_stride, const uint16_t* wk_row0,
                                           void* terms, bool terms_valid, float* out, void* ws, hipStream_t s)
{
    const int kbits = kc->fmt.bits, blockT = kc->fmt.group, r = kc->fmt.d, B = kc->B;
    const int vbits = vc->fmt.bits, vG = vc->fmt.group;
    const int pairs = a->n_kv_heads / 2;
    const int blocks_cap = kc->cap / blockT;
    const WPrepLayout Lk = pairs_layout(r, 128, kbits, pairs);
    const WPrepLayout Ld = pairs_layout(r, 128, 16, pairs);
    const WPrepLayout Lv = pairs_layout(r, vG, vbits, pairs);
    const bool v16 = Lv.t16_bytes != 0 && a->n_q_heads / a->n_kv_heads <= 16;   // pass 2 on the 16-column fragments
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
    size_t blocks_ws = (size_t)max_len / blockT + 1;
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
    if (terms) {                                                             // the caller's own buffer for the per-block terms
        const PcTerms t = carve_pc_terms(terms, B, kc->cap, r, blockT, pairs);
        img = t.img; zw = t.zw; fscale = t.fscale; eblk = t.eblk; blocks_ws = t.blocks_ws;
    }
    const bool compute_terms = !(terms && terms_valid);

    RematParams p{};
    p.q = q;
    p.B = B; p.Hq = a->n_q_heads; p.Hkv = a->n_kv_heads; p.grid_heads = pairs;
    p.scale_log2e = a->softmax_scale * 1.44269504088896340736f;
    p.part_o = part_o; p.part_ml = part_ml; p.chunks_per_seq = chunks;
    p.scores = scores; p.score_stride = score_stride;
    p.d = r; p.row_d = r;
    hipError_t e = hipSuccess;
    if (max_nblk > 0 && compute_terms) {
        pc_block_exponent_kernel<<<dim3(max_nblk, B), dim3(256), 0, s>>>(kc->scale, fscale, eblk, r, blocks_cap, (int)blocks_ws, kbits, nblk);
        PcImageArgs ia{kc->scale, eblk, reinterpret_cast<uint16_t*>(img), r, blocks_cap, (int)blocks_ws, blockT, tiles_coded,
                       Lk.n_main_slabs, 128, 0, nblk, tab};
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
    }
    if (max_nblk > 0) {
        RematParams m = p;                                                   // pass 1, coded blocks
        m.codes = kc->codes; m.eT = reinterpret_cast<const uint16_t*>(img);
        m.cap = kc->cap; m.len = len_coded; m.tiles_per_seq = tiles_coded;
        m.wprep = static_cast<const uint8_t*>(wk_coded);
        m.head_shift = stream_shifts(wk_coded, Lk);
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
    if (k0_f16) {                                                            // the fp16 channel's share of the scores
        outlier_scores_kernel<<<dim3((max_len + 1023) / 1024, p.Hq, B), dim3(256), 0, s>>>(
            q, wk_row0, k0_f16, k0_stride, scores, score_stride, p.Hq, p.Hkv, p.scale_log2e, len);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    // pass 2: values from the per-token cache
    scale_transpose_kernel<<<dim3(tiles_all, B), dim3(TILE_TOKENS), 0, s>>>(vc->scale, eT_v, vc->cap, Lv.ng, Lv.ng, tiles_all, vbits, len, 0,
                                                                            v16 && vG == 64);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    RematParams v = p;
    v.codes = vc->codes; v.zero = vc->zero; v.eT = eT_v;
    v.cap = vc->cap; v.len = len; v.tiles_per_seq = tiles_all;
    v.wprep = static_cast<const uint8_t*>(wv_coded);
    v.head_shift = stream_shifts(wv_coded, Lv);
    v.n_main_slabs = Lv.n_main_slabs; v.n_corr_ksteps = Lv.n_corr_ksteps; v.ng = Lv.ng; v.ng_pad = Lv.ng_pad; v.ng_row = Lv.ng;
    v.head_bytes = (long long)Lv.head_bytes;
    v.chunks_per_seq = tiles_all;                        // one partial per tile
    if (v16) {
        v.wprep += Lv.t16_offset;
        v.head_bytes = (long long)Lv.t16_head_bytes;
        v.n_corr_ksteps = Lv.t16_n_corr_ticks;
        e = launch_tile16(vbits, vG, v, pairs * B * tiles_all, s, MODE_WEIGHTED_SUM);
    } else {
        e = launch_coded<MODE_WEIGHTED_SUM>(vbits, vG, v, pairs * B * tiles_all, s);
    }
    if (e != hipSuccess) return e;
    combine_kernel<<<dim3(p.Hq, B), dim3(128 * COMBINE_GROUPS), 0, s>>>(part_o, part_ml, out, p.Hq, tiles_all, len, 1, TILE_TOKENS);
    return hipGetLastError();
}

// Bulk projection of M rows into the latent space (Sec. 3.3.1), out = bf16(x U): the dense-source contraction
// kernel over one "sequence" of M rows, the n_lat columns laid over n_lat / 256 column blocks, rows stored as bf16.
hipError_t run_project_rows_dense(const uint16_t* x, long long M, int d, int n_lat, const void* proj, uint16_t* out,
                                  hipStream_t s)
{
    const int blocks = n_lat / 256;
    const WPrepLayout L = make_wprep_layout(d, 128, 16, blocks);
    RematParams p{};
    p.acc = x; p.B = 1; p.cap = (int)M; p.d = d; p.row_d = d;
    p.Hq = p.Hkv = blocks; p.grid_heads = blocks; p.tile_major = 1;
    p.len.v[0] = (int)M;
    p.tiles_per_seq = (int)((M + TILE_TOKENS - 1) / TILE_TOKENS);
    p.wprep = static_cast<const uint8_t*>(proj);
    p.n_main_slabs = L.n_main_slabs; p.w_slabs = L.n_main_slabs; p.head_bytes = (long long)L.head_bytes;
    p.rows_out = out;
    return launch_with_lds(remat_attn_dense_kernel<DENSE_STORE_BF16>, LDS_DENSE_TOTAL, p, blocks * p.tiles_per_seq, s);
}

// Bulk cross-layer latent delta (Sec. 3.3.2), out = bf16((x - acc rows) U) for T rows of each of B sequences: the
// same kernel walks the prepared stream of U twice, first against the rows of x, then against the matching
// accumulator rows with flipped signs, so that x U - acc U is summed in one fp32 accumulator and rounded once.
hipError_t run_project_delta_rows_dense(const uint16_t* x, const uint16_t* acc, int B, int T, int cap, const BatchI32& start,
                                        int d, int n_lat, const void* proj, uint16_t* out, hipStream_t s)
{
    const int blocks = n_lat / 256;
    const long long M = (long long)B * T;
    const WPrepLayout L = make_wprep_layout(d, 128, 16, blocks);
    RematParams p{};
    p.acc = x; p.B = 1; p.cap = (int)M; p.d = d; p.row_d = d;
    p.Hq = p.Hkv = blocks; p.grid_heads = blocks; p.tile_major = 1;
    p.len.v[0] = (int)M;
    p.tiles_per_seq = (int)((M + TILE_TOKENS - 1) / TILE_TOKENS);
    p.wprep = static_cast<const uint8_t*>(proj);
    p.w_slabs = L.n_main_slabs; p.n_main_slabs = 2 * L.n_main_slabs; p.head_bytes = (long long)L.head_bytes;
    p.acc2 = acc; p.Tq = T; p.cap2 = cap; p.tok0 = start;
    p.rows_out = out;
    return launch_with_lds(remat_attn_dense_kernel<DENSE_STORE_BF16>, LDS_DENSE_TOTAL, p, blocks * p.tiles_per_seq, s);
}

}  // namespace xq
