/*
 * libxquant -- XQuant / XQuant-CL decode hot path for AMD MI355X (gfx950).
 *
 * C ABI.  Every pointer is caller-owned memory; "dev" marks device (HBM)
 * pointers, "host" marks host pointers.  The library allocates nothing, keeps no
 * state between calls and never synchronises with the host: all work is enqueued
 * on the HIP stream passed in (a hipStream_t cast to void*, NULL = the default
 * stream) and results are valid once the caller has synchronised that stream.
 * Functions return an xq_status_t; nothing throws or aborts across this
 * boundary.  Argument errors are detected on the host before anything is
 * launched.  Device pointers must be 16-byte aligned.  Non-finite inputs are
 * outside the contract.
 *
 * Method (arxiv 2508.10395): instead of a K/V cache, cache the post-norm layer
 * input X quantised to a few bits per element (Sec. 3.1), or, for XQuant-CL,
 * the quantised differences of X between successive layers summed into a running
 * accumulator (Sec. 3.2); at attention time rematerialise K = X^ Wk and
 * V = X^ Wv on the fly (Sec. 3.1, cost model in Sec. 3.4) and attend to them.
 *
 * Storage format of a quantised cache (one tensor per layer; Sec. 4 setup:
 * uniform asymmetric quantisation, one scale and one zero-point per group of
 * `group` consecutive hidden channels of one token, 16 bits each -- the sizes in
 * Tables 1 and 4 imply 32 metadata bits per group):
 *   codes [B][cap][d*bits/8]  each token row is one little-endian bit string,
 *                             code j at bits [j*bits, (j+1)*bits)
 *   scale [B][cap][d/group]   bf16 bit patterns
 *   zero  [B][cap][d/group]   bf16 bit patterns (zero-point = group minimum)
 *   x^[j] = code[j]*scale + zero            (one fp32 fused multiply-add)
 * Quantiser: zero = bf16(min), scale = bf16((max-min)/(2^bits-1)), both
 * round-to-nearest-even; code = clamp(rint((x-zero)/scale), 0, 2^bits-1) in fp32
 * with round-half-to-even, all codes 0 when the stored scale is 0; a zero-point
 * equal to -0 is stored as +0.
 */
#ifndef XQUANT_H
#define XQUANT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    XQ_OK = 0,
    XQ_ERR_INVALID_ARG = -1,  /* NULL/misaligned pointer, inconsistent sizes, row range outside the cache */
    XQ_ERR_UNSUPPORTED = -2,  /* a shape or format this build has no kernel for */
    XQ_ERR_WORKSPACE = -3,    /* workspace / output buffer smaller than the matching *_bytes query */
    XQ_ERR_HIP = -4           /* the HIP runtime refused a launch or a copy */
} xq_status_t;

#define XQ_MAX_BATCH 128      /* largest B any call accepts */

/* Quantisation format: hidden size d, group size (64 or 128, must divide d), bits in {2,3,4,8}. */
typedef struct { int32_t d, group, bits; } xq_qfmt_t;

/* A view of a caller-owned quantised cache (layout above).  cap = rows allocated per sequence; one
 * sequence's codes must stay below 4 GiB (cap * d * bits / 8 < 2^32), else XQ_ERR_UNSUPPORTED. */
typedef struct {
    uint8_t  *codes;   /* dev */
    uint16_t *scale;   /* dev */
    uint16_t *zero;    /* dev */
    int32_t   B, cap;
    xq_qfmt_t fmt;
} xq_cache_t;

/* Attention geometry.  head_dim must be 128; n_q_heads must be a multiple of n_kv_heads. */
typedef struct { int32_t n_q_heads, n_kv_heads, head_dim; float softmax_scale; } xq_attn_t;

const char *xq_status_string(xq_status_t s);
int         xq_version(void);

size_t xq_codes_row_bytes(const xq_qfmt_t *f);   /* d*bits/8, 0 if the format is invalid */
size_t xq_meta_row_elems(const xq_qfmt_t *f);    /* d/group,  0 if the format is invalid */

/*
 * Sec. 3.1 (Fig. 2): quantise the layer input of T new tokens per sequence and
 * append them to the X cache.
 *   x_bf16  dev  [B][T][d] bf16
 *   start   host [B]; rows start[b] .. start[b]+T-1 of sequence b are written
 *           (start[b] >= 0, start[b]+T <= cap)
 * T = 0 is a no-op.
 */
xq_status_t xq_quantize_append(const xq_cache_t *cache, const uint16_t *x_bf16, int32_t T,
                               const int32_t *start, void *stream);

/*
 * Sec. 3.2 (Fig. 4, and App. A for T > 1): cross-layer delta of T new tokens,
 *   dX = X_i - X^_{i-1}   (fp32 difference of two bf16 values),
 * quantised with the same quantiser and written to rows start[b]..start[b]+T-1 of
 * this layer's delta cache.
 *   x_bf16   dev [B][T][d]    true input of layer i
 *   acc_bf16 dev [B][cap][d]  accumulator holding X^_{i-1}; rows start[b]+t are read
 */
xq_status_t xq_cl_delta_quantize(const xq_cache_t *delta, const uint16_t *x_bf16,
                                 const uint16_t *acc_bf16, int32_t T, const int32_t *start,
                                 void *stream);

/*
 * Sec. 3.2: X^_i = X^_{i-1} + dX^_i on the running accumulator, for rows
 * t < len[b] of every sequence:
 *   acc = bf16( (init ? +0 : acc) + fma(code, scale, zero) )   fp32 add, RNE to bf16.
 * init != 0 loads the base layer X_0 (itself a quantised cache) into the accumulator.
 *   acc_bf16 dev [B][cap][d] (cap and d taken from src), updated in place
 *   len      host [B], 0 <= len[b] <= cap
 */
xq_status_t xq_cl_accumulate(uint16_t *acc_bf16, const xq_cache_t *src, const int32_t *len,
                             int32_t init, void *stream);

/*
 * Weight preparation (offline, once per layer; weights are static).  Re-lays
 * [Wk | Wv] (Sec. 3.3.2 writes the column concatenation W_kv) per KV head into the
 * fragment order the rematerialisation kernel streams, together with per-group
 * column sums used to apply the zero-points exactly.
 *   Wk, Wv   dev [d][n_kv_heads*head_dim] bf16, row-major
 *   src_bits 2, 3, 4 or 8: prepared for an X cache of that bit width and group size
 *            `group`; 16: prepared for the bf16 cross-layer accumulator (group ignored).
 *            (8: for xq_remat_attn_decode / _rope / _prefill over a per-token cache only.)
 *   out      dev, at least xq_prepared_weights_bytes(...) bytes
 * Range of the weights: any finite bf16 values.  For src_bits 2, 3, 4 the stream holds fp16 numbers;
 * each KV head's [Wk_h | Wv_h] is scaled by one power of two so that its largest entry sits at the top
 * of the fp16 range (the kernels take the factor out again, exactly), so a layer of uniformly tiny or
 * large weights loses nothing; within one head, entries more than 2^-29 below the head's largest are
 * rounded at 2^-40 of the largest.
 * Size: d x 2 n_kv_heads head_dim 16-bit entries plus the column sums; twice that for groups of 128, for
 * src_bits 8 and for src_bits 16, whose kernels read the weights in a second fragment order that is stored
 * alongside the first (the query below is the authority).
 * xq_prepared_weights_bytes returns 0 for an unsupported combination.
 */
size_t      xq_prepared_weights_bytes(const xq_attn_t *a, int32_t d, int32_t group, int32_t src_bits);
xq_status_t xq_prepare_weights(const xq_attn_t *a, int32_t d, int32_t group, int32_t src_bits,
                               const uint16_t *Wk, const uint16_t *Wv, void *out, size_t out_bytes,
                               void *stream);

/*
 * Sec. 3.1 + Sec. 3.4: one decode step of attention over the cached tokens with
 * K and V rematerialised on the fly and never written to memory.  For every
 * sequence b and query head h (KV head h / (n_q_heads/n_kv_heads)):
 *   K = X^[0:len[b]] Wk_h,  V = X^[0:len[b]] Wv_h,
 *   out[b][h] = softmax(q[b][h] K^T * softmax_scale) V.
 * Exactly one source of X^ is given:
 *   xcache != NULL   an X cache (XQuant), x^ = code*scale + zero;
 *   acc_bf16 != NULL the cross-layer accumulator [B][cap][d] (XQuant-CL); one sequence's rows must stay
 *                    below 4 GiB (cap * d * 2 < 2^32), else XQ_ERR_UNSUPPORTED.
 *   q_bf16   dev [B][n_q_heads][head_dim] bf16
 *   wprep    dev, from xq_prepare_weights with matching d / group / src_bits
 *   len      host [B], 1 <= len[b] <= cap
 *   out      dev [B][n_q_heads][head_dim] fp32
 *   workspace dev, >= xq_remat_attn_workspace_bytes(...) bytes, 16-byte aligned; holds the
 *            per-chunk softmax partials and a tile-ordered copy of the scales; contents are scratch
 * B is taken from xcache->B, or passed in `B` when acc_bf16 is the source.
 * xq_remat_attn_workspace_bytes: max_len = max_b len[b]; d and group are those of the X cache,
 * group = 0 when the accumulator is the source.  Returns 0 for an invalid combination.
 * 8-bit caches (the XQuant-8bit rows of Table 1) are served too: the kernel walks the two nibbles of a
 * code as two 4-bit codes (the high one against 16 times the weight row; x^ = (16 hi + lo) scale + zero
 * exactly), at twice the matrix work of a 4-bit cache.  Size the workspace for such a cache with
 * d = 2 * fmt.d and group = 128 (likewise xq_remat_attn_prefill_workspace_bytes).
 */
size_t      xq_remat_attn_workspace_bytes(const xq_attn_t *a, int32_t B, int32_t max_len, int32_t d,
                                          int32_t group);
xq_status_t xq_remat_attn_decode(const xq_attn_t *a, const uint16_t *q_bf16,
                                 const xq_cache_t *xcache,
                                 const uint16_t *acc_bf16, int32_t B, int32_t cap, int32_t d,
                                 const void *wprep, const int32_t *len, float *out,
                                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * xq_remat_attn_decode for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid it): same arguments, same kernels and same result, but
 * the workspace is a buffer built into the library, XQ_STATIC_SCRATCH_BYTES per GPU, instead of a
 * caller buffer.  The call allocates and frees nothing.  A problem whose
 * xq_remat_attn_workspace_bytes(...) exceeds XQ_STATIC_SCRATCH_BYTES is refused with
 * XQ_ERR_WORKSPACE before anything is launched (the 32 MiB cover e.g. B=8, 32 query heads, context
 * 4096, d=4096, group 128: 19.5 MB).  The buffer belongs to the device that is current at the call
 * (which must be the stream's device); its address is looked up on the first call on each device.
 * All calls on one GPU share that GPU's buffer: calls that overlap in time on one GPU (different
 * streams or threads) race and must be serialised by the caller; the buffer's contents between calls
 * are scratch.
 */
#define XQ_STATIC_SCRATCH_BYTES (32u << 20)
xq_status_t xq_remat_attn_decode_static(const xq_attn_t *a, const uint16_t *q_bf16,
                                        const xq_cache_t *xcache,
                                        const uint16_t *acc_bf16, int32_t B, int32_t cap, int32_t d,
                                        const void *wprep, const int32_t *len, float *out, void *stream);

/*
 * xq_remat_attn_decode with rotary position embedding applied to the rematerialised keys (K = X^ Wk
 * is the key before the rotation; the models the method targets rotate it; RoFormer, cited in
 * Sec. 2).  Pairing: element i with i + head_dim/2.  For cache row t of sequence b, at position
 * pos0[b] + t, with (cos, sin) = rope_cos_sin[position][i]:
 *     k'[i] = k[i] cos - k[i+64] sin,    k'[i+64] = k[i+64] cos + k[i] sin.
 *   rope_cos_sin   dev [rope_positions][head_dim/2][2] fp32 (cos, sin); the frequencies, and any
 *                  scaling of them, are the caller's
 *   pos0           host [B], pos0[b] >= 0 and pos0[b] + len[b] <= rope_positions
 *   q_bf16         is used as given: the caller rotates the query at its own position
 * Everything else as xq_remat_attn_decode.
 */
xq_status_t xq_remat_attn_decode_rope(const xq_attn_t *a, const uint16_t *q_bf16,
                                      const xq_cache_t *xcache, const uint16_t *acc_bf16, int32_t B,
                                      int32_t cap, int32_t d, const void *wprep, const int32_t *len,
                                      const float *rope_cos_sin, int32_t rope_positions,
                                      const int32_t *pos0, float *out, void *workspace,
                                      size_t workspace_bytes, void *stream);

/*
 * Causal attention of the T newest tokens of every sequence (chunked prefill; the method
 * rematerialises K, V for any query that attends to the cache, Sec. 3.1, and App. A treats T > 1
 * new tokens).  The T queries' own rows are already in the cache (xq_quantize_append first):
 * query t of sequence b sits at cache row len[b] - T + t and attends rows 0 .. that row.
 *   q_bf16   dev [B][T][n_q_heads][head_dim] bf16
 *   len      host [B], T <= len[b] <= cap: valid cache rows including the T new ones
 *   rope_cos_sin, rope_positions, pos0: as xq_remat_attn_decode_rope, or NULL, 0, NULL for no rotation
 *   out      dev [B][T][n_q_heads][head_dim] fp32
 *   workspace dev, xq_remat_attn_prefill_workspace_bytes(a, B, T, max len, d, group) bytes
 *             (group = 0 for the accumulator source); B*T <= 65535.
 * Everything else as xq_remat_attn_decode.  Scores and the weighted sum run on the matrix cores
 * with K, V and the softmax weights split into bf16 hi + lo parts (relative error 2^-16).
 */
size_t      xq_remat_attn_prefill_workspace_bytes(const xq_attn_t *a, int32_t B, int32_t T,
                                                  int32_t max_len, int32_t d, int32_t group);
xq_status_t xq_remat_attn_prefill(const xq_attn_t *a, const uint16_t *q_bf16, int32_t T,
                                  const xq_cache_t *xcache, const uint16_t *acc_bf16, int32_t B,
                                  int32_t cap, int32_t d, const void *wprep, const int32_t *len,
                                  const float *rope_cos_sin, int32_t rope_positions,
                                  const int32_t *pos0, float *out, void *workspace,
                                  size_t workspace_bytes, void *stream);

/*
 * Sec. 3.3.1 (models with grouped-query attention): with the offline decompositions
 * Wk = Uk Sk Bk^T and Wv = Uv Sv Bv^T (SVD, rank r = n_kv_heads*head_dim), the cache holds the
 * latent row [x Uk | x Uv] (2r channels) of every token, quantised like any other X cache, and K,
 * V are rematerialised as (x Uk)(Sk Bk^T) and (x Uv)(Sv Bv^T) with the fused r x r matrices.
 *
 * xq_latent_project: the down-projection of M token rows,
 *   out[m][n] = bf16( sum_c x[m][c] * Ut[n][c] ),   fp32 accumulation, one RNE rounding.
 *   x_bf16   dev [M][d] bf16
 *   Ut_bf16  dev [n_lat][d] bf16: U TRANSPOSED, one row per latent channel (for the layout above:
 *            rows 0..r-1 = columns of Uk, rows r..2r-1 = columns of Uv)
 *   out_bf16 dev [M][n_lat] bf16, ready for xq_quantize_append with fmt.d = n_lat
 *   d must be a multiple of 128, n_lat a multiple of 32; M = 0 is a no-op.
 *
 * xq_prepare_weights_latent: prepared streams for a latent cache with fmt.d = 2r:
 *   Wfk, Wfv dev [r][n_kv_heads*head_dim] bf16 row-major = Sk Bk^T and Sv Bv^T
 *   src_bits 2, 3 or 4; r a multiple of 128; n_kv_heads even;
 *   out dev, at least xq_prepared_weights_latent_bytes(a, r, group, src_bits) bytes (0 = unsupported).
 *
 * xq_remat_attn_decode_latent: decode attention from a latent cache and the streams above: the
 *   first r channels of a row rematerialise the keys, the last r the values (two passes; the scores
 *   of pass 1 wait in the workspace).  Arguments as xq_remat_attn_decode with an X cache;
 *   workspace size: xq_remat_attn_latent_workspace_bytes(a, B, max_len, r, group).
 */
/*
 * The same projection for prefill-sized M, on the matrix cores through the dense-source contraction
 * kernel (about ten times the rate of xq_latent_project from a few thousand rows on; same result up to
 * the order of the fp32 accumulation):
 *   xq_prepare_projection: offline re-layout of Ut (dev [n_lat][d] bf16) into out, at least
 *     xq_prepared_projection_bytes(d, n_lat) bytes (0 = unsupported: d multiple of 128, n_lat of 256)
 *   xq_latent_project_bulk: out_bf16[m][n] = bf16( sum_c x[m][c] * Ut[n][c] ) for M rows; x_bf16 dev [M][d],
 *     out_bf16 dev [M][n_lat].  M = 0 is a no-op; M * d must stay below 2^31 (split larger inputs).
 */
size_t      xq_prepared_projection_bytes(int32_t d, int32_t n_lat);
xq_status_t xq_prepare_projection(int32_t d, int32_t n_lat, const uint16_t *Ut_bf16, void *out, size_t out_bytes,
                                  void *stream);
xq_status_t xq_latent_project_bulk(const uint16_t *x_bf16, const void *proj, int64_t M, int32_t d, int32_t n_lat,
                                   uint16_t *out_bf16, void *stream);
size_t      xq_prepared_weights_latent_bytes(const xq_attn_t *a, int32_t r, int32_t group, int32_t src_bits);
size_t      xq_remat_attn_latent_workspace_bytes(const xq_attn_t *a, int32_t B, int32_t max_len, int32_t r,
                                                 int32_t group);
xq_status_t xq_latent_project(const uint16_t *x_bf16, const uint16_t *Ut_bf16, int32_t M, int32_t d,
                              int32_t n_lat, uint16_t *out_bf16, void *stream);
xq_status_t xq_prepare_weights_latent(const xq_attn_t *a, int32_t r, int32_t group, int32_t src_bits,
                                      const uint16_t *Wfk, const uint16_t *Wfv, void *out, size_t out_bytes,
                                      void *stream);
xq_status_t xq_remat_attn_decode_latent(const xq_attn_t *a, const uint16_t *q_bf16,
                                        const xq_cache_t *latent, const void *wprep, const int32_t *len,
                                        float *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Sec. 3.3.2 (XQuant-CL for grouped-query models): with the offline SVD [Wk | Wv] = U_kv S B^T
 * (n_lat = 2 * n_kv_heads * head_dim latent channels), layer i caches the quantised latent delta
 * (X_i - X^_{i-1}) U_kv and merges it into the accumulator through U_kv^T:
 *     X^_i = X^_{i-1} + dequant(cached delta) U_kv^T;
 * K and V then come from xq_remat_attn_decode on the accumulator (xcache = NULL) with Wk, Wv.
 * Ut_bf16 is U_kv TRANSPOSED, dev [n_lat][d] bf16 row-major, in all three calls.
 *
 * xq_cl_latent_delta_project: the latent delta of T new tokens per sequence,
 *   out[b][t][n] = bf16( sum_c (x[b][t][c] - acc[b][start[b]+t][c]) * Ut[n][c] ),
 *   difference and accumulation in fp32, one RNE rounding; ready for xq_quantize_append with
 *   fmt.d = n_lat.
 *   x_bf16 dev [B][T][d]; acc_bf16 dev [B][cap][d]; start host [B], 0 <= start[b], start[b]+T <= cap;
 *   out_bf16 dev [B][T][n_lat].  d multiple of 128, n_lat multiple of 32.  T = 0 is a no-op.
 *
 * xq_cl_latent_delta_project_bulk: the same for prefill-sized T, on the matrix cores (the dense-source
 *   contraction kernel, as xq_latent_project_bulk): proj is xq_prepare_projection(d, n_lat, Ut) and is walked
 *   twice, against the rows of x and against the matching accumulator rows with flipped signs, so that
 *   x U - acc U is summed in one fp32 accumulator and rounded once.  The result equals the one above up to
 *   fp32 accumulation error, which here is relative to sum_c (|x| + |acc|) |U| rather than to the smaller
 *   sum_c |x - acc| |U| (about 2^-16 of it at most, against the output's own 2^-9 rounding).
 *   n_lat multiple of 256; B*T*d and B*cap*d below 2^31 elements (split larger inputs).
 *
 * xq_prepare_upproject: offline re-layout of Ut for xq_cl_accumulate_latent (src_bits 2, 3, 4 of
 *   the delta cache; d multiple of 256, n_lat multiple of 128); out dev, at least
 *   xq_prepared_upproject_bytes(d, n_lat, group, src_bits) bytes (0 = unsupported).
 *
 * xq_cl_accumulate_latent: for rows t < len[b] of every sequence and all d hidden channels n,
 *     acc[b][t][n] = bf16( acc[b][t][n] + sum_c fma(code[c], scale, zero) * Ut[c][n] ),
 *   the sum on the matrix cores with fp32 accumulation, fp32 add, one RNE rounding.  The stored
 *   bf16 can differ from the exactly rounded one by one unit in the last place where the exact
 *   sum lies within the fp32 accumulation error of a rounding boundary.
 *   acc_bf16  dev [B][cap][d] (B, cap from delta), updated in place
 *   delta     cache with fmt.d = n_lat
 *   len       host [B], 0 <= len[b] <= cap
 *   workspace dev, xq_cl_accumulate_latent_workspace_bytes(B, max len, n_lat, group) bytes
 */
xq_status_t xq_cl_latent_delta_project(const uint16_t *x_bf16, const uint16_t *acc_bf16,
                                       const uint16_t *Ut_bf16, int32_t B, int32_t T, int32_t cap,
                                       const int32_t *start, int32_t d, int32_t n_lat,
                                       uint16_t *out_bf16, void *stream);
xq_status_t xq_cl_latent_delta_project_bulk(const uint16_t *x_bf16, const uint16_t *acc_bf16, const void *proj,
                                            int32_t B, int32_t T, int32_t cap, const int32_t *start,
                                            int32_t d, int32_t n_lat, uint16_t *out_bf16, void *stream);
size_t      xq_prepared_upproject_bytes(int32_t d, int32_t n_lat, int32_t group, int32_t src_bits);
xq_status_t xq_prepare_upproject(int32_t d, int32_t n_lat, int32_t group, int32_t src_bits,
                                 const uint16_t *Ut_bf16, void *out, size_t out_bytes, void *stream);
size_t      xq_cl_accumulate_latent_workspace_bytes(int32_t B, int32_t max_len, int32_t n_lat,
                                                    int32_t group);
xq_status_t xq_cl_accumulate_latent(uint16_t *acc_bf16, const xq_cache_t *delta, int32_t d,
                                    const void *uprep, const int32_t *len, void *workspace,
                                    size_t workspace_bytes, void *stream);

/*
 * Per-channel quantisation (Sec. 3.3.1: the paper's best setting for X U_k; groups along the
 * token axis with an unquantised residual window, as in KIVI cited there).  A per-channel cache
 * uses xq_cache_t with
 *   codes  dev [B][cap][d*bits/8]   rows packed exactly as in a per-token cache
 *   scale  dev [B][cap/group][d] bf16,  zero likewise: one pair per (block of `group` tokens, channel)
 *   fmt.group = tokens per block (64 or 128), cap a multiple of it, d a multiple of 128.
 * Only complete blocks are quantised; the newest len % group tokens of a sequence stay in a bf16
 * residual window that the caller keeps ([B][group][d]) and hands to the attention call.
 *
 * xq_quantize_blocks_per_channel: quantise nblk complete blocks per sequence,
 *   x_bf16  dev [B][nblk*group][d] bf16
 *   block0  host [B]: sequence b's blocks block0[b] .. block0[b]+nblk-1 are written
 *           (block0[b] >= 0, (block0[b]+nblk)*group <= cap)
 * with the arithmetic of xq_quantize_append per group (min/max, bf16 zero-point and scale, codes
 * from the stored pair).  nblk = 0 is a no-op.
 */
xq_status_t xq_quantize_blocks_per_channel(const xq_cache_t *cache, const uint16_t *x_bf16,
                                           int32_t nblk, const int32_t *block0, void *stream);

/*
 * xq_remat_attn_decode_per_channel: decode attention (as xq_remat_attn_decode) over len[b] tokens of
 * which the first floor(len[b]/group)*group are read from the per-channel cache (bits 2, 3 or 4) and
 * the remaining len[b] % group from rows 0.. of the residual window.
 *   tail_bf16    dev [B][group][d] bf16: the window (rows past len[b] % group are not read)
 *   len          host [B], len[b] >= 1, floor(len[b]/group)*group <= cap
 *   wprep_coded  xq_prepare_weights(a, d, 128, bits, Wk, Wv): stream for the coded blocks
 *   wprep_dense  xq_prepare_weights(a, d, 0, 16, Wk, Wv): stream for the window and for the
 *                zero-point term (the zero-points of a block times [Wk | Wv], one row per block)
 *   workspace    dev, xq_remat_attn_per_channel_workspace_bytes(a, B, max len, d, group) bytes
 *   terms        dev or NULL.  The terms the call derives from the complete blocks (operand factors,
 *                zero-points times [Wk | Wv], block exponents) change only when a block is completed.
 *                NULL: they are recomputed in the workspace on every call.  Otherwise a buffer the caller
 *                keeps per (cache, weights), xq_per_channel_terms_bytes(B, cap, d, group, n_kv_heads)
 *                bytes, 16-byte aligned, laid out for the cache's capacity:
 *                  terms_valid = 0  the call computes the terms into it, then uses them;
 *                  terms_valid != 0 the call only reads it: the caller states that since the last call
 *                                   with terms_valid = 0 on this buffer no sequence of the batch has
 *                                   completed a block and the cache, the weights and B are the same.
 *                                   Wrong use gives wrong numbers, not a fault.
 *                The library owns nothing here: it keeps no record of what the buffer holds.
 * The per-channel scales enter the contraction on the token operand (one packed fp16 multiply per
 * operand dword), exactly: an 8-bit significand times a 2- or 3-bit code fits fp16, and 4-bit codes
 * enter as code - 8 (the block-constant remainder joins the zero-point term).
 */
size_t      xq_remat_attn_per_channel_workspace_bytes(const xq_attn_t *a, int32_t B, int32_t max_len,
                                                      int32_t d, int32_t group);
/* col_blocks: 256-column blocks of the prepared weights: n_kv_heads for xq_remat_attn_decode_per_channel,
 * n_kv_heads / 2 for xq_remat_attn_decode_latent_per_channel (there d = r).  0 if unsupported. */
size_t      xq_per_channel_terms_bytes(int32_t B, int32_t cap, int32_t d, int32_t group, int32_t col_blocks);
xq_status_t xq_remat_attn_decode_per_channel(const xq_attn_t *a, const uint16_t *q_bf16,
                                             const xq_cache_t *cache, const uint16_t *tail_bf16,
                                             const int32_t *len, const void *wprep_coded,
                                             const void *wprep_dense, void *terms, size_t terms_bytes,
                                             int32_t terms_valid, float *out, void *workspace,
                                             size_t workspace_bytes, void *stream);

/*
 * The setting Sec. 3.3.1 finds best for grouped-query models: X Uk quantised per channel (with its
 * residual window), X Uv per token, each in a cache of its own of width r = n_kv_heads*head_dim.
 *
 * xq_prepare_weights_pairs: prepared stream of ONE fused latent matrix Wf = S B^T, dev [r][n_kv_heads*head_dim]
 *   bf16, whose "head" is a pair of KV heads (as each half of xq_prepare_weights_latent); src_bits 2, 3, 4
 *   (with group 64 or 128) or 16 (group ignored); out dev, xq_prepared_weights_pairs_bytes(...) bytes.
 *
 * xq_remat_attn_decode_latent_per_channel: decode attention over len[b] tokens,
 *   kcache      per-channel cache of X Uk (fmt.d = r): its floor(len[b]/group) complete blocks are read
 *   ktail_bf16  dev [B][kcache group][r] bf16: the window, rows 0 .. len[b] % group - 1
 *   vcache      per-token cache of X Uv (fmt.d = r), rows 0 .. len[b]-1
 *   wk_coded    xq_prepare_weights_pairs(a, r, 128, kcache bits, Sk Bk^T)
 *   wk_dense    xq_prepare_weights_pairs(a, r, 0, 16, Sk Bk^T)
 *   wv_coded    xq_prepare_weights_pairs(a, r, vcache group, vcache bits, Sv Bv^T)
 *   workspace   xq_remat_attn_latent_per_channel_workspace_bytes(a, B, max len, r, kcache group, vcache group)
 *   k0_f16      dev or NULL.  App. B: the first channel of X Uk, which collects the outliers, kept in fp16
 *               instead of being quantised.  If not NULL: [B][k0_stride] IEEE half bit patterns (finite),
 *               k0_stride >= every len[b]; latent key channel 0 of token t of sequence b is
 *               k0_f16[b*k0_stride + t] for all t < len[b], cache blocks and window alike.  The caller
 *               then prepares wk_coded and wk_dense from Sk Bk^T with its row 0 set to zero (so that
 *               whatever the cache and the window hold in channel 0 reaches nothing) and passes that row:
 *   wk_row0_bf16  dev [n_kv_heads*head_dim] bf16, row 0 of Sk Bk^T; read only if k0_f16 != NULL.
 *               The channel's share of a score, k0 * (q . row 0), is added in fp32 between the two passes.
 *   terms, terms_bytes, terms_valid   as in xq_remat_attn_decode_per_channel, for the key cache:
 *               xq_per_channel_terms_bytes(B, kcache cap, r, kcache group, n_kv_heads / 2) bytes, or NULL
 * Two passes as xq_remat_attn_decode_latent; pass 1 takes the keys as xq_remat_attn_decode_per_channel does.
 */
size_t      xq_prepared_weights_pairs_bytes(const xq_attn_t *a, int32_t r, int32_t group, int32_t src_bits);
xq_status_t xq_prepare_weights_pairs(const xq_attn_t *a, int32_t r, int32_t group, int32_t src_bits,
                                     const uint16_t *Wf, void *out, size_t out_bytes, void *stream);
size_t      xq_remat_attn_latent_per_channel_workspace_bytes(const xq_attn_t *a, int32_t B, int32_t max_len,
                                                             int32_t r, int32_t k_group, int32_t v_group);
xq_status_t xq_remat_attn_decode_latent_per_channel(const xq_attn_t *a, const uint16_t *q_bf16,
                                                    const xq_cache_t *kcache, const uint16_t *ktail_bf16,
                                                    const xq_cache_t *vcache, const void *wk_coded,
                                                    const void *wk_dense, const void *wv_coded,
                                                    const int32_t *len, const uint16_t *k0_f16,
                                                    int64_t k0_stride, const uint16_t *wk_row0_bf16,
                                                    void *terms, size_t terms_bytes, int32_t terms_valid,
                                                    float *out, void *workspace, size_t workspace_bytes,
                                                    void *stream);

#ifdef __cplusplus
}
#endif
#endif /* XQUANT_H */
