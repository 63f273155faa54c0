// C ABI of libxquant: argument validation on the host, then dispatch to the kernels.
#include <mutex>

#include "common.hpp"
#include "remat_layout.hpp"

namespace xq {

struct RematParams;   // defined in remat_attn.hip; re-declared field-for-field below via the builder

hipError_t run_quantize_append(const xq_cache_t* c, const uint16_t* x, const uint16_t* acc, int T,
                               const BatchI32& start, hipStream_t s);
hipError_t run_cl_accumulate(uint16_t* acc, const xq_cache_t* c, const BatchI32& len, int max_len,
                             bool init, hipStream_t s);
hipError_t run_prepare_weights(const WPrepLayout& L, const uint16_t* Wk, const uint16_t* Wv, int ncols,
                               int head_stride, void* out, hipStream_t s, bool transposed = false, bool nibbles = false);
hipError_t run_project_rows_dense(const uint16_t* x, long long M, int d, int n_lat, const void* proj, uint16_t* out,
                                  hipStream_t s);
hipError_t run_project_delta_rows_dense(const uint16_t* x, const uint16_t* acc, int B, int T, int cap, const BatchI32& start,
                                        int d, int n_lat, const void* proj, uint16_t* out, hipStream_t s);
hipError_t run_latent_project(const uint16_t* x, const uint16_t* ut, int M, int d, int n_lat, uint16_t* out,
                              hipStream_t s);
hipError_t run_remat_attn_decode(const xq_attn_t* a, const uint16_t* q, const xq_cache_t* xc,
                                 const uint16_t* acc, int B, int cap, int d, const void* wprep,
                                 const BatchI32& len, int max_len, float* out, void* ws,
                                 const float* rope, const BatchI32* pos0, hipStream_t s);
hipError_t run_remat_attn_decode_latent(const xq_attn_t* a, const uint16_t* q, const xq_cache_t* xc,
                                        const void* wprep, const BatchI32& len, int max_len, float* out, void* ws,
                                        hipStream_t s);
size_t remat_latent_workspace_bytes(int B, int Hq, int max_len, int r, int group);
hipError_t run_latent_delta_project(const uint16_t* x, const uint16_t* acc, const uint16_t* ut, int B, int T, int cap,
                                    const BatchI32& start, int d, int n_lat, uint16_t* out, hipStream_t s);
hipError_t run_quantize_blocks_per_channel(const xq_cache_t* c, const uint16_t* x, int nblk, const BatchI32& block0,
                                           hipStream_t s);
size_t remat_pc_workspace_bytes(int B, int Hq, int Hkv, int max_len, int d, int block);
hipError_t run_remat_attn_decode_pc(const xq_attn_t* a, const uint16_t* q, const xq_cache_t* xc, const uint16_t* tail,
                                    const void* wprep_coded, const void* wprep_dense, const BatchI32& len, int max_len,
                                    void* terms, bool terms_valid, float* out, void* ws, hipStream_t s);
size_t pc_terms_bytes(int B, int cap, int d, int block, int col_blocks);
size_t remat_latent_pc_workspace_bytes(int B, int Hq, int Hkv, int max_len, int r, int block, int v_group);
hipError_t run_remat_attn_decode_latent_pc(const xq_attn_t* a, const uint16_t* q, const xq_cache_t* kc,
                                           const uint16_t* ktail, const xq_cache_t* vc, const void* wk_coded,
                                           const void* wk_dense, const void* wv_coded, const BatchI32& len, int max_len,
                                           const uint16_t* k0_f16, long long k0_stride, const uint16_t* wk_row0,
                                           void* terms, bool terms_valid, float* out, void* ws, hipStream_t s);
size_t remat_prefill_workspace_bytes(int B, int T, int Hq, int max_len, int d, int group, bool coded);
hipError_t run_remat_attn_prefill(const xq_attn_t* a, const uint16_t* q, int T, const xq_cache_t* xc,
                                  const uint16_t* acc, int B, int cap, int d, const void* wprep,
                                  const BatchI32& len, int max_len, float* out, void* ws,
                                  const float* rope, const BatchI32* pos0, hipStream_t s);
size_t upproject_workspace_bytes(int B, int max_len, int n_lat, int group);
hipError_t run_cl_accumulate_latent(uint16_t* acc, const xq_cache_t* xc, int d, const void* uprep,
                                    const BatchI32& len, int max_len, void* ws, hipStream_t s);
size_t remat_workspace_bytes(int B, int Hq, int max_len, int d, int group, bool coded);

static bool fmt_ok(const xq_qfmt_t& f)
{
    const bool bits_ok = f.bits == 2 || f.bits == 3 || f.bits == 4 || f.bits == 8;
    const bool group_ok = f.group == 64 || f.group == 128;
    return bits_ok && group_ok && f.d > 0 && f.d % 128 == 0;
}

static xq_status_t check_cache(const xq_cache_t* c)
{
    if (!c || !c->codes || !c->scale || !c->zero) return XQ_ERR_INVALID_ARG;
    if (c->B < 1 || c->cap < 1) return XQ_ERR_INVALID_ARG;
    if (c->B > XQ_MAX_BATCH) return XQ_ERR_UNSUPPORTED;
    if (c->fmt.d <= 0 || c->fmt.group <= 0 || c->fmt.d % c->fmt.group != 0) return XQ_ERR_INVALID_ARG;
    if (!fmt_ok(c->fmt)) return XQ_ERR_UNSUPPORTED;
    if (!aligned16(c->codes) || !aligned16(c->scale) || !aligned16(c->zero)) return XQ_ERR_INVALID_ARG;
    // (the kernels address the rows of one sequence with 32-bit byte offsets)
    if ((long long)c->cap * c->fmt.d * c->fmt.bits / 8 >= (1LL << 32)) return XQ_ERR_UNSUPPORTED;
    return XQ_OK;
}

static xq_status_t check_attn(const xq_attn_t* a)
{
    if (!a) return XQ_ERR_INVALID_ARG;
    if (a->n_q_heads < 1 || a->n_kv_heads < 1 || a->n_q_heads % a->n_kv_heads != 0) return XQ_ERR_INVALID_ARG;
    if (a->head_dim != 128) return XQ_ERR_UNSUPPORTED;
    if (a->n_q_heads / a->n_kv_heads > 16) return XQ_ERR_UNSUPPORTED;
    return XQ_OK;
}

static bool wprep_combo_ok(int d, int group, int src_bits)
{
    if (d <= 0 || d % 128 != 0) return false;
    if (src_bits == 16) return true;
    return (src_bits == 2 || src_bits == 3 || src_bits == 4) && (group == 64 || group == 128);
}

// ... plus 8-bit per-token caches, which only the plain decode / prefill attention calls walk
static bool wprep_cache_combo_ok(int d, int group, int src_bits)
{
    if (src_bits == 8) return d > 0 && d % 128 == 0 && (group == 64 || group == 128);
    return wprep_combo_ok(d, group, src_bits);
}

}  // namespace xq

using namespace xq;

extern "C" {

const char* xq_status_string(xq_status_t s)
{
    switch (s) {
        case XQ_OK: return "ok";
        case XQ_ERR_INVALID_ARG: return "invalid argument";
        case XQ_ERR_UNSUPPORTED: return "unsupported shape or format";
        case XQ_ERR_WORKSPACE: return "workspace or output buffer too small";
        case XQ_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

int xq_version(void) { return 100; }

size_t xq_codes_row_bytes(const xq_qfmt_t* f)
{
    if (!f || f->d <= 0 || f->bits <= 0 || (f->d * f->bits) % 8 != 0) return 0;
    return (size_t)f->d * f->bits / 8;
}

size_t xq_meta_row_elems(const xq_qfmt_t* f)
{
    if (!f || f->d <= 0 || f->group <= 0 || f->d % f->group != 0) return 0;
    return (size_t)f->d / f->group;
}

static xq_status_t quantize_common(const xq_cache_t* cache, const uint16_t* x, const uint16_t* acc,
                                   bool need_acc, int32_t T, const int32_t* start, void* stream)
{
    xq_status_t st = check_cache(cache);
    if (st != XQ_OK) return st;
    if (!start || T < 0) return XQ_ERR_INVALID_ARG;
    if (T > 0 && (!x || !aligned16(x))) return XQ_ERR_INVALID_ARG;   // no rows: x is not read
    if (T > 0 && need_acc && (!acc || !aligned16(acc))) return XQ_ERR_INVALID_ARG;
    BatchI32 sv{};
    for (int b = 0; b < cache->B; ++b) {
        if (start[b] < 0 || (long long)start[b] + T > cache->cap) return XQ_ERR_INVALID_ARG;
        sv.v[b] = start[b];
    }
    if (T == 0) return XQ_OK;
    hipError_t e = run_quantize_append(cache, x, need_acc ? acc : nullptr, T, sv, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? XQ_OK : XQ_ERR_HIP;
}

xq_status_t xq_quantize_append(const xq_cache_t* cache, const uint16_t* x_bf16, int32_t T,
                               const int32_t* start, void* stream)
{
    return quantize_common(cache, x_bf16, nullptr, false, T, start, stream);
}

xq_status_t xq_cl_delta_quantize(const xq_cache_t* delta, const uint16_t* x_bf16, const uint16_t* acc_bf16,
                                 int32_t T, const int32_t* start, void* stream)
{
    return quantize_common(delta, x_bf16, acc_bf16, true, T, start, stream);
}

xq_status_t xq_cl_accumulate(uint16_t* acc_bf16, const xq_cache_t* src, const int32_t* len, int32_t init,
                             void* stream)
{
    xq_status_t st = check_cache(src);
    if (st != XQ_OK) return st;
    if (!acc_bf16 || !len || !aligned16(acc_bf16)) return XQ_ERR_INVALID_ARG;
    BatchI32 lv{};
    int max_len = 0;
    for (int b = 0; b < src->B; ++b) {
        if (len[b] < 0 || len[b] > src->cap) return XQ_ERR_INVALID_ARG;
        lv.v[b] = len[b];
        if (len[b] > max_len) max_len = len[b];
    }
    hipError_t e = run_cl_accumulate(acc_bf16, src, lv, max_len, init != 0, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? XQ_OK : XQ_ERR_HIP;
}

size_t xq_prepared_weights_bytes(const xq_attn_t* a, int32_t d, int32_t group, int32_t src_bits)
{
    if (check_attn(a) != XQ_OK || !wprep_cache_combo_ok(d, group, src_bits)) return 0;
    return make_wprep_layout_for_cache(d, group, src_bits, a->n_kv_heads).total_bytes;
}

xq_status_t xq_prepare_weights(const xq_attn_t* a, int32_t d, int32_t group, int32_t src_bits,
                               const uint16_t* Wk, const uint16_t* Wv, void* out, size_t out_bytes,
                               void* stream)
{
    xq_status_t st = check_attn(a);
    if (st != XQ_OK) return st;
    if (!Wk || !Wv || !out || !aligned16(Wk) || !aligned16(Wv) || !aligned16(out)) return XQ_ERR_INVALID_ARG;
    if (d <= 0) return XQ_ERR_INVALID_ARG;
    if (!wprep_cache_combo_ok(d, group, src_bits)) return XQ_ERR_UNSUPPORTED;
    const WPrepLayout L = make_wprep_layout_for_cache(d, group, src_bits, a->n_kv_heads);
    if (out_bytes < L.total_bytes) return XQ_ERR_WORKSPACE;
    hipError_t e = run_prepare_weights(L, Wk, Wv, a->n_kv_heads * 128, 128, out, static_cast<hipStream_t>(stream), false,
                                       src_bits == 8);
    return e == hipSuccess ? XQ_OK : XQ_ERR_HIP;
}

static bool latent_combo_ok(const xq_attn_t* a, int r, int group, int src_bits)
{
    return r > 0 && r % 128 == 0 && a->n_kv_heads % 2 == 0 && src_bits != 16 && wprep_combo_ok(r, group, src_bits);
}

size_t xq_prepared_weights_latent_bytes(const xq_attn_t* a, int32_t r, int32_t group, int32_t src_bits)
{
    if (check_attn(a) != XQ_OK || !latent_combo_ok(a, r, group, src_bits)) return 0;
    return 2 * make_wprep_layout_for_cache(r, group, src_bits, a->n_kv_heads / 2).total_bytes;
}

xq_status_t xq_prepare_weights_latent(const xq_attn_t* a, int32_t r, int32_t group, int32_t src_bits,
                                      const uint16_t* Wfk, const uint16_t* Wfv, void* out, size_t out_bytes,
                                      void* stream)
{
    xq_status_t st = check_attn(a);
    if (st != XQ_OK) return st;
    if (!Wfk || !Wfv || !out || !aligned16(Wfk) || !aligned16(Wfv) || !aligned16(out)) return XQ_ERR_INVALID_ARG;
    if (r <= 0) return XQ_ERR_INVALID_ARG;
    if (!latent_combo_ok(a, r, group, src_bits)) return XQ_ERR_UNSUPPORTED;
    // one stream per half; a stream's "head" is a pair of KV heads = 256 adjacent columns of the fused matrix
    const WPrepLayout L = make_wprep_layout_for_cache(r, group, src_bits, a->n_kv_heads / 2);
    if (out_bytes < 2 * L.total_bytes) return XQ_ERR_WORKSPACE;
    const int ncols = a->n_kv_heads * 128;
    hipError_t e = run_prepare_weights(L, Wfk, Wfk + 128, ncols, 256, out, static_cast<hipStream_t>(stream));
    if (e == hipSuccess)
        e = run_prepare_weights(L, Wfv, Wfv + 128, ncols, 256, static_cast<uint8_t*>(out) + L.total_bytes,
                                static_cast<hipStream_t>(stream));
    return e == hipSuccess ? XQ_OK : XQ_ERR_HIP;
}

xq_status_t xq_latent_project(const uint16_t* x_bf16, const uint16_t* Ut_bf16, int32_t M, int32_t d, int32_t n_lat,
                              uint16_t* out_bf16, void* stream)
{
    if (M < 0 || d <= 0 || n_lat <= 0) return XQ_ERR_INVALID_ARG;
    if (d % 128 != 0 || n_lat % 32 != 0) return XQ_ERR_UNSUPPORTED;
    if (M == 0) return XQ_OK;
    if (M > 65535 * 32) return XQ_ERR_UNSUPPORTED;
    if (!x_bf16 || !Ut_bf16 || !out_bf16 || !aligned16(x_bf16) || !aligned16(Ut_bf16) || !aligned16(out_bf16))
        return XQ_ERR_INVALID_ARG;
    hipError_t e = run_latent_project(x_bf16, Ut_bf16, M, d, n_lat, out_bf16, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? XQ_OK : XQ_ERR_HIP;
}

size_t xq_remat_attn_workspace_bytes(const xq_attn_t* a, int32_t B, int32_t max_len, int32_t d, int32_t group)
{
    if (check_attn(a) != XQ_OK || B < 1 || max_len < 1 || d <= 0 || d % 128 != 0) return 0;
    if (group != 0 && group != 64 && group != 128) return 0;
    return remat_workspace_bytes(B, a->n_q_heads, max_len, d, group ? group : 128, group != 0);
}

size_t xq_remat_attn_prefill_workspace_bytes(const xq_attn_t* a, int32_t B, int32_t T, int32_t max_len, int32_t d,
                                             int32_t group)
{
    if (check_attn(a) != XQ_OK || B < 1 || T < 1 || max_len < 1 || d <= 0 || d % 128 != 0) return 0;
    if (group != 0 && group != 64 && group != 128) return 0;
    return remat_prefill_workspace_bytes(B, T, a->n_q_heads, max_len, d, group ? group : 128, group != 0);
}

static xq_status_t remat_attn_common(const xq_attn_t* a, const uint16_t* q_bf16, const xq_cache_t* xcache,
                                     const uint16_t* acc_bf16, int32_t B, int32_t cap, int32_t d,
                                     const void* wprep, const int32_t* len, float* out, void* workspace,
                                     size_t workspace_bytes, const float* rope, int32_t rope_positions,
                                     const int32_t* pos0, void* stream, int32_t T = 0)
{
    // T = 0: one decode query per sequence; T >= 1: the T newest rows are queries (causal)
    xq_status_t st = check_attn(a);
    if (T < 0) return XQ_ERR_INVALID_ARG;
    if (st != XQ_OK) return st;
    if ((xcache != nullptr) == (acc_bf16 != nullptr)) return XQ_ERR_INVALID_ARG;
    if (!q_bf16 || !wprep || !len || !out || !workspace) return XQ_ERR_INVALID_ARG;
    if (!aligned16(q_bf16) || !aligned16(wprep) || !aligned16(out) || !aligned16(workspace))
        return XQ_ERR_INVALID_ARG;
    if (xcache) {
        st = check_cache(xcache);
        if (st != XQ_OK) return st;
        B = xcache->B; cap = xcache->cap; d = xcache->fmt.d;
    } else {
        if (!aligned16(acc_bf16) || B < 1 || cap < 1 || d <= 0) return XQ_ERR_INVALID_ARG;
        if (B > XQ_MAX_BATCH || d % 128 != 0) return XQ_ERR_UNSUPPORTED;
        if ((long long)cap * d * 2 >= (1LL << 32)) return XQ_ERR_UNSUPPORTED;     // (32-bit row offsets within a sequence)
    }
    BatchI32 lv{};
    int max_len = 0;
    for (int b = 0; b < B; ++b) {
        if (len[b] < 1 || len[b] > cap || len[b] < T) return XQ_ERR_INVALID_ARG;
        lv.v[b] = len[b];
        if (len[b] > max_len) max_len = len[b];
    }
    if (T > 0 && (long long)B * T > 65535) return XQ_ERR_UNSUPPORTED;
    // (an 8-bit cache is walked as 4-bit groups of 128 nibbles over twice the width)
    const bool nib = xcache && xcache->fmt.bits == 8;
    const int wd = nib ? 2 * d : d, wg = nib ? 128 : xcache ? xcache->fmt.group : 0;
    const size_t need = T > 0 ? xq_remat_attn_prefill_workspace_bytes(a, B, T, max_len, wd, wg)
                              : xq_remat_attn_workspace_bytes(a, B, max_len, wd, wg);
    if (need == 0) return XQ_ERR_UNSUPPORTED;
    if (workspace_bytes < need) return XQ_ERR_WORKSPACE;
    BatchI32 pv{};
    if (rope) {
        if (!pos0 || !aligned16(rope) || rope_positions < 1) return XQ_ERR_INVALID_ARG;
        for (int b = 0; b < B; ++b) {                     // every attended row must have a table row
            if (pos0[b] < 0 || (long long)pos0[b] + len[b] > rope_positions) return XQ_ERR_INVALID_ARG;
            pv.v[b] = pos0[b];
        }
    }
    hipError_t e = T > 0 ? run_remat_attn_prefill(a, q_bf16, T, xcache, acc_bf16, B, cap, d, wprep, lv, max_len, out,
                                                  workspace, rope, &pv, static_cast<hipStream_t>(stream))
                         : run_remat_attn_decode(a, q_bf16, xcache, acc_bf16, B, cap, d, wprep, lv, max_len, out,
                                                 workspace, rope, &pv, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? XQ_OK : XQ_ERR_HIP;
}

xq_status_t xq_remat_attn_decode(const xq_attn_t* a, const uint16_t* q_bf16, const xq_cache_t* xcache,
                                 const uint16_t* acc_bf16, int32_t B, int32_t cap, int32_t d,
                                 const void* wprep, const int32_t* len, float* out, void* workspace,
                                 size_t workspace_bytes, void* stream)
{
    return remat_attn_common(a, q_bf16, xcache, acc_bf16, B, cap, d, wprep, len, out, workspace, workspace_bytes,
                             nullptr, 0, nullptr, stream);
}

xq_status_t xq_remat_attn_decode_rope(const xq_attn_t* a, const uint16_t* q_bf16, const xq_cache_t* xcache,
                                      const uint16_t* acc_bf16, int32_t B, int32_t cap, int32_t d,
                                      const void* wprep, const int32_t* len, const float* rope_cos_sin,
                                      int32_t rope_positions, const int32_t* pos0, float* out, void* workspace,
                                      size_t workspace_bytes, void* stream)
{
    if (!rope_cos_sin) return XQ_ERR_INVALID_ARG;
    return remat_attn_common(a, q_bf16, xcache, acc_bf16, B, cap, d, wprep, len, out, workspace, workspace_bytes,
                             rope_cos_sin, rope_positions, pos0, stream);
}

size_t xq_remat_attn_latent_workspace_bytes(const xq_attn_t* a, int32_t B, int32_t max_len, int32_t r, int32_t group)
{
    if (check_attn(a) != XQ_OK || B < 1 || max_len < 1 || r <= 0 || r % 128 != 0) return 0;
    if (group != 64 && group != 128) return 0;
    return remat_latent_workspace_bytes(B, a->n_q_heads, max_len, r, group);
}

xq_status_t xq_remat_attn_decode_latent(const xq_attn_t* a, const uint16_t* q_bf16, const xq_cache_t* latent,
                                        const void* wprep, const int32_t* len, float* out, void* workspace,
                                        size_t workspace_bytes, void* stream)
{
    xq_status_t st = check_attn(a);
    if (st != XQ_OK) return st;
    if (!q_bf16 || !wprep || !len || !out || !workspace) return XQ_ERR_INVALID_ARG;
    if (!aligned16(q_bf16) || !aligned16(wprep) || !aligned16(out) || !aligned16(workspace)) return XQ_ERR_INVALID_ARG;
    st = check_cache(latent);
    if (st != XQ_OK) return st;
    if (latent->fmt.d % 256 != 0 || !latent_combo_ok(a, latent->fmt.d / 2, latent->fmt.group, latent->fmt.bits))
        return XQ_ERR_UNSUPPORTED;
    BatchI32 lv{};
    int max_len = 0;
    for (int b = 0; b < latent->B; ++b) {
        if (len[b] < 1 || len[b] > latent->cap) return XQ_ERR_INVALID_ARG;
        lv.v[b] = len[b];
        if (len[b] > max_len) max_len = len[b];
    }
    if (workspace_bytes < xq_remat_attn_latent_workspace_bytes(a, latent->B, max_len, latent->fmt.d / 2, latent->fmt.group))
        return XQ_ERR_WORKSPACE;
    hipError_t e = run_remat_attn_decode_latent(a, q_bf16, latent, wprep, lv, max_len, out, workspace,
                                                static_cast<hipStream_t>(stream));
    return e == hipSuccess ? XQ_OK : XQ_ERR_HIP;
}

xq_status_t xq_remat_attn_prefill(const xq_attn_t* a, const uint16_t* q_bf16, int32_t T, const xq_cache_t* xcache,
                                  const uint16_t* acc_bf16, int32_t B, int32_t cap, int32_t d, const void* wprep,
                                  const int32_t* len, const float* rope_cos_sin, int32_t rope_positions,
                                  const int32_t* pos0, float* out, void* workspace, size_t workspace_bytes,
                                  void* stream)
{
    if (T < 1) return XQ_ERR_INVALID_ARG;
    return remat_attn_common(a, q_bf16, xcache, acc_bf16, B, cap, d, wprep, len, out, workspace, workspace_bytes,
                             rope_cos_sin, rope_positions, pos0, stream, T);
}

// per-channel cache: the struct of a per-token cache with scale / zero [B][cap/group][d]
static xq_status_t check_cache_per_channel(const xq_cache_t* c)
{
    if (!c || !c->codes || !c->scale || !c->zero) return XQ_ERR_INVALID_ARG;
    if (c->B < 1 || c->cap < 1 || c->fmt.d <= 0 || c->fmt.group <= 0) return XQ_ERR_INVALID_ARG;
    if (c->B > XQ_MAX_BATCH) return XQ_ERR_UNSUPPORTED;
    if (c->fmt.group != 64 && c->fmt.group != 128) return XQ_ERR_UNSUPPORTED;
    if (c->fmt.bits != 2 && c->fmt.bits != 3 && c->fmt.bits != 4 && c->fmt.bits != 8) return XQ_ERR_UNSUPPORTED;
    if (c->fmt.d % 128 != 0) return XQ_ERR_UNSUPPORTED;
    if (c->cap % c->fmt.group != 0) return XQ_ERR_INVALID_ARG;
    if (!aligned16(c->codes) || !aligned16(c->scale) || !aligned16(c->zero)) return XQ_ERR_INVALID_ARG;
    if ((long long)c->cap * c->fmt.d * c->fmt.bits / 8 >= (1LL << 32)) return XQ_ERR_UNSUPPORTED;   // (32-bit row offsets)
    return XQ_OK;
}

xq_status_t xq_quantize_blocks_per_channel(const xq_cache_t* cache, const uint16_t* x_bf16, int32_t nblk,
                                           const int32_t* block0, void* stream)
{
    xq_status_t st = check_cache_per_channel(cache);
    if (st != XQ_OK) return st;
    if (!block0 || nblk < 0) return XQ_ERR_INVALID_ARG;
    BatchI32 bv{};
    for (int b = 0; b < cache->B; ++b) {
        if (block0[b] < 0 || ((long long)block0[b] + nblk) * cache->fmt.group > cache->cap) return XQ_ERR_INVALID_ARG;
        bv.v[b] = block0[b];
    }
    if (nblk == 0) return XQ_OK;
    if (nblk > 65535) return XQ_ERR_UNSUPPORTED;
    if (!x_bf16 || !aligned16(x_bf16)) return XQ_ERR_INVALID_ARG;
    hipError_t e = run_quantize_blocks_per_channel(cache, x_bf16, nblk, bv, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? XQ_OK : XQ_ERR_HIP;
}

size_t xq_remat_attn_per_channel_workspace_bytes(const xq_attn_t* a, int32_t B, int32_t max_len, int32_t d, int32_t group)
{
    if (check_attn(a) != XQ_OK || B < 1 || max_len < 1 || d <= 0 || d % 128 != 0) return 0;
    if (group != 64 && group != 128) return 0;
    return remat_pc_workspace_bytes(B, a->n_q_heads, a->n_kv_heads, max_len, d, group);
}

size_t xq_per_channel_terms_bytes(int32_t B, int32_t cap, int32_t d, int32_t group, int32_t col_blocks)
{
    if (B < 1 || B > XQ_MAX_BATCH || cap < 1 || d <= 0 || d % 128 != 0 || col_blocks < 1) return 0;
    if ((group != 64 && group != 128) || cap % group != 0) return 0;
    return pc_terms_bytes(B, cap, d, group, col_blocks);
}

xq_status_t xq_remat_attn_decode_per_channel(const xq_attn_t* a, const uint16_t* q_bf16, const xq_cache_t* cache,
                                             const uint16_t* tail_bf16, const int32_t* len, const void* wprep_coded,
                                             const void* wprep_dense, void* terms, size_t terms_bytes,
                                             int32_t terms_valid, float* out, void* workspace,
                                             size_t workspace_bytes, void* stream)
{
    xq_status_t st = check_attn(a);
    if (st != XQ_OK) return st;
    st = check_cache_per_channel(cache);
    if (st != XQ_OK) return st;
    if (cache->fmt.bits == 8) return XQ_ERR_UNSUPPORTED;
    if (!q_bf16 || !tail_bf16 || !len || !wprep_coded || !wprep_dense || !out || !workspace) return XQ_ERR_INVALID_ARG;
    if (!aligned16(q_bf16) || !aligned16(tail_bf16) || !aligned16(wprep_coded) || !aligned16(wprep_dense) ||
        !aligned16(out) || !aligned16(workspace))
        return XQ_ERR_INVALID_ARG;
    BatchI32 lv{};
    int max_len = 0;
    for (int b = 0; b < cache->B; ++b) {
        // the blocks must fit the cache; the window holds at most group - 1 tokens by construction
        if (len[b] < 1 || (len[b] / cache->fmt.group) * cache->fmt.group > cache->cap) return XQ_ERR_INVALID_ARG;
        lv.v[b] = len[b];
        if (len[b] > max_len) max_len = len[b];
    }
    if (workspace_bytes < xq_remat_attn_per_channel_workspace_bytes(a, cache->B, max_len, cache->fmt.d, cache->fmt.group))
        return XQ_ERR_WORKSPACE;
    if (terms) {
        if (!aligned16(terms)) return XQ_ERR_INVALID_ARG;
        if (terms_bytes < pc_terms_bytes(cache->B, cache->cap, cache->fmt.d, cache->fmt.group, a->n_kv_heads)) return XQ_ERR_WORKSPACE;
    }
    hipError_t e = run_remat_attn_decode_pc(a, q_bf16, cache, tail_bf16, wprep_coded, wprep_dense, lv, max_len, terms,
                                            terms_valid != 0, out, workspace, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? XQ_OK : XQ_ERR_HIP;
}

// one fused latent matrix (Sec. 3.3.1) as a prepared stream whose "head" is a pair of KV heads
static bool pairs_combo_ok(const xq_attn_t* a, int r, int group, int src_bits)
{
    return r > 0 && r % 128 == 0 && a->n_kv_heads % 2 == 0 && wprep_combo_ok(r, group, src_bits);
}

size_t xq_prepared_weights_pairs_bytes(const xq_attn_t* a, int32_t r, int32_t group, int32_t src_bits)
{
    if (check_attn(a) != XQ_OK || !pairs_combo_ok(a, r, group, src_bits)) return 0;
    return pairs_layout(r, group, src_bits, a->n_kv_heads / 2).total_bytes;
}

xq_status_t xq_prepare_weights_pairs(const xq_attn_t* a, int32_t r, int32_t group, int32_t src_bits, const uint16_t* Wf,
                                     void* out, size_t out_bytes, void* stream)
{
    xq_status_t st = check_attn(a);
    if (st != XQ_OK) return st;
    if (!Wf || !out || !aligned16(Wf) || !aligned16(out) || r <= 0) return XQ_ERR_INVALID_ARG;
    if (!pairs_combo_ok(a, r, group, src_bits)) return XQ_ERR_UNSUPPORTED;
    const WPrepLayout L = pairs_layout(r, group, src_bits, a->n_kv_heads / 2);
    if (out_bytes < L.total_bytes) return XQ_ERR_WORKSPACE;
    hipError_t e = run_prepare_weights(L, Wf, Wf + 128, a->n_kv_heads * 128, 256, out, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? XQ_OK : XQ_ERR_HIP;
}

size_t xq_remat_attn_latent_per_channel_workspace_bytes(const xq_attn_t* a, int32_t B, int32_t max_len, int32_t r,
                                                        int32_t k_group, int32_t v_group)
{
    if (check_attn(a) != XQ_OK || B < 1 || max_len < 1 || r <= 0 || r % 128 != 0 || a->n_kv_heads % 2 != 0) return 0;
    if ((k_group != 64 && k_group != 128) || (v_group != 64 && v_group != 128)) return 0;
    return remat_latent_pc_workspace_bytes(B, a->n_q_heads, a->n_kv_heads, max_len, r, k_group, v_group);
}

xq_status_t xq_remat_attn_decode_latent_per_channel(const xq_attn_t* a, const uint16_t* q_bf16, const xq_cache_t* kcache,
                                                    const uint16_t* ktail_bf16, const xq_cache_t* vcache,
                                                    const void* wk_coded, const void* wk_dense, const void* wv_coded,
                                                    const int32_t* len, const uint16_t* k0_f16, int64_t k0_stride,
                                                    const uint16_t* wk_row0_bf16, void* terms, size_t terms_bytes,
                                                    int32_t terms_valid, float* out, void* workspace,
                                                    size_t workspace_bytes, void* stream)
{
    xq_status_t st = check_attn(a);
    if (st != XQ_OK) return st;
    st = check_cache_per_channel(kcache);
    if (st != XQ_OK) return st;
    st = check_cache(vcache);
    if (st != XQ_OK) return st;
    if (kcache->fmt.bits == 8 || vcache->fmt.bits == 8 || a->n_kv_heads % 2 != 0) return XQ_ERR_UNSUPPORTED;
    if (vcache->fmt.d != kcache->fmt.d || vcache->B != kcache->B) return XQ_ERR_INVALID_ARG;
    if (!pairs_combo_ok(a, vcache->fmt.d, vcache->fmt.group, vcache->fmt.bits)) return XQ_ERR_UNSUPPORTED;
    if (!q_bf16 || !ktail_bf16 || !len || !wk_coded || !wk_dense || !wv_coded || !out || !workspace) return XQ_ERR_INVALID_ARG;
    if (!aligned16(q_bf16) || !aligned16(ktail_bf16) || !aligned16(wk_coded) || !aligned16(wk_dense) || !aligned16(wv_coded) ||
        !aligned16(out) || !aligned16(workspace))
        return XQ_ERR_INVALID_ARG;
    BatchI32 lv{};
    int max_len = 0;
    for (int b = 0; b < kcache->B; ++b) {
        if (len[b] < 1 || len[b] > vcache->cap || (len[b] / kcache->fmt.group) * kcache->fmt.group > kcache->cap)
            return XQ_ERR_INVALID_ARG;
        lv.v[b] = len[b];
        if (len[b] > max_len) max_len = len[b];
    }
    if (workspace_bytes < xq_remat_attn_latent_per_channel_workspace_bytes(a, kcache->B, max_len, kcache->fmt.d,
                                                                           kcache->fmt.group, vcache->fmt.group))
        return XQ_ERR_WORKSPACE;
    if (terms) {
        if (!aligned16(terms)) return XQ_ERR_INVALID_ARG;
        if (terms_bytes < pc_terms_bytes(kcache->B, kcache->cap, kcache->fmt.d, kcache->fmt.group, a->n_kv_heads / 2))
            return XQ_ERR_WORKSPACE;
    }
    if (k0_f16 && (!wk_row0_bf16 || k0_stride < max_len)) return XQ_ERR_INVALID_ARG;
    hipError_t e = run_remat_attn_decode_latent_pc(a, q_bf16, kcache, ktail_bf16, vcache, wk_coded, wk_dense, wv_coded, lv,
                                                   max_len, k0_f16, k0_stride, wk_row0_bf16, terms, terms_valid != 0, out,
                                                   workspace, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? XQ_OK : XQ_ERR_HIP;
}

// bulk projection (prefill-sized M) through the dense-source contraction kernel
size_t xq_prepared_projection_bytes(int32_t d, int32_t n_lat)
{
    if (d <= 0 || d % 128 != 0 || n_lat <= 0 || n_lat % 256 != 0) return 0;
    return make_wprep_layout(d, 128, 16, n_lat / 256).total_bytes;
}

xq_status_t xq_prepare_projection(int32_t d, int32_t n_lat, const uint16_t* Ut_bf16, void* out, size_t out_bytes,
                                  void* stream)
{
    if (!Ut_bf16 || !out || !aligned16(Ut_bf16) || !aligned16(out) || d <= 0 || n_lat <= 0) return XQ_ERR_INVALID_ARG;
    const size_t need = xq_prepared_projection_bytes(d, n_lat);
    if (need == 0) return XQ_ERR_UNSUPPORTED;
    if (out_bytes < need) return XQ_ERR_WORKSPACE;
    const WPrepLayout L = make_wprep_layout(d, 128, 16, n_lat / 256);
    hipError_t e = run_prepare_weights(L, Ut_bf16, Ut_bf16 + (size_t)128 * d, n_lat, 256, out,
                                       static_cast<hipStream_t>(stream), true);
    return e == hipSuccess ? XQ_OK : XQ_ERR_HIP;
}

xq_status_t xq_latent_project_bulk(const uint16_t* x_bf16, const void* proj, int64_t M, int32_t d, int32_t n_lat,
                                   uint16_t* out_bf16, void* stream)
{
    if (M < 0 || d <= 0 || n_lat <= 0) return XQ_ERR_INVALID_ARG;
    // (the kernel addresses the rows of a sequence with 32-bit byte offsets)
    if (xq_prepared_projection_bytes(d, n_lat) == 0 || M * (long long)d * 2 >= (1LL << 32)) return XQ_ERR_UNSUPPORTED;
    if (M == 0) return XQ_OK;
    if (!x_bf16 || !proj || !out_bf16 || !aligned16(x_bf16) || !aligned16(proj) || !aligned16(out_bf16))
        return XQ_ERR_INVALID_ARG;
    hipError_t e = run_project_rows_dense(x_bf16, M, d, n_lat, proj, out_bf16, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? XQ_OK : XQ_ERR_HIP;
}

xq_status_t xq_cl_latent_delta_project_bulk(const uint16_t* x_bf16, const uint16_t* acc_bf16, const void* proj, int32_t B,
                                            int32_t T, int32_t cap, const int32_t* start, int32_t d, int32_t n_lat,
                                            uint16_t* out_bf16, void* stream)
{
    if (B < 1 || T < 0 || cap < 1 || d <= 0 || n_lat <= 0 || !start) return XQ_ERR_INVALID_ARG;
    if (B > XQ_MAX_BATCH || xq_prepared_projection_bytes(d, n_lat) == 0) return XQ_ERR_UNSUPPORTED;
    // (the kernel addresses the rows of either tensor with 32-bit byte offsets)
    if ((long long)B * T * d * 2 >= (1LL << 32) || (long long)B * cap * d * 2 >= (1LL << 32)) return XQ_ERR_UNSUPPORTED;
    BatchI32 sv{};
    for (int b = 0; b < B; ++b) {
        if (start[b] < 0 || (long long)start[b] + T > cap) return XQ_ERR_INVALID_ARG;
        sv.v[b] = start[b];
    }
    if (T == 0) return XQ_OK;
    if (!x_bf16 || !acc_bf16 || !proj || !out_bf16) return XQ_ERR_INVALID_ARG;
    if (!aligned16(x_bf16) || !aligned16(acc_bf16) || !aligned16(proj) || !aligned16(out_bf16)) return XQ_ERR_INVALID_ARG;
    hipError_t e = run_project_delta_rows_dense(x_bf16, acc_bf16, B, T, cap, sv, d, n_lat, proj, out_bf16,
                                                static_cast<hipStream_t>(stream));
    return e == hipSuccess ? XQ_OK : XQ_ERR_HIP;
}

static bool upproject_combo_ok(int d, int n_lat, int group, int src_bits)
{
    return d > 0 && d % 256 == 0 && src_bits != 16 && wprep_combo_ok(n_lat, group, src_bits);
}

xq_status_t xq_cl_latent_delta_project(const uint16_t* x_bf16, const uint16_t* acc_bf16, const uint16_t* Ut_bf16,
                                       int32_t B, int32_t T, int32_t cap, const int32_t* start, int32_t d,
                                       int32_t n_lat, uint16_t* out_bf16, void* stream)
{
    if (B < 1 || T < 0 || cap < 1 || d <= 0 || n_lat <= 0 || !start) return XQ_ERR_INVALID_ARG;
    if (B > XQ_MAX_BATCH || d % 128 != 0 || n_lat % 32 != 0) return XQ_ERR_UNSUPPORTED;
    BatchI32 sv{};
    for (int b = 0; b < B; ++b) {
        if (start[b] < 0 || (long long)start[b] + T > cap) return XQ_ERR_INVALID_ARG;
        sv.v[b] = start[b];
    }
    if (T == 0) return XQ_OK;
    if ((long long)B * T > 65535LL * 32) return XQ_ERR_UNSUPPORTED;
    if (!x_bf16 || !acc_bf16 || !Ut_bf16 || !out_bf16 || !aligned16(x_bf16) || !aligned16(acc_bf16) ||
        !aligned16(Ut_bf16) || !aligned16(out_bf16))
        return XQ_ERR_INVALID_ARG;
    hipError_t e = run_latent_delta_project(x_bf16, acc_bf16, Ut_bf16, B, T, cap, sv, d, n_lat, out_bf16,
                                            static_cast<hipStream_t>(stream));
    return e == hipSuccess ? XQ_OK : XQ_ERR_HIP;
}

size_t xq_prepared_upproject_bytes(int32_t d, int32_t n_lat, int32_t group, int32_t src_bits)
{
    if (!upproject_combo_ok(d, n_lat, group, src_bits)) return 0;
    return make_wprep_layout(n_lat, group, src_bits, d / 256).total_bytes;
}

xq_status_t xq_prepare_upproject(int32_t d, int32_t n_lat, int32_t group, int32_t src_bits, const uint16_t* Ut_bf16,
                                 void* out, size_t out_bytes, void* stream)
{
    if (!Ut_bf16 || !out || !aligned16(Ut_bf16) || !aligned16(out) || d <= 0 || n_lat <= 0) return XQ_ERR_INVALID_ARG;
    if (!upproject_combo_ok(d, n_lat, group, src_bits)) return XQ_ERR_UNSUPPORTED;
    // the contraction runs over the latent channels; a "head" is 256 adjacent hidden channels
    const WPrepLayout L = make_wprep_layout(n_lat, group, src_bits, d / 256);
    if (out_bytes < L.total_bytes) return XQ_ERR_WORKSPACE;
    hipError_t e = run_prepare_weights(L, Ut_bf16, Ut_bf16 + 128, d, 256, out, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? XQ_OK : XQ_ERR_HIP;
}

size_t xq_cl_accumulate_latent_workspace_bytes(int32_t B, int32_t max_len, int32_t n_lat, int32_t group)
{
    if (B < 1 || max_len < 1 || n_lat <= 0 || (group != 64 && group != 128) || n_lat % 128 != 0) return 0;
    return upproject_workspace_bytes(B, max_len, n_lat, group);
}

xq_status_t xq_cl_accumulate_latent(uint16_t* acc_bf16, const xq_cache_t* delta, int32_t d, const void* uprep,
                                    const int32_t* len, void* workspace, size_t workspace_bytes, void* stream)
{
    xq_status_t st = check_cache(delta);
    if (st != XQ_OK) return st;
    if (!acc_bf16 || !uprep || !len || !aligned16(acc_bf16) || !aligned16(uprep) || d <= 0) return XQ_ERR_INVALID_ARG;
    if (!upproject_combo_ok(d, delta->fmt.d, delta->fmt.group, delta->fmt.bits)) return XQ_ERR_UNSUPPORTED;
    BatchI32 lv{};
    int max_len = 0;
    for (int b = 0; b < delta->B; ++b) {
        if (len[b] < 0 || len[b] > delta->cap) return XQ_ERR_INVALID_ARG;
        lv.v[b] = len[b];
        if (len[b] > max_len) max_len = len[b];
    }
    if (max_len == 0) return XQ_OK;
    if (!workspace || !aligned16(workspace)) return XQ_ERR_INVALID_ARG;
    if (workspace_bytes < upproject_workspace_bytes(delta->B, max_len, delta->fmt.d, delta->fmt.group))
        return XQ_ERR_WORKSPACE;
    hipError_t e = run_cl_accumulate_latent(acc_bf16, delta, d, uprep, lv, max_len, workspace,
                                            static_cast<hipStream_t>(stream));
    return e == hipSuccess ? XQ_OK : XQ_ERR_HIP;
}

// ---- decode attention for callers that cannot allocate ------------------------------------------
// The workspace of xq_remat_attn_decode (softmax partials + the tile-ordered scale copy) lives in a
// file-scope device array instead of a caller buffer.  Every GPU the library runs on holds its own
// copy of the array at its own address until the process ends; the address is looked up once per
// device, with that device current, and kept.  In host code the array's name is only a handle for
// that lookup: kernels and memory calls get the looked-up pointer.
static __device__ __attribute__((used)) __align__(256) unsigned char scratch[XQ_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES];
std::mutex g_scratch_mutex;

xq_status_t static_scratch_of_current_device(void** ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return XQ_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return XQ_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return XQ_OK;
}
}  // namespace

xq_status_t xq_remat_attn_decode_static(const xq_attn_t* a, const uint16_t* q_bf16, const xq_cache_t* xcache,
                                        const uint16_t* acc_bf16, int32_t B, int32_t cap, int32_t d,
                                        const void* wprep, const int32_t* len, float* out, void* stream)
{
    // size check first, on the host, from the same query the caller-workspace entry point uses
    xq_status_t st = check_attn(a);
    if (st != XQ_OK) return st;
    if ((xcache != nullptr) == (acc_bf16 != nullptr) || !len) return XQ_ERR_INVALID_ARG;
    if (xcache) {
        st = check_cache(xcache);
        if (st != XQ_OK) return st;
        B = xcache->B; cap = xcache->cap; d = xcache->fmt.d;
    } else if (B < 1 || B > XQ_MAX_BATCH) {
        return B < 1 ? XQ_ERR_INVALID_ARG : XQ_ERR_UNSUPPORTED;
    }
    int max_len = 0;
    for (int b = 0; b < B; ++b) {
        if (len[b] < 1 || len[b] > cap) return XQ_ERR_INVALID_ARG;
        if (len[b] > max_len) max_len = len[b];
    }
    const bool nib = xcache && xcache->fmt.bits == 8;
    const size_t need = xq_remat_attn_workspace_bytes(a, B, max_len, nib ? 2 * d : d, nib ? 128 : xcache ? xcache->fmt.group : 0);
    if (need == 0) return XQ_ERR_UNSUPPORTED;
    if (need > (size_t)XQ_STATIC_SCRATCH_BYTES) return XQ_ERR_WORKSPACE;     // beyond the built-in buffer
    void* ws = nullptr;
    st = static_scratch_of_current_device(&ws);
    if (st != XQ_OK) return st;
    // nothing in the buffer has to start at zero: the scale pre-pass and the attention kernel write every
    // element that the combine reads for these lengths
    return remat_attn_common(a, q_bf16, xcache, acc_bf16, B, cap, d, wprep, len, out, ws, XQ_STATIC_SCRATCH_BYTES,
                             nullptr, 0, nullptr, stream);
}

}  // extern "C"
