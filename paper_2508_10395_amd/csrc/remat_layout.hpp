// Layout of the prepared weight stream consumed by the rematerialisation kernel.
//
// Per KV head: (n_main_slabs + n_corr_slabs) slabs of 64 KiB.  A slab is the LDS
// image of 8 MFMA k-steps (128 contraction indices) x 256 output columns
// ([Wk_h | Wv_h]):  [k-step 8][column block 8][lane 64][8 bf16], i.e. one 1 KiB
// 32x16 operand fragment per (k-step, column block), lane-major, so that the copy
// HBM -> LDS is linear and every lane's ds_read_b128 is conflict-free.
//
// Lane l feeds row (l % 32) of its column block and, with half = l / 32, the
// contraction slots
//   dense source:  slab s covers hidden channels [128 s, 128 s + 128):
//                  channel = 128 s + 16 ks + 8 half + i
//   coded source:  the kernel walks the d/16 k-steps cyclically and column block nb
//                  runs 7 - nb k-steps behind the walk, so position (slab s, k-step
//                  ks, block nb) holds k-step kappa = (8 s + ks - (7 - nb)) mod (d/16)
//                  = (slab s', k-step ks'):  group gi = ks' / (G/16); unit u, k-step j
//                  inside the unit;
//                  channel = 128 s' + G gi + (G/2) half + 32 u + code_of_slot[j][i],
//                  value scaled by 2^wexp_of_code (see unpack.hpp).
// Main slabs hold bf16 for the dense source and fp16 for coded sources.  fp16 has five exponent bits, so a
// coded stream is normalised per head: every weight of head h is multiplied by 2^shift[h], chosen so
// that the head's largest entry sits at the top of the fp16 range (exact: a power of two; entries
// more than 2^-29 below the largest are then still normal numbers).  shift[Hkv] (int32) follows the
// column sums; the kernel takes 2^-shift[h] out again with its final scale.
// Correction slabs (coded sources only, bf16) hold, for contraction index
// kappa = 16 kk + 8 half + i, term = kappa / ng_pad, group g = kappa % ng_pad:
//   term 0,1,2: bf16 hi, mid, lo parts of S_g[n] = sum of the group's weight rows
// against which the kernel multiplies the stored zero-points.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace xq {

constexpr int SLAB_KSTEPS = 8;
constexpr int SLAB_BYTES = 65536;
constexpr int N_CORR_TERMS = 3;
constexpr int COL_BLOCK_LAG_MAX = 7;  // coded sources: column block nb lags by 7 - nb k-steps
constexpr int TILE_TOKENS = 256;     // tokens per workgroup
constexpr int CHUNK_TOKENS = 32;     // tokens per wave = one softmax partial

struct WPrepLayout {
    int d, G, bits, Hkv;
    int n_main_slabs, ng, ng_pad, n_corr_ksteps, n_corr_slabs;
    size_t head_bytes, stream_bytes, colsum_bytes, shift_bytes, total_bytes;
    // second stream, in 16-column fragments (see below); 0 bytes when the combination has none
    int t16_n_corr_ticks, t16_n_corr_slabs;
    size_t t16_offset, t16_head_bytes, t16_bytes;
};

inline WPrepLayout make_wprep_layout(int d, int G, int bits, int Hkv)
{
    WPrepLayout L{};
    L.d = d; L.G = G; L.bits = bits; L.Hkv = Hkv;
    L.n_main_slabs = d / 128;
    if (bits == 16) {
        L.ng = L.ng_pad = L.n_corr_ksteps = L.n_corr_slabs = 0;
    } else {
        L.ng = d / G;
        L.ng_pad = (L.ng + 7) / 8 * 8;
        L.n_corr_ksteps = (N_CORR_TERMS * L.ng_pad + 15) / 16;
        L.n_corr_slabs = (L.n_corr_ksteps + SLAB_KSTEPS - 1) / SLAB_KSTEPS;
    }
    L.head_bytes = (size_t)(L.n_main_slabs + L.n_corr_slabs) * SLAB_BYTES;
    L.stream_bytes = L.head_bytes * Hkv;
    L.colsum_bytes = (size_t)Hkv * L.ng * 256 * sizeof(float);
    L.shift_bytes = bits == 16 ? 0 : ((size_t)Hkv * sizeof(int32_t) + 15) / 16 * 16;   // per-head exponent shift of the fp16 stream
    L.total_bytes = L.stream_bytes + L.colsum_bytes + L.shift_bytes;
    return L;
}

// An 8-bit per-token cache is walked as a 4-bit cache of twice the width: a code's low and high nibble are
// two adjacent 4-bit codes of the row's bit string, the weight row of the high nibble is 16 times the code's
// (exact), and a group of G codes is 2 G / 128 groups of 128 nibbles that share its scale and zero-point.
// Twice the matrix work of a 4-bit cache; x^ = (16 hi + lo) scale + zero comes out exactly as for the
// other widths.
//
// Second stream ("16-column fragments"), for the kernels built on v_mfma_f32_16x16x32 (remat_attn16.hip; coded
// sources with groups of 128 codes -- 2-bit codes also with groups of 64 -- and the dense source, decode and prefill).  Same slabs of 64 KiB, but a slab is 4 ticks of 32
// contraction indices x 16 column tiles:  [tick 4][tile 16][lane 64][8 fp16], one 1 KiB 16 x 32 fragment per
// (tick, tile); lane l feeds column 16 tile + l % 16 and, with quarter q = l / 16, the slots
//   channel = 128 s' + 32 q + code_of_slot[j'][i]      (unit q of the slab's 128 codes, k-step j' of the unit)
// (groups of 64: channel = 128 s' + 32 j' + code_of_slot[q][i]: tick j' is unit j' of the slab, quarter q its k-step
// q, so that a tick stays inside one group)
// of the k32-step kappa = 4 s' + j' that the position holds: tile ct runs TILE16_LAG(ct) ticks behind the walk,
// so position (slab s, tick j, tile ct) holds kappa = (4 s + j - lag) mod (d / 32).  Correction slabs (bf16):
// contraction index 32 kk + 8 q + i -> term, group as in the first stream.  It follows the first stream's
// column sums and shifts (which it shares) at t16_offset.  The dense source's second stream holds bf16 in
// natural order and without lag: position (slab s, tick j, tile ct), lane l holds channels 128 s + 32 j + 8 q + i.
constexpr int TILE16_TICKS = 4;                       // k32-steps per slab
constexpr int tile16_lag(int ct) { return 3 - (ct >> 2); }

inline WPrepLayout make_wprep_layout_for_cache(int d, int G, int bits, int Hkv)
{
    WPrepLayout L = bits == 8 ? make_wprep_layout(2 * d, 128, 4, Hkv) : make_wprep_layout(d, bits == 16 ? 128 : G, bits, Hkv);
    if (L.bits == 16 || L.G == 128 || (L.G == 64 && L.bits == 2)) {
        L.t16_n_corr_ticks = L.bits == 16 ? 0 : (N_CORR_TERMS * L.ng_pad + 31) / 32;
        L.t16_n_corr_slabs = (L.t16_n_corr_ticks + TILE16_TICKS - 1) / TILE16_TICKS;
        L.t16_head_bytes = (size_t)(L.n_main_slabs + L.t16_n_corr_slabs) * SLAB_BYTES;
        L.t16_bytes = L.t16_head_bytes * Hkv;
        L.t16_offset = L.total_bytes;
        L.total_bytes += L.t16_bytes;
    }
    return L;
}

// A stream whose "head" is a pair of KV heads (one fused latent matrix, Sec. 3.3.1): coded streams carry the
// 16-column fragments too (the value pass runs on them), dense ones (the window's and the zero-point rows') do not.
inline WPrepLayout pairs_layout(int r, int G, int bits, int pairs)
{
    return bits == 16 ? make_wprep_layout(r, 128, 16, pairs) : make_wprep_layout_for_cache(r, G, bits, pairs);
}

}  // namespace xq
