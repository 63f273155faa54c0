"""ctypes front-end of the CPU oracle (oracle/xq_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke entry and by the
benchmark's cpu_baseline leg.  The product package never imports this module.
All arrays are host numpy arrays; bf16 tensors travel as uint16 bit patterns.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_LIB = None


def lib():
    global _LIB
    if _LIB is None:
        _LIB = C.CDLL(_build.build())
        _LIB.xqo_max_threads.restype = C.c_int
    return _LIB


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _c(a, dtype):
    a = np.ascontiguousarray(a)
    assert a.dtype == dtype, (a.dtype, dtype)
    return a


def max_threads():
    return int(lib().xqo_max_threads())


def bf16_to_f32(bits):
    bits = _c(bits, np.uint16)
    out = np.empty(bits.shape, np.float32)
    lib().xqo_bf16_to_f32(_p(bits), C.c_int64(bits.size), _p(out))
    return out


def f32_to_bf16(x):
    x = _c(x, np.float32)
    out = np.empty(x.shape, np.uint16)
    lib().xqo_f32_to_bf16(_p(x), C.c_int64(x.size), _p(out))
    return out


def quantize_rows(x_f32, G, bits):
    """x_f32 [..., d] fp32 -> (codes u8 [..., d], scale u16 [..., d/G], zero u16 [..., d/G])."""
    x = _c(x_f32, np.float32)
    d = x.shape[-1]
    rows = x.size // d
    assert d % G == 0
    codes = np.empty(x.shape, np.uint8)
    scale = np.empty(x.shape[:-1] + (d // G,), np.uint16)
    zero = np.empty_like(scale)
    lib().xqo_quantize_rows(_p(x), C.c_int64(rows), C.c_int(d), C.c_int(G), C.c_int(bits),
                            _p(codes), _p(scale), _p(zero))
    return codes, scale, zero


def quantize_blocks_per_channel(x_f32, G, bits):
    """Per-channel groups of G consecutive tokens: x [..., nblk*G, d] fp32 -> codes uint8 same shape,
    scale / zero bf16 bits [..., nblk, d]."""
    x = _c(x_f32, np.float32)
    rows, d = x.shape[-2], x.shape[-1]
    assert rows % G == 0
    lead = int(np.prod(x.shape[:-2], dtype=np.int64))
    nblk = lead * (rows // G)
    codes = np.empty(x.shape, np.uint8)
    scale = np.empty(x.shape[:-2] + (rows // G, d), np.uint16)
    zero = np.empty_like(scale)
    lib().xqo_quantize_blocks_per_channel(_p(x), C.c_int64(nblk), C.c_int(d), C.c_int(G), C.c_int(bits),
                                          _p(codes), _p(scale), _p(zero))
    return codes, scale, zero


def dequantize_blocks_per_channel(codes, scale, zero, G):
    codes = _c(codes, np.uint8)
    scale = _c(scale, np.uint16)
    zero = _c(zero, np.uint16)
    rows, d = codes.shape[-2], codes.shape[-1]
    lead = int(np.prod(codes.shape[:-2], dtype=np.int64))
    out = np.empty(codes.shape, np.float32)
    lib().xqo_dequantize_blocks_per_channel(_p(codes), _p(scale), _p(zero), C.c_int64(lead * (rows // G)), C.c_int(d),
                                            C.c_int(G), _p(out))
    return out


def pack_rows(codes, bits):
    codes = _c(codes, np.uint8)
    d = codes.shape[-1]
    rows = codes.size // d
    assert (d * bits) % 8 == 0
    packed = np.empty(codes.shape[:-1] + (d * bits // 8,), np.uint8)
    lib().xqo_pack_rows(_p(codes), C.c_int64(rows), C.c_int(d), C.c_int(bits), _p(packed))
    return packed


def unpack_rows(packed, d, bits):
    packed = _c(packed, np.uint8)
    rb = packed.shape[-1]
    assert rb == d * bits // 8
    rows = packed.size // rb
    codes = np.empty(packed.shape[:-1] + (d,), np.uint8)
    lib().xqo_unpack_rows(_p(packed), C.c_int64(rows), C.c_int(d), C.c_int(bits), _p(codes))
    return codes


def dequantize_rows(codes, scale, zero, G):
    codes = _c(codes, np.uint8)
    scale = _c(scale, np.uint16)
    zero = _c(zero, np.uint16)
    d = codes.shape[-1]
    rows = codes.size // d
    out = np.empty(codes.shape, np.float32)
    lib().xqo_dequantize_rows(_p(codes), _p(scale), _p(zero), C.c_int64(rows), C.c_int(d),
                              C.c_int(G), _p(out))
    return out


def cl_delta_rows(x_bf16, acc_bf16):
    x = _c(x_bf16, np.uint16)
    a = _c(acc_bf16, np.uint16)
    assert x.shape == a.shape
    out = np.empty(x.shape, np.float32)
    lib().xqo_cl_delta_rows(_p(x), _p(a), C.c_int64(x.size), _p(out))
    return out


def cl_accumulate_rows(acc_bf16, codes, scale, zero, G, init):
    """In place on acc_bf16 (uint16, C-contiguous)."""
    assert acc_bf16.dtype == np.uint16 and acc_bf16.flags.c_contiguous
    codes = _c(codes, np.uint8)
    scale = _c(scale, np.uint16)
    zero = _c(zero, np.uint16)
    d = codes.shape[-1]
    rows = codes.size // d
    assert acc_bf16.size == codes.size
    lib().xqo_cl_accumulate_rows(_p(acc_bf16), _p(codes), _p(scale), _p(zero), C.c_int64(rows),
                                 C.c_int(d), C.c_int(G), C.c_int(1 if init else 0))
    return acc_bf16


def project_rows(x_bf16, Ut_bf16):
    """Latent down-projection (Sec. 3.3.1): x [M][d] bf16 bits, Ut [n_lat][d] bf16 bits (U transposed)
    -> [M][n_lat] bf16 bits of x U, accumulated in double and rounded once."""
    x = _c(x_bf16, np.uint16)
    ut = _c(Ut_bf16, np.uint16)
    d = x.shape[-1]
    n_lat = ut.shape[0]
    assert ut.shape[1] == d
    M = x.size // d
    out = np.empty((*x.shape[:-1], n_lat), np.uint16)
    lib().xqo_project_rows(_p(x), _p(ut), C.c_int64(M), C.c_int(d), C.c_int(n_lat), _p(out))
    return out


def project_delta_rows(x_bf16, acc_bf16, Ut_bf16):
    """Latent cross-layer delta (Sec. 3.3.2): (x - acc) U_kv for rows x, acc [M][d] bf16 bits and
    Ut = U_kv transposed [n_lat][d] bf16 bits -> [M][n_lat] bf16 bits."""
    x = _c(x_bf16, np.uint16)
    a = _c(acc_bf16, np.uint16)
    ut = _c(Ut_bf16, np.uint16)
    assert x.shape == a.shape
    d = x.shape[-1]
    n_lat = ut.shape[0]
    assert ut.shape[1] == d
    M = x.size // d
    out = np.empty((*x.shape[:-1], n_lat), np.uint16)
    lib().xqo_project_delta_rows(_p(x), _p(a), _p(ut), C.c_int64(M), C.c_int(d), C.c_int(n_lat), _p(out))
    return out


def cl_accumulate_latent_rows(acc_bf16, codes, scale, zero, Ut_bf16, G):
    """Sec. 3.3.2, in place on acc_bf16 [rows][d] (uint16, C-contiguous):
    acc += dequant(codes [rows][n_lat]) @ Ut, Ut = U_kv transposed [n_lat][d]."""
    assert acc_bf16.dtype == np.uint16 and acc_bf16.flags.c_contiguous
    codes = _c(codes, np.uint8)
    scale = _c(scale, np.uint16)
    zero = _c(zero, np.uint16)
    ut = _c(Ut_bf16, np.uint16)
    n_lat, d = ut.shape
    assert codes.shape[-1] == n_lat and acc_bf16.shape[-1] == d
    rows = codes.size // n_lat
    assert acc_bf16.size == rows * d
    lib().xqo_cl_accumulate_latent_rows(_p(acc_bf16), _p(codes), _p(scale), _p(zero), _p(ut),
                                        C.c_int64(rows), C.c_int(d), C.c_int(n_lat), C.c_int(G))
    return acc_bf16


def remat_head(xhat_f32, W_bf16, col0, hd):
    x = _c(xhat_f32, np.float32)
    W = _c(W_bf16, np.uint16)
    L, d = x.shape
    assert W.shape[0] == d
    out = np.empty((L, hd), np.float64)
    lib().xqo_remat_head(_p(x), _p(W), C.c_int(L), C.c_int(d), C.c_int(W.shape[1]),
                         C.c_int(col0), C.c_int(hd), _p(out))
    return out


def attention(q_bf16, K, V, softmax_scale):
    q = _c(q_bf16, np.uint16)
    K = _c(K, np.float64)
    V = _c(V, np.float64)
    L, hd = K.shape
    out = np.empty(hd, np.float32)
    lib().xqo_attention(_p(q), _p(K), _p(V), C.c_int(L), C.c_int(hd),
                        C.c_double(softmax_scale), _p(out))
    return out


def remat_attn_pairs(*, q_bf16, Wk, Wv, Hq, Hkv, hd, softmax_scale, lens, pairs,
                     packed=None, scale=None, zero=None, G=0, bits=0, acc_bf16=None,
                     rope_cos_sin=None, pos0=None):
    """Attention output [npairs][hd] fp32 for the listed (b, q-head) pairs.

    Either (packed, scale, zero, G, bits) -- the X cache, layouts [B][cap][...] --
    or acc_bf16 [B][cap][d] -- the cross-layer accumulator.
    rope_cos_sin (fp32 [n_pos][hd/2][2]) rotates the keys; pos0[b] = position of cache row 0.
    """
    q = _c(q_bf16, np.uint16)
    Wk = _c(Wk, np.uint16)
    Wv = _c(Wv, np.uint16)
    d = Wk.shape[0]
    lens = _c(np.asarray(lens, np.int32), np.int32)
    pb = _c(np.asarray([p[0] for p in pairs], np.int32), np.int32)
    ph = _c(np.asarray([p[1] for p in pairs], np.int32), np.int32)
    if packed is not None:
        packed = _c(packed, np.uint8)
        scale = _c(scale, np.uint16)
        zero = _c(zero, np.uint16)
        cap = packed.shape[1]
        assert acc_bf16 is None
    else:
        acc_bf16 = _c(acc_bf16, np.uint16)
        cap = acc_bf16.shape[1]
        G, bits = d, 16
    out = np.empty((len(pairs), hd), np.float32)
    args = [_p(packed), _p(scale), _p(zero), _p(acc_bf16), C.c_int(cap),
            C.c_int(d), C.c_int(G), C.c_int(bits), _p(q), _p(Wk), _p(Wv),
            C.c_int(Hq), C.c_int(Hkv), C.c_int(hd),
            C.c_double(softmax_scale), _p(lens), _p(pb), _p(ph), C.c_int(len(pairs))]
    if rope_cos_sin is None:
        lib().xqo_remat_attn_pairs(*args, _p(out))
    else:
        tab = _c(rope_cos_sin, np.float32)
        assert tab.ndim == 3 and tab.shape[1] == hd // 2 and tab.shape[2] == 2
        p0 = _c(np.zeros(len(lens), np.int32) if pos0 is None else np.asarray(pos0, np.int32), np.int32)
        assert int((p0.astype(np.int64) + lens).max()) <= tab.shape[0]
        lib().xqo_remat_attn_pairs_rope(*args, _p(tab), _p(p0), _p(out))
    return out


def remat_attn_pairs_per_channel(*, q_bf16, Wk, Wv, Hq, Hkv, hd, softmax_scale, lens, pairs,
                                 packed, scale, zero, G, bits, tail_bf16):
    """Decode attention from a per-channel cache with a residual window (Sec. 3.3.1): of the lens[b]
    tokens of sequence b the first floor(lens[b]/G)*G are read from the cache (packed [B][cap][d*bits/8],
    scale / zero [B][cap/G][d]) and the remaining lens[b] % G from rows 0.. of tail_bf16 [B][G][d], which
    holds them unquantised.  Composition of pinned pieces only: unpack, per-channel dequantise,
    xqo_remat_head, xqo_attention.  Returns [npairs][hd] fp32."""
    q = _c(q_bf16, np.uint16)
    packed = _c(packed, np.uint8)
    tail = _c(tail_bf16, np.uint16)
    d = Wk.shape[0]
    g = Hq // Hkv
    out = np.empty((len(pairs), hd), np.float32)
    xhat_cache = {}
    for i, (b, hq) in enumerate(pairs):
        if b not in xhat_cache:
            n = int(lens[b])
            nblk, rem = n // G, n % G
            coded = np.empty((0, d), np.float32)
            if nblk:
                codes = unpack_rows(packed[b, :nblk * G], d, bits)
                coded = dequantize_blocks_per_channel(codes, scale[b, :nblk], zero[b, :nblk], G)
            xhat_cache[b] = np.concatenate([coded, bf16_to_f32(tail[b, :rem])], axis=0)
        xhat = xhat_cache[b]
        hk = hq // g
        K = remat_head(xhat, Wk, hk * hd, hd)
        V = remat_head(xhat, Wv, hk * hd, hd)
        out[i] = attention(q[b, hq], K, V, softmax_scale)
    return out


def latent_attn_pairs_per_channel(*, q_bf16, Wfk, Wfv, Hq, Hkv, hd, softmax_scale, lens, pairs,
                                  k_packed, k_scale, k_zero, k_G, k_bits, k_tail_bf16,
                                  v_packed, v_scale, v_zero, v_G, v_bits, k0_f16=None):
    """Sec. 3.3.1's setting for grouped-query models: keys from a per-channel cache of X Uk (complete blocks
    of k_G tokens, the rest in the bf16 window k_tail) through Wfk = Sk Bk^T, values from a per-token cache
    of X Uv through Wfv = Sv Bv^T.  Composition of pinned pieces only.  Returns [npairs][hd] fp32.

    k0_f16 (App. B): [B][>= lens[b]] IEEE half bit patterns.  If given, the first channel of X Uk, the one that
    collects the outliers, is kept in fp16 instead of being quantised: channel 0 of every latent key row
    (cache blocks and window alike) is k0_f16[b][t]; whatever the cache and the window hold there is unused."""
    q = _c(q_bf16, np.uint16)
    r = Wfk.shape[0]
    g = Hq // Hkv
    out = np.empty((len(pairs), hd), np.float32)
    cache = {}
    for i, (b, hq) in enumerate(pairs):
        if b not in cache:
            n = int(lens[b])
            nblk, rem = n // k_G, n % k_G
            coded = np.empty((0, r), np.float32)
            if nblk:
                coded = dequantize_blocks_per_channel(unpack_rows(_c(k_packed, np.uint8)[b, :nblk * k_G], r, k_bits),
                                                      k_scale[b, :nblk], k_zero[b, :nblk], k_G)
            xk = np.concatenate([coded, bf16_to_f32(_c(k_tail_bf16, np.uint16)[b, :rem])], axis=0)
            if k0_f16 is not None:
                xk[:, 0] = _c(k0_f16, np.uint16)[b, :n].view(np.float16).astype(np.float32)
            xv = dequantize_rows(unpack_rows(_c(v_packed, np.uint8)[b, :n], r, v_bits), v_scale[b, :n], v_zero[b, :n], v_G)
            cache[b] = (xk, xv)
        xk, xv = cache[b]
        hk = hq // g
        K = remat_head(xk, Wfk, hk * hd, hd)
        V = remat_head(xv, Wfv, hk * hd, hd)
        out[i] = attention(q[b, hq], K, V, softmax_scale)
    return out


def prefill_attn_triples(*, q_bf16, lens, triples, **kw):
    """Causal attention of the T newest tokens of every sequence (chunked prefill; T = 1 is the
    decode step): q_bf16 [B][T][Hq][hd]; query t of sequence b sits at cache row lens[b] - T + t
    and attends rows 0 .. that row.  By definition this is the decode attention of that query
    over the prefix that ends at its own row, so each listed (b, t, q-head) triple is one call
    of remat_attn_pairs with the prefix length -- nothing else is computed here.
    Returns [ntriples][hd] fp32 in the order of `triples`; other arguments as remat_attn_pairs."""
    q = _c(q_bf16, np.uint16)
    B, T = q.shape[0], q.shape[1]
    lens = np.asarray(lens, np.int64)
    assert lens.shape == (B,) and np.all(lens >= T)
    out = None
    for t in sorted({tr[1] for tr in triples}):
        idx = [i for i, tr in enumerate(triples) if tr[1] == t]
        res = remat_attn_pairs(q_bf16=np.ascontiguousarray(q[:, t]), lens=(lens - T + t + 1).astype(np.int32),
                               pairs=[(triples[i][0], triples[i][2]) for i in idx], **kw)
        if out is None:
            out = np.empty((len(triples), res.shape[1]), np.float32)
        out[idx] = res
    return out


def rope_rows(K, cos_sin, pos0=0):
    """Rotate key rows K [L][hd] (float64, in place on a copy) by the table; returns the copy."""
    K = np.array(K, np.float64, order="C")
    tab = _c(cos_sin, np.float32)
    L, hd = K.shape
    assert tab.shape[1] == hd // 2 and pos0 + L <= tab.shape[0]
    lib().xqo_rope_rows(_p(K), C.c_int(L), C.c_int(hd), _p(tab), C.c_int(pos0))
    return K
