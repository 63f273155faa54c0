"""Pins for the oracle's causal attention of several new tokens per sequence (chunked prefill;
Sec. 3.1 of arxiv 2508.10395 rematerialises K, V for whatever queries attend to the cache, and
App. A treats T > 1 new tokens): textbook masked attention, and the properties that define
causality."""
import numpy as np
from scipy.special import softmax

import xq_inputs as xi
from oracle import xq_oracle as xo


def bf(x):
    return xi.from_bf16_bits(x)


def bits(x):
    return xi.to_bf16_bits(np.asarray(x, np.float32))


def _setup(seed, B=2, L=37, T=5, d=256, Hq=4, Hkv=2, hd=128):
    rng = np.random.default_rng(seed)
    x = bits(rng.standard_normal((B, L, d)))
    wk = bits(rng.standard_normal((d, Hkv * hd)) * d ** -0.5)
    wv = bits(rng.standard_normal((d, Hkv * hd)) * d ** -0.5)
    q = bits(rng.standard_normal((B, T, Hq, hd)) * 2.0)
    return x, wk, wv, q


def _masked_attention(xhat, wk, wv, q, lens, T, Hq, Hkv, hd):
    """softmax(Q K^T / sqrt(hd) + causal mask) V with the full T x len score matrix, fp64."""
    B = xhat.shape[0]
    g = Hq // Hkv
    out = np.zeros((B, T, Hq, hd))
    for b in range(B):
        n = lens[b]
        X = xhat[b, :n].astype(np.float64)
        for hq in range(Hq):
            hk = hq // g
            K = X @ bf(wk)[:, hk * hd:(hk + 1) * hd].astype(np.float64)
            V = X @ bf(wv)[:, hk * hd:(hk + 1) * hd].astype(np.float64)
            S = bf(q)[b, :, hq].astype(np.float64) @ K.T * hd ** -0.5               # [T][n]
            rows = np.arange(n)[None, :]
            pos = (n - T + np.arange(T))[:, None]
            S = np.where(rows <= pos, S, -np.inf)
            out[b, :, hq] = softmax(S, axis=1) @ V
    return out


def test_prefill_equals_textbook_masked_attention():
    B, L, T, d, Hq, Hkv, hd = 2, 37, 5, 256, 4, 2, 128
    x, wk, wv, q = _setup(1, B, L, T, d, Hq, Hkv, hd)
    lens = [37, 11]
    triples = [(b, t, h) for b in range(B) for t in range(T) for h in range(Hq)]
    got = xo.prefill_attn_triples(q_bf16=q, lens=lens, triples=triples, Wk=wk, Wv=wv, Hq=Hq, Hkv=Hkv, hd=hd,
                                  softmax_scale=hd ** -0.5, acc_bf16=x)
    ref = _masked_attention(bf(x), wk, wv, q, lens, T, Hq, Hkv, hd)
    ref = np.array([ref[b, t, h] for b, t, h in triples])
    assert np.allclose(got, ref, rtol=1e-5, atol=1e-6)


def test_prefill_from_a_quantised_cache_and_order_of_triples():
    B, L, T, d, Hq, Hkv, hd = 2, 40, 3, 256, 2, 2, 128
    x, wk, wv, q = _setup(2, B, L, T, d, Hq, Hkv, hd)
    codes, scale, zero = xo.quantize_rows(bf(x), 64, 3)
    kw = dict(q_bf16=q, lens=[40, 9], Wk=wk, Wv=wv, Hq=Hq, Hkv=Hkv, hd=hd, softmax_scale=hd ** -0.5,
              packed=xo.pack_rows(codes, 3), scale=scale, zero=zero, G=64, bits=3)
    triples = [(1, 2, 0), (0, 0, 1), (1, 0, 1), (0, 2, 0)]                     # scrambled on purpose
    got = xo.prefill_attn_triples(triples=triples, **kw)
    ref = _masked_attention(xo.dequantize_rows(codes, scale, zero, 64), wk, wv, q, [40, 9], T, Hq, Hkv, hd)
    assert np.allclose(got, np.array([ref[b, t, h] for b, t, h in triples]), rtol=1e-5, atol=1e-6)


def test_one_new_token_is_the_decode_step_and_the_last_query_sees_everything():
    B, L, T, d, Hq, Hkv, hd = 2, 30, 4, 256, 2, 1, 128
    x, wk, wv, q = _setup(3, B, L, T, d, Hq, Hkv, hd)
    lens = [30, 22]
    kw = dict(Wk=wk, Wv=wv, Hq=Hq, Hkv=Hkv, hd=hd, softmax_scale=hd ** -0.5, acc_bf16=x)
    pairs = [(b, h) for b in range(B) for h in range(Hq)]
    dec = xo.remat_attn_pairs(q_bf16=np.ascontiguousarray(q[:, T - 1]), lens=lens, pairs=pairs, **kw)
    last = xo.prefill_attn_triples(q_bf16=q, lens=lens, triples=[(b, T - 1, h) for b, h in pairs], **kw)
    assert np.array_equal(dec, last)
    one = xo.prefill_attn_triples(q_bf16=np.ascontiguousarray(q[:, T - 1:]), lens=lens,
                                  triples=[(b, 0, h) for b, h in pairs], **kw)
    assert np.array_equal(dec, one)


def test_causality_later_rows_do_not_reach_earlier_queries():
    B, L, T, d, Hq, Hkv, hd = 1, 20, 4, 256, 2, 2, 128
    x, wk, wv, q = _setup(4, B, L, T, d, Hq, Hkv, hd)
    kw = dict(q_bf16=q, lens=[20], Wk=wk, Wv=wv, Hq=Hq, Hkv=Hkv, hd=hd, softmax_scale=hd ** -0.5)
    triples = [(0, t, h) for t in range(T) for h in range(Hq)]
    a = xo.prefill_attn_triples(triples=triples, acc_bf16=x, **kw)
    x2 = x.copy()
    x2[0, 18:] = bits(np.random.default_rng(9).standard_normal((2, d)))          # rows of queries 2 and 3
    b = xo.prefill_attn_triples(triples=triples, acc_bf16=x2, **kw)
    a, b = a.reshape(T, Hq, hd), b.reshape(T, Hq, hd)
    assert np.array_equal(a[:2], b[:2])                   # queries at rows 16, 17 cannot see rows 18, 19
    assert not np.allclose(a[2:], b[2:])
    # a query whose prefix is one row returns that row's value exactly
    first = xo.prefill_attn_triples(q_bf16=q[:, :1], lens=[1], triples=[(0, 0, 0)], Wk=wk, Wv=wv, Hq=Hq, Hkv=Hkv,
                                    hd=hd, softmax_scale=hd ** -0.5, acc_bf16=x)
    v0 = bf(x)[0, 0].astype(np.float64) @ bf(wv)[:, :hd].astype(np.float64)
    assert np.allclose(first[0], v0, rtol=1e-6, atol=1e-7)
