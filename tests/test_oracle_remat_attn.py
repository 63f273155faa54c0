"""CPU pins for the oracle's cross-layer accumulator, rematerialisation and
attention (no GPU): identities from Sec. 3.2, numpy/scipy library routines and
closed forms."""
import numpy as np
import pytest
import torch
from scipy.special import logsumexp, softmax

import xq_inputs as xi
from oracle import xq_oracle as xo


def bf(x):
    return xi.from_bf16_bits(x)


def tb(x_f32):
    """torch's own fp32 -> bf16 cast, as bits (library routine, independent of the oracle)."""
    return torch.from_numpy(np.ascontiguousarray(x_f32, np.float32)).to(torch.bfloat16) \
        .view(torch.int16).numpy().view(np.uint16)


# ------------------------------------------------------------- cross-layer


def _cl_stack(w, layers, base_bits=4, delta_bits=2, G=128):
    """Run the decode-side cross-layer recurrence with the oracle; return the
    true inputs X_i, the accumulators acc_i and the per-layer delta scales."""
    xs = [xi.gen_x(w)]
    for l in range(1, layers):
        xs.append(xi.gen_next_layer_x(w, xs[-1], l))
    c, s, z = xo.quantize_rows(bf(xs[0]), G, base_bits)
    acc = np.zeros_like(xs[0])
    xo.cl_accumulate_rows(acc, c, s, z, G, init=True)
    accs, scales = [acc.copy()], [s]
    for l in range(1, layers):
        delta = xo.cl_delta_rows(xs[l], acc)
        c, s, z = xo.quantize_rows(delta, G, delta_bits)
        xo.cl_accumulate_rows(acc, c, s, z, G, init=False)
        accs.append(acc.copy())
        scales.append(s)
    return xs, accs, scales


def test_cl_exact_grid_deltas_telescope_to_the_true_input():
    """If every delta lies exactly on its quantisation grid, Q is the identity on
    it and X^_i = X_0 + sum of deltas reproduces X_i bit for bit (Sec. 3.2)."""
    rng = np.random.default_rng(0)
    d, G, L, layers = 256, 128, 6, 5
    x0 = (rng.integers(-8, 8, (1, L, d)) * 0.25).astype(np.float32)   # 4-bit grid, step .25
    x0[..., 0::G], x0[..., 1::G] = -2.0, 1.75
    xs = [x0]
    for _ in range(1, layers):
        step = (rng.integers(0, 4, (1, L, d)) * 0.125 - 0.25).astype(np.float32)   # 2-bit grid
        step[..., 0::G], step[..., 1::G] = -0.25, 0.125
        xs.append(xs[-1] + step)
    xs = [xi.to_bf16_bits(x) for x in xs]
    for x in xs:
        assert np.array_equal(bf(x), bf(x).astype(np.float32))
    c, s, z = xo.quantize_rows(bf(xs[0]), G, 4)
    acc = np.zeros_like(xs[0])
    xo.cl_accumulate_rows(acc, c, s, z, G, init=True)
    assert np.array_equal(acc, xs[0])
    for l in range(1, layers):
        c, s, z = xo.quantize_rows(xo.cl_delta_rows(xs[l], acc), G, 2)
        xo.cl_accumulate_rows(acc, c, s, z, G, init=False)
        assert np.array_equal(acc, xs[l]), l


def test_cl_error_does_not_grow_with_depth():
    """Because each delta is taken against the running approximation, the error
    after layer i is one quantisation step of layer i only: |X_i - X^_i| <=
    scale_i/2 + zero-point rounding + accumulator rounding, at every depth."""
    w = xi.C3.scaled(B=1, L=8)
    xs, accs, scales = _cl_stack(w, layers=12)
    worst = []
    for l in range(1, 12):
        x, a = bf(xs[l]), bf(accs[l])
        sf = np.repeat(bf(scales[l]), 128, -1)
        # zero is bf16(min delta): |delta| <~ 2.5, so its rounding is <= 2^-8 * 2.5 ; acc RNE <= 2^-8 |acc|
        bound = sf / 2 + 2.0 ** -8 * 2.5 + 2.0 ** -8 * np.abs(a) + 1e-6
        assert np.all(np.abs(x - a) <= bound), l
        worst.append(float(np.abs(x - a).max()))
    assert max(worst[6:]) < 2.0 * max(worst[:3])          # flat, not accumulating


def test_cl_accumulator_is_the_sequentially_rounded_sum():
    """acc_i = bf16(acc_{i-1} + (code*scale+zero)) with fp32 arithmetic: rebuilt
    here with numpy float64 products rounded once to fp32 and torch's bf16 cast."""
    w = xi.C3.scaled(B=1, L=4)
    xs = [xi.gen_x(w), None]
    xs[1] = xi.gen_next_layer_x(w, xs[0], 1)
    c0, s0, z0 = xo.quantize_rows(bf(xs[0]), 128, 4)
    acc = np.zeros_like(xs[0])
    xo.cl_accumulate_rows(acc, c0, s0, z0, 128, init=True)

    def deq(c, s, z):
        return (c.astype(np.float64) * np.repeat(bf(s).astype(np.float64), 128, -1)
                + np.repeat(bf(z).astype(np.float64), 128, -1)).astype(np.float32)

    assert np.array_equal(acc, tb(deq(c0, s0, z0)))
    delta = xo.cl_delta_rows(xs[1], acc)
    assert np.array_equal(delta, bf(xs[1]) - bf(acc))
    c1, s1, z1 = xo.quantize_rows(delta, 128, 2)
    acc1 = acc.copy()
    xo.cl_accumulate_rows(acc1, c1, s1, z1, 128, init=False)
    assert np.array_equal(acc1, tb(bf(acc) + deq(c1, s1, z1)))


# ------------------------------------------------------------ rematerialise


def test_identity_quantiser_remat_is_plain_matmul():
    """With Q = identity the rematerialised K, V are X Wk, X Wv: the oracle's loop
    against numpy's float64 matmul."""
    w = xi.C1.scaled(L=37)
    x = bf(xi.gen_x(w))[0]
    wk, wv = xi.gen_weights(w)
    for W in (wk, wv):
        ref = x.astype(np.float64) @ bf(W).astype(np.float64)
        for h in range(w.Hkv):
            got = xo.remat_head(x, W, h * w.hd, w.hd)
            assert np.allclose(got, ref[:, h * w.hd:(h + 1) * w.hd], rtol=1e-12, atol=1e-12)


def test_remat_of_a_unit_row_reads_one_weight_row():
    d, hd = 64, 16
    W = xi.to_bf16_bits(np.arange(d * 48, dtype=np.float32).reshape(d, 48) / 8)
    x = np.zeros((3, d), np.float32)
    x[0, 5], x[1, 63], x[2, 0] = 1.0, 2.0, -1.0
    got = xo.remat_head(x, W, 32, hd)
    Wf = bf(W).astype(np.float64)
    assert np.array_equal(got[0], Wf[5, 32:48])
    assert np.array_equal(got[1], 2 * Wf[63, 32:48])
    assert np.array_equal(got[2], -Wf[0, 32:48])


# ---------------------------------------------------------------- attention


def _rand_kv(L, hd, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((L, hd)), rng.standard_normal((L, hd)),
            xi.to_bf16_bits(rng.standard_normal(hd).astype(np.float32)))


def test_attention_uniform_scores_give_the_mean_value():
    K, V, q = _rand_kv(50, 128, 0)
    out = xo.attention(q, np.zeros_like(K), V, 0.3)
    assert np.allclose(out, V.mean(0), rtol=1e-6, atol=1e-7)


def test_attention_two_tokens_is_a_logistic_mix():
    hd = 128
    _, V, q = _rand_kv(2, hd, 1)
    qf = bf(q).astype(np.float64)
    K = np.zeros((2, hd))
    K[0] = qf / (qf @ qf) * 1.7          # score gap of exactly 1.7 * scale
    scale = 0.5
    p0 = 1.0 / (1.0 + np.exp(-1.7 * scale))
    out = xo.attention(q, K, V, scale)
    assert np.allclose(out, p0 * V[0] + (1 - p0) * V[1], rtol=1e-6, atol=1e-7)


def test_attention_matches_scipy_softmax_and_is_shift_permutation_split_invariant():
    L, hd = 300, 128
    K, V, q = _rand_kv(L, hd, 2)
    K *= 3.0
    scale = hd ** -0.5
    qf = bf(q).astype(np.float64)
    s = (K @ qf) * scale
    ref = softmax(s) @ V
    out = xo.attention(q, K, V, scale)
    assert np.allclose(out, ref, rtol=2e-7, atol=1e-7)
    # adding the same multiple of q to every key shifts all scores equally
    out_shift = xo.attention(q, K + 40.0 * qf / np.linalg.norm(qf), V, scale)
    assert np.allclose(out_shift, out, rtol=1e-5, atol=1e-6)
    # no positional term: permuting the cached rows changes nothing
    perm = np.random.default_rng(9).permutation(L)
    assert np.allclose(xo.attention(q, K[perm], V[perm], scale), out, rtol=1e-6, atol=1e-7)
    # split the context, merge the two partial results by their log-sum-exp weights
    a, b = slice(0, 77), slice(77, L)
    oa, ob = xo.attention(q, K[a], V[a], scale), xo.attention(q, K[b], V[b], scale)
    la, lb = logsumexp(s[a]), logsumexp(s[b])
    wa = 1.0 / (1.0 + np.exp(lb - la))
    assert np.allclose(wa * oa + (1 - wa) * ob, out, rtol=1e-5, atol=1e-6)


def test_attention_large_scores_do_not_overflow():
    K, V, q = _rand_kv(20, 128, 3)
    out = xo.attention(q, K * 1e4, V, 1.0)
    assert np.all(np.isfinite(out))


# -------------------------------------------------------------- composition


def _brute_force(w, xhat, wk, wv, q, lens, pairs):
    """float64 numpy attention over rematerialised K, V, for a few pairs."""
    out = []
    g = w.Hq // w.Hkv
    for b, hq in pairs:
        hk = hq // g
        X = xhat[b, :lens[b]].astype(np.float64)
        K = X @ bf(wk)[:, hk * w.hd:(hk + 1) * w.hd].astype(np.float64)
        V = X @ bf(wv)[:, hk * w.hd:(hk + 1) * w.hd].astype(np.float64)
        s = K @ bf(q)[b, hq].astype(np.float64) * w.hd ** -0.5
        out.append(softmax(s) @ V)
    return np.array(out)


@pytest.mark.parametrize("w,bits,G", [(xi.C1.scaled(L=96), 4, 128),
                                      (xi.C4.scaled(B=2, L=40, d=512), 2, 64),
                                      (xi.C2.scaled(B=2, L=33, d=384, Hq=4, Hkv=4), 3, 128)])
def test_pairs_composition_equals_brute_force(w, bits, G):
    x = xi.gen_x(w)
    wk, wv = xi.gen_weights(w)
    q = xi.gen_q(w)
    codes, scale, zero = xo.quantize_rows(bf(x), G, bits)
    packed = xo.pack_rows(codes, bits)
    lens = [w.L - 3 * b for b in range(w.B)]
    pairs = [(b, h) for b in range(w.B) for h in range(w.Hq)]
    got = xo.remat_attn_pairs(q_bf16=q, Wk=wk, Wv=wv, Hq=w.Hq, Hkv=w.Hkv, hd=w.hd,
                              softmax_scale=w.hd ** -0.5, lens=lens, pairs=pairs,
                              packed=packed, scale=scale, zero=zero, G=G, bits=bits)
    xhat = xo.dequantize_rows(codes, scale, zero, G)
    ref = _brute_force(w, xhat, wk, wv, q, lens, pairs)
    assert np.allclose(got, ref, rtol=1e-5, atol=1e-6)
    # quantisation is visible: the same attention on the unquantised X differs
    ref_fp = _brute_force(w, bf(x), wk, wv, q, lens, pairs)
    assert not np.allclose(got, ref_fp, rtol=1e-5, atol=1e-6)


def test_pairs_accumulator_source_and_gqa_equals_replicated_mha():
    w = xi.C4.scaled(B=2, L=24, d=256, Hq=4, Hkv=2)
    acc = xi.gen_x(w)
    wk, wv = xi.gen_weights(w)
    q = xi.gen_q(w)
    lens = [24, 17]
    pairs = [(b, h) for b in range(2) for h in range(4)]
    kw = dict(q_bf16=q, Hq=4, hd=w.hd, softmax_scale=w.hd ** -0.5, lens=lens, pairs=pairs, acc_bf16=acc)
    got = xo.remat_attn_pairs(Wk=wk, Wv=wv, Hkv=2, **kw)
    assert np.allclose(got, _brute_force(w, bf(acc), wk, wv, q, lens, pairs), rtol=1e-5, atol=1e-6)
    # GQA == MHA whose KV weights are the GQA ones replicated per query head
    rep = lambda W: np.ascontiguousarray(np.repeat(W.reshape(w.d, 2, w.hd), 2, axis=1).reshape(w.d, 4 * w.hd))
    got_mha = xo.remat_attn_pairs(Wk=rep(wk), Wv=rep(wv), Hkv=4, **kw)
    assert np.array_equal(got, got_mha)
