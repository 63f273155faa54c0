"""Pins for the oracle's rotary position embedding of rematerialised keys (half-split pairing,
RoFormer as cited in Sec. 2 of arxiv 2508.10395; K = X Wk is the key before the rotation)."""
import numpy as np

import xq_inputs as xi
from oracle import xq_oracle as xo


def bits(x):
    return xi.to_bf16_bits(np.asarray(x, np.float32))


def bf(x):
    return xi.from_bf16_bits(x)


def table(n_pos, hd, base=10000.0):
    """cos/sin of pos * base^(-2i/hd), the textbook frequencies, [n_pos][hd/2][2] fp32."""
    inv = base ** (-np.arange(hd // 2, dtype=np.float64) * 2.0 / hd)
    ang = np.arange(n_pos, dtype=np.float64)[:, None] * inv[None, :]
    return np.stack([np.cos(ang), np.sin(ang)], axis=-1).astype(np.float32)


def test_quarter_turn_by_hand():
    """cos = 0, sin = 1 everywhere: k'[i] = -k[i+hd/2], k'[i+hd/2] = k[i]."""
    hd = 8
    k = np.arange(1.0, 9.0)[None, :]
    tab = np.zeros((1, hd // 2, 2), np.float32)
    tab[..., 1] = 1.0
    assert np.array_equal(xo.rope_rows(k, tab)[0], [-5, -6, -7, -8, 1, 2, 3, 4])


def test_zero_angle_is_identity_and_norms_are_kept():
    rng = np.random.default_rng(0)
    k = rng.standard_normal((9, 128))
    ident = np.zeros((9, 64, 2), np.float32)
    ident[..., 0] = 1.0
    assert np.array_equal(xo.rope_rows(k, ident), k)
    tab = table(64, 128)
    r = xo.rope_rows(k, tab, pos0=17)
    # each (i, i+64) pair is rotated in its own plane: pair norms are unchanged
    assert np.allclose(r[:, :64] ** 2 + r[:, 64:] ** 2, k[:, :64] ** 2 + k[:, 64:] ** 2, rtol=1e-6)
    # against complex multiplication, the textbook form of the same rotation
    z = (k[:, :64] + 1j * k[:, 64:]) * (tab[17:26, :, 0].astype(np.float64) + 1j * tab[17:26, :, 1].astype(np.float64))
    assert np.allclose(r[:, :64], z.real, atol=1e-12) and np.allclose(r[:, 64:], z.imag, atol=1e-12)


def test_scores_depend_on_relative_position_only():
    """<R(p) q, R(t) k> = <R(p + s) q, R(t + s) k>: shifting every position by s changes nothing."""
    rng = np.random.default_rng(1)
    hd, L = 128, 6
    tab = table(64, hd).astype(np.float64).astype(np.float32)
    q = rng.standard_normal((1, hd))
    k = rng.standard_normal((L, hd))
    s0 = xo.rope_rows(k, tab, pos0=0) @ xo.rope_rows(q, tab, pos0=10)[0]
    s1 = xo.rope_rows(k, tab, pos0=23) @ xo.rope_rows(q, tab, pos0=33)[0]
    assert np.allclose(s0, s1, rtol=0, atol=2e-5 * np.abs(s0).max())      # table entries are fp32


def test_attention_with_rope_against_brute_force():
    """xqo_remat_attn_pairs with a table == numpy: X W, rotate rows, softmax, weighted sum (GQA, 2 seqs)."""
    w = xi.C4.scaled(B=2, L=37, d=256, Hq=4, Hkv=2, n_outlier=0)
    x, (wk, wv), q = xi.gen_x(w), xi.gen_weights(w), xi.gen_q(w)
    tab = table(64, w.hd)
    lens, pos0 = [37, 20], [5, 0]
    pairs = [(b, h) for b in range(2) for h in range(4)]
    got = xo.remat_attn_pairs(q_bf16=q, Wk=wk, Wv=wv, Hq=4, Hkv=2, hd=w.hd, softmax_scale=w.hd ** -0.5,
                              lens=lens, pairs=pairs, acc_bf16=x, rope_cos_sin=tab, pos0=pos0)
    X, WK, WV, Q = (bf(a).astype(np.float64) for a in (x, wk, wv, q))
    for i, (b, h) in enumerate(pairs):
        hk, L = h // 2, lens[b]
        K = X[b, :L] @ WK[:, hk * 128:(hk + 1) * 128]
        V = X[b, :L] @ WV[:, hk * 128:(hk + 1) * 128]
        cs = tab[pos0[b]:pos0[b] + L].astype(np.float64)
        Kr = np.concatenate([K[:, :64] * cs[..., 0] - K[:, 64:] * cs[..., 1],
                             K[:, 64:] * cs[..., 0] + K[:, :64] * cs[..., 1]], axis=1)
        s = Kr @ Q[b, h] * w.hd ** -0.5
        p = np.exp(s - s.max())
        ref = (p / p.sum()) @ V
        assert np.allclose(got[i], ref, rtol=1e-5, atol=1e-6)
    # and the table matters: without it the output differs
    plain = xo.remat_attn_pairs(q_bf16=q, Wk=wk, Wv=wv, Hq=4, Hkv=2, hd=w.hd, softmax_scale=w.hd ** -0.5,
                                lens=lens, pairs=pairs, acc_bf16=x)
    assert not np.allclose(plain, got, rtol=1e-3)
