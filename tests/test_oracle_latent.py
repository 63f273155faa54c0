"""Pins for the oracle's latent (grouped-query) path, Sec. 3.3.1 of arxiv 2508.10395:
the down-projection X U and the fact that rematerialising from the latent cache with the
fused matrices S B^T gives back plain X W."""
import numpy as np
import pytest

import xq_inputs as xi
from oracle import xq_oracle as xo


def bf(x):
    return xi.from_bf16_bits(x)


def bits(x):
    return xi.to_bf16_bits(np.asarray(x, np.float32))


def _bf16_ulp(v):
    """Spacing of bf16 numbers around |v| (v != 0)."""
    e = np.floor(np.log2(np.abs(v)))
    return 2.0 ** (e - 7)


def test_projection_is_the_nearest_bf16_of_the_fp64_product():
    rng = np.random.default_rng(11)
    x = bits(rng.standard_normal((7, 384)))
    ut = bits(rng.standard_normal((96, 384)) * 0.05)
    got = bf(xo.project_rows(x, ut)).astype(np.float64)
    ref = bf(x).astype(np.float64) @ bf(ut).astype(np.float64).T          # library routine, fp64
    assert np.all(np.abs(got - ref) <= 0.5 * _bf16_ulp(ref) * (1 + 1e-9))


def test_projection_exact_when_everything_is_representable():
    """Small integers times +-1/16: every product and every sum is exact, so the result is fixed
    to the bit by the mathematics."""
    rng = np.random.default_rng(5)
    x = rng.integers(-1, 2, size=(9, 256)).astype(np.float32)
    u = (rng.integers(0, 2, size=(256, 64)) * 2 - 1).astype(np.float32) / 16.0
    ref = x.astype(np.float64) @ u.astype(np.float64)                     # integers / 16, |.| <= 16
    got = bf(xo.project_rows(bits(x), bits(u.T)))
    assert np.array_equal(got.astype(np.float64), ref)


def test_projection_identity_and_operand_order():
    rng = np.random.default_rng(6)
    x = bits(rng.standard_normal((4, 128)))
    eye = bits(np.eye(128))
    assert np.array_equal(xo.project_rows(x, eye), x)                     # U = I
    u = rng.standard_normal((128, 128)).astype(np.float32)
    a = xo.project_rows(x, bits(u.T))                                     # x U
    b = xo.project_rows(x, bits(u))                                       # x U^T: a different matrix
    assert not np.array_equal(a, b)
    ref = bf(x).astype(np.float64) @ bf(bits(u)).astype(np.float64)
    assert np.allclose(bf(a), ref, rtol=2 ** -8, atol=1e-6)


def _hadamard(n):
    h = np.array([[1.0]])
    while h.shape[0] < n:
        h = np.block([[h, h], [h, -h]])
    return h


def _exact_factors(d, r, ncols, seed):
    """U (d x r, orthonormal columns), S (r), Bt (r x ncols) whose entries, and those of
    W = U S Bt, are powers of two times +-1: exactly representable in bf16."""
    rng = np.random.default_rng(seed)
    assert int(round(np.sqrt(d))) ** 2 == d and (d & (d - 1)) == 0          # d = 4^k: 1/sqrt(d) is a power of two
    u = _hadamard(d)[:, rng.permutation(d)[:r]] / np.sqrt(d)
    s = 2.0 ** rng.integers(-2, 3, size=r)
    perm = rng.permutation(ncols)[:r]
    bt = np.zeros((r, ncols))
    bt[np.arange(r), perm] = rng.integers(0, 2, size=r) * 2 - 1           # signed partial permutation
    return u, s, bt


def test_latent_remat_equals_plain_remat_when_nothing_rounds():
    """Wk = Uk Sk Bk^T, Wv = Uv Sv Bv^T with exactly representable factors and small-integer X:
    K, V rematerialised from the latent rows [X Uk | X Uv] with the block-diagonal fused weights
    must equal X Wk, X Wv (the derivation of Sec. 3.3.1 with the identity quantiser)."""
    d, r, hd, L = 256, 128, 128, 12
    uk, sk, btk = _exact_factors(d, r, hd, 1)
    uv, sv, btv = _exact_factors(d, r, hd, 2)
    wk, wv = uk @ np.diag(sk) @ btk, uv @ np.diag(sv) @ btv
    assert np.array_equal(bf(bits(wk)).astype(np.float64), wk)            # representable, as claimed
    rng = np.random.default_rng(3)
    x = rng.integers(-1, 2, size=(L, d)).astype(np.float32)
    ut = bits(np.concatenate([uk, uv], axis=1).T)                         # [2r][d]
    lat = xo.project_rows(bits(x), ut)                                    # [L][2r], exact
    assert np.array_equal(bf(lat).astype(np.float64), x.astype(np.float64) @ np.concatenate([uk, uv], axis=1))
    wfk, wfv = np.diag(sk) @ btk, np.diag(sv) @ btv                        # fused r x hd
    wk_cat = bits(np.concatenate([wfk, np.zeros_like(wfv)], axis=0))      # [[Sk Bk^T], [0]]
    wv_cat = bits(np.concatenate([np.zeros_like(wfk), wfv], axis=0))      # [[0], [Sv Bv^T]]
    k_lat = xo.remat_head(bf(lat), wk_cat, 0, hd)
    v_lat = xo.remat_head(bf(lat), wv_cat, 0, hd)
    k_ref = xo.remat_head(x, bits(wk), 0, hd)
    v_ref = xo.remat_head(x, bits(wv), 0, hd)
    assert np.array_equal(k_lat, k_ref) and np.array_equal(v_lat, v_ref)
    assert np.array_equal(k_ref, x.astype(np.float64) @ wk)


def test_latent_attention_equals_plain_attention_same_setting():
    d, r, hd, L = 256, 128, 128, 20
    uk, sk, btk = _exact_factors(d, r, hd, 7)
    uv, sv, btv = _exact_factors(d, r, hd, 8)
    wk, wv = uk @ np.diag(sk) @ btk, uv @ np.diag(sv) @ btv
    rng = np.random.default_rng(9)
    x = rng.integers(-1, 2, size=(1, L, d)).astype(np.float32)
    q = bits(rng.standard_normal((1, 1, hd)))
    lat = xo.project_rows(bits(x), bits(np.concatenate([uk, uv], axis=1).T))
    wfk, wfv = np.diag(sk) @ btk, np.diag(sv) @ btv
    wk_cat = bits(np.concatenate([wfk, np.zeros_like(wfv)], axis=0))
    wv_cat = bits(np.concatenate([np.zeros_like(wfk), wfv], axis=0))
    common = dict(q_bf16=q, Hq=1, Hkv=1, hd=hd, softmax_scale=hd ** -0.5, lens=[L], pairs=[(0, 0)])
    o_lat = xo.remat_attn_pairs(Wk=wk_cat, Wv=wv_cat, acc_bf16=lat, **common)
    o_ref = xo.remat_attn_pairs(Wk=bits(wk), Wv=bits(wv), acc_bf16=bits(x), **common)
    assert np.array_equal(o_lat, o_ref)


def test_svd_factors_close_the_loop():
    """numpy's SVD, as the offline step would use it: U S B^T reproduces W, U has orthonormal
    columns, and with float64 factors latent remat equals X W to rounding."""
    rng = np.random.default_rng(4)
    d, r = 192, 64
    w = rng.standard_normal((d, r)) / np.sqrt(d)
    u, s, bt = np.linalg.svd(w, full_matrices=False)
    assert np.allclose(u @ np.diag(s) @ bt, w, atol=1e-12)
    assert np.allclose(u.T @ u, np.eye(r), atol=1e-12)
    x = rng.standard_normal((5, d))
    assert np.allclose((x @ u) @ (np.diag(s) @ bt), x @ w, atol=1e-12)
    assert np.all(np.diff(s) <= 0) and s[-1] > 0                          # ordered, full rank
