"""Pins for the oracle's cross-layer path of grouped-query models, Sec. 3.3.2 of arxiv
2508.10395: deltas are cached in the shared latent space of U_kv (left singular vectors of
[Wk | Wv]) and merged into the accumulator through U_kv^T."""
from fractions import Fraction

import numpy as np

import xq_inputs as xi
from oracle import xq_oracle as xo


def bf(x):
    return xi.from_bf16_bits(x)


def bits(x):
    return xi.to_bf16_bits(np.asarray(x, np.float32))


def _bf16_ulp(v):
    e = np.floor(np.log2(np.maximum(np.abs(v), 1e-300)))
    return 2.0 ** (e - 7)


def _random_cache_rows(rng, rows, n_lat, G, b, spread=0.05):
    codes = rng.integers(0, 2 ** b, size=(rows, n_lat)).astype(np.uint8)
    scale = bits(np.abs(rng.standard_normal((rows, n_lat // G))) * spread + 1e-3)
    zero = bits(rng.standard_normal((rows, n_lat // G)) * spread)
    return codes, scale, zero


def test_delta_projection_is_the_nearest_bf16_of_the_fp64_product():
    rng = np.random.default_rng(21)
    x = bits(rng.standard_normal((6, 256)))
    a = bits(bf(x) + 0.1 * rng.standard_normal((6, 256)))
    ut = bits(rng.standard_normal((64, 256)) * 0.06)
    got = bf(xo.project_delta_rows(x, a, ut)).astype(np.float64)
    ref = (bf(x).astype(np.float64) - bf(a).astype(np.float64)) @ bf(ut).astype(np.float64).T
    assert np.all(np.abs(got - ref) <= 0.5 * _bf16_ulp(ref) * (1 + 1e-9))


def test_delta_projection_special_cases():
    rng = np.random.default_rng(22)
    x = bits(rng.standard_normal((3, 128)))
    ut = bits(rng.standard_normal((32, 128)))
    # accumulator equal to the input: the delta and hence its projection are exactly zero
    assert not np.any(bf(xo.project_delta_rows(x, x, ut)))
    # zero accumulator: the plain projection (pinned separately)
    assert np.array_equal(xo.project_delta_rows(x, bits(np.zeros((3, 128))), ut), xo.project_rows(x, ut))
    # the sign of the difference: swapping the operands negates every output
    a = bits(rng.standard_normal((3, 128)))
    p, q = bf(xo.project_delta_rows(x, a, ut)), bf(xo.project_delta_rows(a, x, ut))
    assert np.array_equal(p, -q) and np.any(p != 0)


def test_accumulate_latent_against_exact_rational_arithmetic():
    """Tiny case, every step redone with exact fractions: fp32 fma of the dequantisation (one
    rounding of an exact value), exact sum, exact addition, one rounding to bf16."""
    rng = np.random.default_rng(23)
    rows, n_lat, d, G, b = 3, 8, 5, 4, 3
    codes, scale, zero = _random_cache_rows(rng, rows, n_lat, G, b)
    ut = bits(rng.standard_normal((n_lat, d)))
    acc0 = bits(rng.standard_normal((rows, d)))
    got = xo.cl_accumulate_latent_rows(acc0.copy(), codes, scale, zero, ut, G)
    sf, zf, uf, af = bf(scale), bf(zero), bf(ut), bf(acc0)
    for r in range(rows):
        for n in range(d):
            tot = Fraction(float(af[r, n]))
            for c in range(n_lat):
                g = c // G
                dq_exact = Fraction(int(codes[r, c])) * Fraction(float(sf[r, g])) + Fraction(float(zf[r, g]))
                dqd = float(dq_exact)
                assert Fraction(dqd) == dq_exact           # code * bf16 + bf16 fits a double, so ...
                dq = np.float32(dqd)                       # ... this is the single rounding of the fp32 fma
                tot += Fraction(float(dq)) * Fraction(float(uf[c, n]))
            # nearest bf16 of the exact total: rounding through double and fp32 could round twice, so
            # pick among the neighbours with exact arithmetic
            near = int(bits(np.float32(float(tot))).reshape(-1)[0])
            best = min((near - 1, near, near + 1),
                       key=lambda u: abs(Fraction(float(bf(np.array([u], np.uint16))[0])) - tot))
            assert int(got[r, n]) == best


def test_accumulate_latent_with_a_selection_matrix_is_the_plain_accumulate():
    """U_kv whose columns are unit vectors: the up-projection scatters latent channel c to hidden
    channel perm[c] and leaves the other hidden channels alone, so those columns must equal the
    (separately pinned) element-wise accumulate bit for bit."""
    rng = np.random.default_rng(24)
    rows, n_lat, d, G, b = 5, 128, 320, 64, 2
    codes, scale, zero = _random_cache_rows(rng, rows, n_lat, G, b)
    perm = rng.permutation(d)[:n_lat]
    ut = np.zeros((n_lat, d), np.float32)
    ut[np.arange(n_lat), perm] = 1.0
    acc0 = bits(rng.standard_normal((rows, d)))
    got = xo.cl_accumulate_latent_rows(acc0.copy(), codes, scale, zero, bits(ut), G)
    sub = np.ascontiguousarray(acc0[:, perm])
    want_sub = xo.cl_accumulate_rows(sub, codes, scale, zero, G, init=False)
    assert np.array_equal(got[:, perm], want_sub)
    rest = np.setdiff1d(np.arange(d), perm)
    assert np.array_equal(got[:, rest], acc0[:, rest])


def test_accumulate_latent_matches_fp64_matmul():
    rng = np.random.default_rng(25)
    rows, n_lat, d, G, b = 9, 256, 384, 128, 4
    codes, scale, zero = _random_cache_rows(rng, rows, n_lat, G, b)
    ut = bits(rng.standard_normal((n_lat, d)) * 0.06)
    acc0 = bits(rng.standard_normal((rows, d)))
    got = bf(xo.cl_accumulate_latent_rows(acc0.copy(), codes, scale, zero, ut, G)).astype(np.float64)
    dq = xo.dequantize_rows(codes, scale, zero, G).astype(np.float64)          # pinned separately
    ref = bf(acc0).astype(np.float64) + dq @ bf(ut).astype(np.float64)         # library routine, fp64
    assert np.all(np.abs(got - ref) <= 0.5 * _bf16_ulp(ref) * (1 + 1e-6))


def test_up_projection_closes_the_loop_of_the_derivation():
    """The derivation closing Sec. 3.3.2: with W_kv = U S B^T and U^T U = I,
    (X^ + D U^T) W_kv = (X^ U + D) S B^T for any latent D.  A transposed U, a dropped accumulator
    or a wrong sign breaks it.  bf16 storage of U and of the result bounds the agreement."""
    rng = np.random.default_rng(26)
    d, n_lat, rows, G, b = 256, 128, 6, 64, 4
    W = rng.standard_normal((d, n_lat)) / np.sqrt(d)
    U, S, Bt = np.linalg.svd(W, full_matrices=False)
    ut = bits(U.T)                                                            # stored U_kv^T
    Ub = bf(ut).astype(np.float64).T
    codes, scale, zero = _random_cache_rows(rng, rows, n_lat, G, b, spread=0.2)
    D = xo.dequantize_rows(codes, scale, zero, G).astype(np.float64)
    acc0 = bits(rng.standard_normal((rows, d)))
    acc1 = bf(xo.cl_accumulate_latent_rows(acc0.copy(), codes, scale, zero, ut, G)).astype(np.float64)
    lhs = acc1 @ W
    rhs = (bf(acc0).astype(np.float64) @ Ub + D) * S @ Bt
    scale_ref = np.abs(rhs).max()
    assert np.abs(lhs - rhs).max() <= 0.02 * scale_ref
    # and it is the transpose that matters: with U^T U = I the other orientation is no identity
    wrong = bf(acc0).astype(np.float64) + D @ Ub.T[:, ::-1]
    assert np.abs(wrong @ W - rhs).max() > 0.2 * scale_ref


def test_delta_then_accumulate_recovers_a_delta_inside_the_subspace():
    """If X - X^ lies in the span of U_kv, projecting it down and back up loses nothing but the
    quantiser's and bf16's rounding (Sec. 3.3.2: lossless for an identity quantiser)."""
    rng = np.random.default_rng(27)
    d, n_lat, rows, G, b = 256, 128, 4, 128, 4
    U, _ = np.linalg.qr(rng.standard_normal((d, n_lat)))
    ut = bits(U.T)
    Ub = bf(ut).astype(np.float64).T
    acc0 = bits(rng.standard_normal((rows, d)))
    lat_true = rng.standard_normal((rows, n_lat))
    x = bits(bf(acc0).astype(np.float64) + lat_true @ Ub.T)
    lat = xo.project_delta_rows(x, acc0, ut)
    qc, qs, qz = xo.quantize_rows(bf(lat), G, b)
    acc1 = bf(xo.cl_accumulate_latent_rows(acc0.copy(), qc, qs, qz, ut, G)).astype(np.float64)
    err_before = np.abs(bf(x).astype(np.float64) - bf(acc0).astype(np.float64)).mean()
    err_after = np.abs(bf(x).astype(np.float64) - acc1).mean()
    # 4-bit codes over a range of about 6 sigma: step ~0.4 sigma, mean |error| ~0.1 sigma
    assert err_after < 0.2 * err_before


def test_accumulate_latent_rows_are_independent_and_empty_is_a_noop():
    rng = np.random.default_rng(28)
    rows, n_lat, d, G, b = 4, 64, 128, 64, 3
    codes, scale, zero = _random_cache_rows(rng, rows, n_lat, G, b)
    ut = bits(rng.standard_normal((n_lat, d)) * 0.1)
    acc0 = bits(rng.standard_normal((rows, d)))
    full = xo.cl_accumulate_latent_rows(acc0.copy(), codes, scale, zero, ut, G)
    for r in range(rows):
        one = xo.cl_accumulate_latent_rows(acc0[r:r + 1].copy(), codes[r:r + 1], scale[r:r + 1], zero[r:r + 1], ut, G)
        assert np.array_equal(one[0], full[r])
    empty = np.zeros((0, d), np.uint16)
    xo.cl_accumulate_latent_rows(empty, codes[:0], scale[:0], zero[:0], ut, G)
