"""Pins for the oracle's per-channel quantiser (groups of G consecutive tokens per channel,
Sec. 3.3.1 of arxiv 2508.10395: the paper's best setting for X U_k)."""
import numpy as np

import xq_inputs as xi
from oracle import xq_oracle as xo


def bf(x):
    return xi.from_bf16_bits(x)


def _x(seed, rows, d):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, d)).astype(np.float32)
    x[:, 3] *= 40.0                                   # an outlier channel: per-channel groups isolate it
    return bf(xi.to_bf16_bits(x))


def test_per_channel_is_the_per_token_quantiser_on_the_transposed_block():
    """A group is the same arithmetic whichever axis it runs along: block^T quantised per token
    with one group per row (the pinned quantiser) must give the same codes, scales, zero-points."""
    G, d = 64, 96
    for bits in (2, 3, 4):
        x = _x(bits, 3 * G, d)
        codes, scale, zero = xo.quantize_blocks_per_channel(x, G, bits)
        for blk in range(3):
            xt = np.ascontiguousarray(x[blk * G:(blk + 1) * G].T)                # [d][G]
            c2, s2, z2 = xo.quantize_rows(xt, G, bits)
            assert np.array_equal(codes[blk * G:(blk + 1) * G], c2.T)
            assert np.array_equal(scale[blk], s2[:, 0]) and np.array_equal(zero[blk], z2[:, 0])


def test_exact_grid_and_dequantisation():
    """Channel c of block b holds min + k*step exactly (representable values): codes are k, and the
    dequantised block is the input bit for bit."""
    G, d, bits = 32, 8, 3
    k = np.random.default_rng(0).integers(0, 8, size=(2 * G, d))
    k[0], k[1] = 0, 7                                                            # every channel spans the range
    k[G], k[G + 1] = 0, 7
    step = 2.0 ** -np.arange(d)                                                  # bf16-exact steps
    mn = -np.arange(d, dtype=np.float64)
    x = (mn + k * step).astype(np.float32)
    codes, scale, zero = xo.quantize_blocks_per_channel(x, G, bits)
    assert np.array_equal(codes, k.astype(np.uint8))
    assert np.array_equal(bf(scale)[0], step.astype(np.float32)) and np.array_equal(bf(zero)[1], mn.astype(np.float32))
    assert np.array_equal(xo.dequantize_blocks_per_channel(codes, scale, zero, G), x)


def test_round_trip_bound_and_outlier_isolation():
    G, d, bits = 128, 64, 4
    x = _x(9, 2 * G, d)
    codes, scale, zero = xo.quantize_blocks_per_channel(x, G, bits)
    xh = xo.dequantize_blocks_per_channel(codes, scale, zero, G)
    s = np.repeat(bf(scale).astype(np.float64), G, axis=0)
    z = np.repeat(bf(zero).astype(np.float64), G, axis=0)
    # half a step, plus what rounding the zero-point and the step to bf16 moves the grid by
    qmax = 2 ** bits - 1
    assert np.all(np.abs(xh - x) <= 0.5 * s + np.abs(z) * 2.0 ** -8 + qmax * s * 2.0 ** -8 + 1e-30)
    # the outlier channel does not spoil its neighbours (it would under per-token groups)
    err_pc = np.abs(xh - x)[:, :3].mean()
    ct, st, zt = xo.quantize_rows(x, 64, bits)
    err_pt = np.abs(xo.dequantize_rows(ct, st, zt, 64) - x)[:, :3].mean()
    assert err_pc < 0.25 * err_pt


def test_dequantisation_is_one_fma_per_element():
    G, d, bits = 16, 5, 2
    rng = np.random.default_rng(4)
    codes = rng.integers(0, 4, size=(G, d)).astype(np.uint8)
    scale = xi.to_bf16_bits(rng.random((1, d)).astype(np.float32) + 0.1)
    zero = xi.to_bf16_bits(rng.standard_normal((1, d)).astype(np.float32))
    got = xo.dequantize_blocks_per_channel(codes, scale, zero, G)
    exact = codes.astype(np.float64) * bf(scale).astype(np.float64) + bf(zero).astype(np.float64)   # exact in fp64
    assert np.array_equal(got, exact.astype(np.float32))                        # one rounding


def test_attention_from_per_channel_cache_and_residual_window_equals_brute_force():
    from scipy.special import softmax
    rng = np.random.default_rng(12)
    B, L, d, G, bits, Hq, Hkv, hd = 2, 3 * 32 + 9, 256, 32, 4, 4, 2, 128
    x = xi.to_bf16_bits(rng.standard_normal((B, L, d)).astype(np.float32))
    wk = xi.to_bf16_bits((rng.standard_normal((d, Hkv * hd)) * d ** -0.5).astype(np.float32))
    wv = xi.to_bf16_bits((rng.standard_normal((d, Hkv * hd)) * d ** -0.5).astype(np.float32))
    q = xi.to_bf16_bits(rng.standard_normal((B, Hq, hd)).astype(np.float32))
    lens = [L, 2 * 32]                                   # one sequence with a window of 9, one with none
    cap = 4 * 32
    codes = np.zeros((B, cap, d), np.uint8)
    scale = np.zeros((B, cap // G, d), np.uint16)
    zero = np.zeros_like(scale)
    tail = np.zeros((B, G, d), np.uint16)
    xhat = []
    for b in range(B):
        nblk, rem = lens[b] // G, lens[b] % G
        c, s, z = xo.quantize_blocks_per_channel(bf(x[b, :nblk * G]), G, bits)
        codes[b, :nblk * G], scale[b, :nblk], zero[b, :nblk] = c, s, z
        tail[b, :rem] = x[b, nblk * G:lens[b]]
        xhat.append(np.concatenate([xo.dequantize_blocks_per_channel(c, s, z, G), bf(x[b, nblk * G:lens[b]])]))
    pairs = [(b, h) for b in range(B) for h in range(Hq)]
    got = xo.remat_attn_pairs_per_channel(q_bf16=q, Wk=wk, Wv=wv, Hq=Hq, Hkv=Hkv, hd=hd, softmax_scale=hd ** -0.5,
                                          lens=lens, pairs=pairs, packed=xo.pack_rows(codes, bits), scale=scale,
                                          zero=zero, G=G, bits=bits, tail_bf16=tail)
    for i, (b, hq) in enumerate(pairs):
        hk = hq // (Hq // Hkv)
        X = xhat[b].astype(np.float64)
        K = X @ bf(wk)[:, hk * hd:(hk + 1) * hd].astype(np.float64)
        V = X @ bf(wv)[:, hk * hd:(hk + 1) * hd].astype(np.float64)
        ref = softmax(K @ bf(q)[b, hq].astype(np.float64) * hd ** -0.5) @ V
        assert np.allclose(got[i], ref, rtol=1e-5, atol=1e-6)


def test_latent_attention_with_per_channel_keys_equals_brute_force():
    from scipy.special import softmax
    rng = np.random.default_rng(31)
    B, L, r, Gk, Gv, kb, vb, Hq, Hkv, hd = 2, 70, 256, 32, 64, 3, 4, 4, 2, 128
    lk = xi.to_bf16_bits(rng.standard_normal((B, L, r)).astype(np.float32))       # X Uk rows
    lv = xi.to_bf16_bits(rng.standard_normal((B, L, r)).astype(np.float32))       # X Uv rows
    wfk = xi.to_bf16_bits((rng.standard_normal((r, Hkv * hd)) * r ** -0.5).astype(np.float32))
    wfv = xi.to_bf16_bits((rng.standard_normal((r, Hkv * hd)) * r ** -0.5).astype(np.float32))
    q = xi.to_bf16_bits(rng.standard_normal((B, Hq, hd)).astype(np.float32))
    lens = [70, 64]
    cap = 96
    kcodes = np.zeros((B, cap, r), np.uint8)
    kscale = np.zeros((B, cap // Gk, r), np.uint16)
    kzero = np.zeros_like(kscale)
    ktail = np.zeros((B, Gk, r), np.uint16)
    xk = []
    for b in range(B):
        nblk, rem = lens[b] // Gk, lens[b] % Gk
        c, s, z = xo.quantize_blocks_per_channel(bf(lk[b, :nblk * Gk]), Gk, kb)
        kcodes[b, :nblk * Gk], kscale[b, :nblk], kzero[b, :nblk] = c, s, z
        ktail[b, :rem] = lk[b, nblk * Gk:lens[b]]
        xk.append(np.concatenate([xo.dequantize_blocks_per_channel(c, s, z, Gk), bf(lk[b, nblk * Gk:lens[b]])]))
    vc, vs, vz = xo.quantize_rows(bf(lv), Gv, vb)
    xv = xo.dequantize_rows(vc, vs, vz, Gv)
    pairs = [(b, h) for b in range(B) for h in range(Hq)]
    got = xo.latent_attn_pairs_per_channel(q_bf16=q, Wfk=wfk, Wfv=wfv, Hq=Hq, Hkv=Hkv, hd=hd, softmax_scale=hd ** -0.5,
                                           lens=lens, pairs=pairs, k_packed=xo.pack_rows(kcodes, kb), k_scale=kscale,
                                           k_zero=kzero, k_G=Gk, k_bits=kb, k_tail_bf16=ktail,
                                           v_packed=xo.pack_rows(vc, vb), v_scale=vs, v_zero=vz, v_G=Gv, v_bits=vb)
    for i, (b, hq) in enumerate(pairs):
        hk = hq // (Hq // Hkv)
        K = xk[b].astype(np.float64) @ bf(wfk)[:, hk * hd:(hk + 1) * hd].astype(np.float64)
        V = xv[b, :lens[b]].astype(np.float64) @ bf(wfv)[:, hk * hd:(hk + 1) * hd].astype(np.float64)
        ref = softmax(K @ bf(q)[b, hq].astype(np.float64) * hd ** -0.5) @ V
        assert np.allclose(got[i], ref, rtol=1e-5, atol=1e-6)


def _latent_case(seed, lens, B=2, L=70, r=256, Gk=32, Gv=64, kb=2, vb=4, Hq=4, Hkv=2, hd=128, ch0=None):
    """Caches of synthetic latent rows; ch0(b) may overwrite channel 0 of X Uk before quantising."""
    rng = np.random.default_rng(seed)
    lkf = rng.standard_normal((B, L, r)).astype(np.float32)
    lkf[..., 0] *= 30.0                                                           # the outlier channel of X Uk
    if ch0 is not None:
        lkf[..., 0] = ch0
    lk = xi.to_bf16_bits(lkf)
    lv = xi.to_bf16_bits(rng.standard_normal((B, L, r)).astype(np.float32))
    wfk = xi.to_bf16_bits((rng.standard_normal((r, Hkv * hd)) * r ** -0.5).astype(np.float32))
    wfv = xi.to_bf16_bits((rng.standard_normal((r, Hkv * hd)) * r ** -0.5).astype(np.float32))
    q = xi.to_bf16_bits(rng.standard_normal((B, Hq, hd)).astype(np.float32))
    cap = (L + Gk - 1) // Gk * Gk
    kcodes = np.zeros((B, cap, r), np.uint8)
    kscale = np.zeros((B, cap // Gk, r), np.uint16)
    kzero = np.zeros_like(kscale)
    ktail = np.zeros((B, Gk, r), np.uint16)
    xk = []
    for b in range(B):
        nblk, rem = lens[b] // Gk, lens[b] % Gk
        c, s, z = xo.quantize_blocks_per_channel(bf(lk[b, :nblk * Gk]), Gk, kb)
        kcodes[b, :nblk * Gk], kscale[b, :nblk], kzero[b, :nblk] = c, s, z
        ktail[b, :rem] = lk[b, nblk * Gk:lens[b]]
        xk.append(np.concatenate([xo.dequantize_blocks_per_channel(c, s, z, Gk), bf(lk[b, nblk * Gk:lens[b]])]))
    vc, vs, vz = xo.quantize_rows(bf(lv), Gv, vb)
    kw = dict(q_bf16=q, Wfk=wfk, Wfv=wfv, Hq=Hq, Hkv=Hkv, hd=hd, softmax_scale=hd ** -0.5, lens=lens,
              pairs=[(b, h) for b in range(B) for h in range(Hq)], k_packed=xo.pack_rows(kcodes, kb), k_scale=kscale,
              k_zero=kzero, k_G=Gk, k_bits=kb, k_tail_bf16=ktail, v_packed=xo.pack_rows(vc, vb), v_scale=vs, v_zero=vz,
              v_G=Gv, v_bits=vb)
    return kw, xk, xo.dequantize_rows(vc, vs, vz, Gv), lkf


def test_fp16_outlier_channel_equals_brute_force():
    """App. B: channel 0 of X Uk kept in fp16.  Brute force: the dequantised latent keys with column 0 (and no
    other column) replaced by the fp16 values, then textbook attention."""
    from scipy.special import softmax
    lens = [70, 64]
    kw, xk, xv, lkf = _latent_case(41, lens)
    k0 = lkf[..., 0].astype(np.float16)                                           # [B][L] IEEE half
    got = xo.latent_attn_pairs_per_channel(k0_f16=k0.view(np.uint16), **kw)
    plain = xo.latent_attn_pairs_per_channel(**kw)
    Hq, Hkv, hd = kw["Hq"], kw["Hkv"], kw["hd"]
    for i, (b, hq) in enumerate(kw["pairs"]):
        hk = hq // (Hq // Hkv)
        lat = xk[b].astype(np.float64).copy()
        lat[:, 0] = k0[b, :lens[b]].astype(np.float64)
        K = lat @ bf(kw["Wfk"])[:, hk * hd:(hk + 1) * hd].astype(np.float64)
        V = xv[b, :lens[b]].astype(np.float64) @ bf(kw["Wfv"])[:, hk * hd:(hk + 1) * hd].astype(np.float64)
        ref = softmax(K @ bf(kw["q_bf16"])[b, hq].astype(np.float64) * hd ** -0.5) @ V
        assert np.allclose(got[i], ref, rtol=1e-5, atol=1e-6)
    # 2-bit codes of a channel thirty times wider than the others: keeping it in fp16 must matter
    assert np.abs(got - plain).max() > 1e-3 * np.abs(plain).max()


def test_fp16_outlier_channel_special_cases():
    lens = [70, 64]
    # a constant channel 0 dequantises to its zero-point exactly (scale 0), a small bf16 number that fp16 holds
    # exactly, and so do the window rows: the fp16 copy then changes nothing at all
    kw, _, _, lkf = _latent_case(42, lens, ch0=1.25)
    k0 = lkf[..., 0].astype(np.float16)
    assert np.array_equal(xo.latent_attn_pairs_per_channel(k0_f16=k0.view(np.uint16), **kw),
                          xo.latent_attn_pairs_per_channel(**kw))
    # with a zero first row of Sk Bk^T the channel cannot reach the keys, whatever it holds
    kw, _, _, lkf = _latent_case(43, lens)
    wz = kw["Wfk"].copy()
    wz[0, :] = 0
    a = xo.latent_attn_pairs_per_channel(**dict(kw, Wfk=wz))
    junk = np.random.default_rng(1).standard_normal(lkf[..., 0].shape).astype(np.float16)
    assert np.array_equal(xo.latent_attn_pairs_per_channel(k0_f16=junk.view(np.uint16), **dict(kw, Wfk=wz)), a)
    # rows past lens[b] of the fp16 array are not read
    k0 = lkf[..., 0].astype(np.float16)
    k0b = k0.copy()
    k0b[1, lens[1]:] = np.float16(np.nan)
    assert np.array_equal(xo.latent_attn_pairs_per_channel(k0_f16=k0.view(np.uint16), **kw),
                          xo.latent_attn_pairs_per_channel(k0_f16=k0b.view(np.uint16), **kw))
