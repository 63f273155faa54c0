"""CPU pins for the oracle's quantiser, packer and dequantiser (no GPU).

Each test pins the oracle to something that is not the oracle: closed forms,
exact rational arithmetic, torch's own bf16 conversion, hand-written bytes, and
the cache sizes the paper prints.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import xq_inputs as xi
from oracle import xq_oracle as xo

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def bf(x):
    return xi.from_bf16_bits(x)


# ---------------------------------------------------------------- closed forms


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
@pytest.mark.parametrize("G", [64, 128])
def test_exact_grid_gives_its_own_indices(bits, G):
    """A group that is exactly {mn + k*s} with power-of-two s quantises to k and
    dequantises without error."""
    nlev = 1 << bits
    s, mn = 0.25, -1.5
    k = (np.arange(G * 3) * 7) % nlev
    k[0::G], k[1::G] = 0, nlev - 1               # both extremes present in every group
    x = (mn + k * s).astype(np.float32).reshape(1, -1)
    codes, scale, zero = xo.quantize_rows(x, G, bits)
    assert np.array_equal(codes.reshape(-1), k.astype(np.uint8))
    assert np.all(bf(scale) == np.float32(s)) and np.all(bf(zero) == np.float32(mn))
    assert np.array_equal(xo.dequantize_rows(codes, scale, zero, G), x)


def test_constant_group_and_signed_zero():
    x = np.full((2, 128), 3.25, np.float32)
    x[1, :] = -0.0
    codes, scale, zero = xo.quantize_rows(x, 128, 3)
    assert not codes.any() and not scale.any()
    assert bf(zero)[0, 0] == np.float32(3.25)
    assert zero[1, 0] == 0                       # -0 stored as +0
    assert np.array_equal(xo.dequantize_rows(codes, scale, zero, 128)[0], x[0])


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_two_valued_group_hits_the_ends(bits):
    rng = np.random.default_rng(1)
    pick = rng.integers(0, 2, 128).astype(bool)
    pick[:2] = [False, True]
    x = np.where(pick, np.float32(0.7), np.float32(-2.1)).reshape(1, 128).astype(np.float32)
    codes, _, _ = xo.quantize_rows(bf(xi.to_bf16_bits(x)), 128, bits)
    assert np.array_equal(codes[0], np.where(pick, (1 << bits) - 1, 0))


def test_ties_round_half_to_even():
    """mn=0, mx=3, 2 bits -> step 1: 0.5 -> 0, 1.5 -> 2, 2.5 -> 2."""
    x = np.zeros((1, 128), np.float32)
    x[0, :6] = [0.0, 3.0, 0.5, 1.5, 2.5, 1.0]
    codes, scale, _ = xo.quantize_rows(x, 128, 2)
    assert bf(scale)[0, 0] == 1.0
    assert codes[0, :6].tolist() == [0, 3, 0, 2, 2, 1]
    # 3 bits, step 0.5 on [0, 3.5]: 0.25 -> 0 (0.5 ties to 0), 0.75 -> 2, 1.25 -> 2
    y = np.zeros((1, 128), np.float32)
    y[0, :5] = [0.0, 3.5, 0.25, 0.75, 1.25]
    codes, scale, _ = xo.quantize_rows(y, 128, 3)
    assert bf(scale)[0, 0] == 0.5
    assert codes[0, :5].tolist() == [0, 7, 0, 2, 2]


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_monotone_and_extremes(bits):
    w = xi.C2.scaled(B=1, L=16)
    x = bf(xi.gen_x(w))[0]
    codes, scale, zero = xo.quantize_rows(x, 128, bits)
    xg = x.reshape(16, -1, 128)
    cg = codes.reshape(16, -1, 128).astype(np.int32)
    order = np.argsort(xg, axis=-1, kind="stable")
    assert np.all(np.diff(np.take_along_axis(cg, order, -1), axis=-1) >= 0)
    assert np.all(np.take_along_axis(cg, xg.argmin(-1)[..., None], -1) == 0)
    assert np.all(np.take_along_axis(cg, xg.argmax(-1)[..., None], -1) == (1 << bits) - 1)
    assert np.array_equal(bf(zero), xg.min(-1))          # bf16 inputs: zero is the exact minimum


# ------------------------------------------------- metadata rounding, exactness


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_scale_and_zero_bits_match_torch_bf16(bits):
    """scale = RNE_bf16(fp32(mx-mn)/fp32(2^b-1)), zero = RNE_bf16(mn): checked with
    torch's float32 division and torch's bfloat16 cast (library routines)."""
    rng = np.random.default_rng(5 + bits)
    x = (rng.standard_normal((64, 512)) * rng.choice([1e-3, 1.0, 37.0], (64, 1))).astype(np.float32)
    _, scale, zero = xo.quantize_rows(x, 128, bits)
    xt = torch.from_numpy(x).reshape(64, 4, 128)
    mn, mx = xt.amin(-1), xt.amax(-1)
    st = ((mx - mn) / float((1 << bits) - 1)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    zt = mn.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(scale, st)
    assert np.array_equal(zero, zt)


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_codes_equal_exact_rational_rounding(bits):
    """fp32 divide followed by rint equals round-half-even of the exact quotient
    (x - zero)/scale taken over the rationals -- for fp32 inputs (delta-like data)
    and bf16 inputs (many exact ties)."""
    rng = np.random.default_rng(11 + bits)
    xa = rng.standard_normal((4, 128)).astype(np.float32) * np.float32(0.3)
    xb = bf(xi.to_bf16_bits(rng.standard_normal((60, 128)).astype(np.float32)))
    x = np.concatenate([xa, xb])
    codes, scale, zero = xo.quantize_rows(x, 128, bits)
    qmax = (1 << bits) - 1
    n_ties = 0
    for r in range(x.shape[0]):
        sf = Fraction(float(bf(scale)[r, 0]))
        for i in range(128):
            num = Fraction(float(np.float32(x[r, i]) - np.float32(bf(zero)[r, 0])))  # fp32 subtract
            quo = num / sf
            fl = quo.numerator // quo.denominator
            rem = quo - fl
            if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
                fl += 1
            n_ties += rem == Fraction(1, 2)
            assert codes[r, i] == min(max(fl, 0), qmax), (r, i)
    if bits <= 4:
        assert n_ties > 0          # the bf16 rows really exercise the tie rule


@pytest.mark.parametrize("w,bits,G", [(xi.C1, 4, 128), (xi.C2, 3, 128), (xi.C4, 2, 64), (xi.C5, 2, 128),
                                      (xi.C2, 8, 128)])
def test_round_trip_within_half_step(w, bits, G):
    """|x - x^| <= scale/2 (+ fp32 rounding slack) for every element; bf16 inputs
    store the minimum exactly, so there is no zero-point term.  The stored scale
    is rounded to bf16 (relative error <= 2^-8), so the top code can fall short of
    the maximum by (2^b-1)*scale*2^-8: below half a step for b <= 6, up to one
    step at 8 bits."""
    x = bf(xi.gen_x(w.scaled(B=1, L=32)))[0]
    codes, scale, zero = xo.quantize_rows(x, G, bits)
    xh = xo.dequantize_rows(codes, scale, zero, G)
    sf = np.repeat(bf(scale), G, axis=-1)
    slack = 4 * np.spacing(np.abs(x) + np.abs(xh)).astype(np.float32)
    qmax = (1 << bits) - 1
    assert np.all(np.abs(x - xh) <= np.maximum(sf / 2, qmax * sf / 256) + slack)
    assert bits > 4 or qmax / 256 < 0.5
    assert np.abs(x - xh).max() > 0                      # it is a lossy quantiser


def test_dequantize_is_one_fused_multiply_add():
    """code*scale+zero with a single rounding: compare with float64 evaluation
    rounded once (exact, since the product has < 53 significant bits)."""
    rng = np.random.default_rng(3)
    codes = rng.integers(0, 16, (8, 256)).astype(np.uint8)
    scale = xi.to_bf16_bits(rng.uniform(0.01, 3, (8, 2)).astype(np.float32))
    zero = xi.to_bf16_bits(rng.standard_normal((8, 2)).astype(np.float32) * 100)
    xh = xo.dequantize_rows(codes, scale, zero, 128)
    ref = (codes.astype(np.float64) * np.repeat(bf(scale).astype(np.float64), 128, -1)
           + np.repeat(bf(zero).astype(np.float64), 128, -1)).astype(np.float32)
    assert np.array_equal(xh, ref)


# ------------------------------------------------------------------- packing


def _pack_vectors():
    out = []
    for line in open(os.path.join(GOLD, "pack_vectors.txt")):
        if line.startswith("#") or not line.strip():
            continue
        b, c, y = line.split("|")
        out.append((int(b), [int(t) for t in c.split()], bytes.fromhex(y.strip().replace(" ", ""))))
    return out


@pytest.mark.parametrize("bits,codes,expect", _pack_vectors())
def test_pack_golden_bytes(bits, codes, expect):
    packed = xo.pack_rows(np.array([codes], np.uint8), bits)
    assert packed.tobytes() == expect
    assert xo.unpack_rows(packed, len(codes), bits)[0].tolist() == codes


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_pack_unpack_round_trip_and_bit_positions(bits):
    rng = np.random.default_rng(bits)
    codes = rng.integers(0, 1 << bits, (5, 384)).astype(np.uint8)
    packed = xo.pack_rows(codes, bits)
    assert packed.shape == (5, 384 * bits // 8)
    assert np.array_equal(xo.unpack_rows(packed, 384, bits), codes)
    # brute force: the row as one big little-endian integer
    for r in range(5):
        big = int.from_bytes(packed[r].tobytes(), "little")
        for j in (0, 1, 7, 31, 32, 33, 200, 383):
            assert (big >> (j * bits)) & ((1 << bits) - 1) == codes[r, j]


# -------------------------------------------------- storage format vs the paper


def _size_rows():
    rows = []
    for line in open(os.path.join(GOLD, "cache_sizes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        t, m, nt, b, v = line.split()
        rows.append((t, m, int(nt), int(b), float(v)))
    return rows


@pytest.mark.parametrize("table,method,ntens,bits,printed", _size_rows())
def test_stored_bytes_reproduce_the_papers_cache_sizes(table, method, ntens, bits, printed):
    """Bytes the oracle actually emits per token (packed codes + scale + zero),
    relative to an fp16 K+V cache, round to the sizes printed in Tables 1 and 4."""
    d, G = 4096, 128
    x = bf(xi.gen_x(xi.C2.scaled(B=1, L=2)))[0]

    def token_bytes(b):
        codes, scale, zero = xo.quantize_rows(x, G, b)
        return (xo.pack_rows(codes, b).nbytes + scale.nbytes + zero.nbytes) / x.shape[0]

    # ntens = 1: one X tensor of width d replaces K and V; ntens = 2: K and V each of width d
    fp16_kv = 2 * 2 * d
    if table == "table1":
        frac = ntens * token_bytes(bits) / fp16_kv
    else:                                   # first 3 of 32 layers at 4 bits
        frac = ntens * (3 * token_bytes(4) + 29 * token_bytes(bits)) / (32 * fp16_kv)
    assert abs(frac - printed) <= 0.005 + 1e-9, (frac, printed)
