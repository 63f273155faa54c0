"""GPU parity: xq_quantize_append / xq_cl_delta_quantize / xq_cl_accumulate against the
CPU oracle, bit for bit (codes, scales, zero-points, accumulator)."""
import numpy as np
import pytest
import torch

import xq_inputs as xi
from oracle import xq_oracle as xo
from tests.util import bits_to_torch, torch_to_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def xq():
    import paper_2508_10395_amd as m
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    m.load_library()
    return m


def bf(x):
    return xi.from_bf16_bits(x)


def _oracle_rows(x_bits, G, bits):
    codes, scale, zero = xo.quantize_rows(bf(x_bits), G, bits)
    return xo.pack_rows(codes, bits), scale, zero


def _append_and_compare(xq, x_bits, G, bits, starts, cap):
    B, T, d = x_bits.shape
    cache = xq.alloc_cache(B, cap, d, G, bits)
    cache.codes.fill_(0xA5)
    cache.scale.view(torch.int16).fill_(0x1234)
    cache.zero.view(torch.int16).fill_(0x4321)
    xq.xq_quantize_append(cache, bits_to_torch(x_bits), starts)
    torch.cuda.synchronize()
    packed, scale, zero = _oracle_rows(x_bits, G, bits)
    gc, gs, gz = cache.codes.cpu().numpy(), torch_to_bits(cache.scale), torch_to_bits(cache.zero)
    for b in range(B):
        rows = slice(starts[b], starts[b] + T)
        assert np.array_equal(gs[b, rows], scale[b]), ("scale", b)
        assert np.array_equal(gz[b, rows], zero[b]), ("zero", b)
        assert np.array_equal(gc[b, rows], packed[b]), ("codes", b)
        untouched = np.ones(cap, bool)
        untouched[rows] = False
        assert np.all(gc[b, untouched] == 0xA5) and np.all(gs[b, untouched] == 0x1234) \
            and np.all(gz[b, untouched] == 0x4321), ("rows outside the append were written", b)


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
@pytest.mark.parametrize("G", [64, 128])
def test_append_matches_oracle_ragged(xq, bits, G):
    w = xi.C2.scaled(B=3, L=37, d=1280, n_outlier=13)
    x = xi.gen_x(w)
    _append_and_compare(xq, x, G, bits, starts=[0, 5, 11], cap=64)


@pytest.mark.parametrize("w,bits,G", [(xi.C1, 4, 128), (xi.C2.scaled(B=2, L=300), 3, 128),
                                      (xi.C4.scaled(B=2, L=129), 2, 64), (xi.C5.scaled(B=1, L=515), 2, 128)])
def test_append_config_shapes(xq, w, bits, G):
    x = xi.gen_x(w)
    _append_and_compare(xq, x, G, bits, starts=[3] * w.B, cap=w.L + 8)


def test_decode_append_single_token_and_noop(xq):
    w = xi.C2.scaled(B=8, L=1)
    x = xi.gen_x(w)
    _append_and_compare(xq, x, 128, 3, starts=list(range(8)), cap=16)
    cache = xq.alloc_cache(2, 4, 256, 128, 4)
    xq.xq_quantize_append(cache, torch.empty((2, 0, 256), dtype=torch.bfloat16, device="cuda"), [0, 4])
    torch.cuda.synchronize()
    assert not cache.codes.any()


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_degenerate_and_tie_groups(xq, bits):
    """Constant groups, signed zeros, two-valued groups, exact ties, huge and tiny magnitudes."""
    rng = np.random.default_rng(bits)
    rows = []
    base = rng.standard_normal((6, 256)).astype(np.float32)
    rows.append(np.full(256, 3.25, np.float32))
    rows.append(np.where(np.arange(256) % 2 == 0, np.float32(-0.0), np.float32(0.0)))
    rows.append(np.where(rng.integers(0, 2, 256) == 0, np.float32(-2.0), np.float32(0.75)))
    tie = np.zeros(256, np.float32)
    qmax = (1 << bits) - 1
    tie[:128] = (np.arange(128) % (2 * qmax + 1)) * 0.5        # steps of 0.5 on [0, qmax]: every tie
    tie[127] = qmax
    tie[128:] = (np.arange(128) % (2 * qmax + 1)) * 0.125 - 1.0
    tie[255] = qmax * 0.25 - 1.0
    rows.append(tie)
    rows.append(base[0] * np.float32(2.0 ** 60))
    rows.append(base[1] * np.float32(2.0 ** -60))
    rows.append(base[2] * np.float32(1e-3) + np.float32(100.0))   # large offset, small range
    rows.append(np.abs(base[3]))
    x = xi.to_bf16_bits(np.stack(rows))[None]
    _append_and_compare(xq, x, 128, bits, starts=[1], cap=12)
    _append_and_compare(xq, x, 64, bits, starts=[0], cap=8)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_every_bf16_scale_mantissa_and_many_exponents(xq, bits):
    """Groups built so that the stored scale runs over all 128 bf16 mantissas and
    exponents 2^-40..2^40: exercises the reciprocal-based rounding for every divisor."""
    qmax = (1 << bits) - 1
    rng = np.random.default_rng(40 + bits)
    mant = np.arange(128, dtype=np.uint32)
    exps = np.arange(87, 168, 4, dtype=np.uint32)                       # biased exponents
    sbits = ((exps[:, None] << 7) | mant[None, :]).reshape(-1).astype(np.uint16)
    s = bf(sbits).astype(np.float64)
    n = s.size
    frac = rng.uniform(0, qmax, (n, 128))
    frac[:, 0], frac[:, 1] = 0.0, qmax
    frac[:, 2:66] = np.round(frac[:, 2:66] * 2) / 2                     # plenty of exact half-steps
    x = xi.to_bf16_bits((frac * s[:, None]).astype(np.float32)).reshape(1, n // 2, 256)
    _append_and_compare(xq, x, 128, bits, starts=[0], cap=n // 2)


def _cl_reference(w, layers, base_bits, delta_bits, G, lens):
    xs = [xi.gen_x(w)]
    for l in range(1, layers):
        xs.append(xi.gen_next_layer_x(w, xs[-1], l))
    out = []
    c, s, z = xo.quantize_rows(bf(xs[0]), G, base_bits)
    acc = np.zeros_like(xs[0])
    for b in range(w.B):
        xo.cl_accumulate_rows(acc[b, :lens[b]], c[b, :lens[b]], s[b, :lens[b]], z[b, :lens[b]], G, init=True)
    out.append((xo.pack_rows(c, base_bits), s, z, acc.copy()))
    for l in range(1, layers):
        delta = xo.cl_delta_rows(xs[l], acc)
        c, s, z = xo.quantize_rows(delta, G, delta_bits)
        for b in range(w.B):
            xo.cl_accumulate_rows(acc[b, :lens[b]], c[b, :lens[b]], s[b, :lens[b]], z[b, :lens[b]], G, init=False)
        out.append((xo.pack_rows(c, delta_bits), s, z, acc.copy()))
    return xs, out


@pytest.mark.parametrize("base_bits,delta_bits,G", [(4, 2, 128), (4, 3, 64), (8, 4, 128)])
def test_cross_layer_stack_bit_exact(xq, base_bits, delta_bits, G):
    """Base layer -> accumulator, then per layer: delta-quantise against the accumulator,
    accumulate.  Every delta cache and every accumulator state must equal the oracle's bits."""
    w = xi.C3.scaled(B=2, L=70, d=512)
    layers, lens = 5, [70, 41]
    xs, ref = _cl_reference(w, layers, base_bits, delta_bits, G, lens)
    acc = torch.full((w.B, w.L, w.d), 7.0, dtype=torch.bfloat16, device="cuda")
    base = xq.alloc_cache(w.B, w.L, w.d, G, base_bits)
    xq.xq_quantize_append(base, bits_to_torch(xs[0]), [0, 0])
    xq.xq_cl_accumulate(acc, base, lens, init=True)
    torch.cuda.synchronize()
    got = torch_to_bits(acc)
    for b in range(w.B):
        assert np.array_equal(got[b, :lens[b]], ref[0][3][b, :lens[b]])
        assert np.all(got[b, lens[b]:] == 0x40E0)                       # rows >= len untouched (7.0)
    for l in range(1, layers):
        # rows >= len of the accumulator are not part of the state: make both sides agree on them
        acc_np = torch_to_bits(acc)
        ref_acc_prev = ref[l - 1][3]
        for b in range(w.B):
            acc_np[b, lens[b]:] = ref_acc_prev[b, lens[b]:]
        acc = bits_to_torch(acc_np)
        delta = xq.alloc_cache(w.B, w.L, w.d, G, delta_bits)
        xq.xq_cl_delta_quantize(delta, bits_to_torch(xs[l]), acc, [0, 0])
        xq.xq_cl_accumulate(acc, delta, lens, init=False)
        torch.cuda.synchronize()
        packed, s, z, racc = ref[l]
        assert np.array_equal(delta.codes.cpu().numpy(), packed), l
        assert np.array_equal(torch_to_bits(delta.scale), s), l
        assert np.array_equal(torch_to_bits(delta.zero), z), l
        got = torch_to_bits(acc)
        for b in range(w.B):
            assert np.array_equal(got[b, :lens[b]], racc[b, :lens[b]]), (l, b)


def test_cross_layer_decode_append_one_token(xq):
    """Decode-time use: the new token's delta goes to row len-1 of the delta cache."""
    w = xi.C3.scaled(B=3, L=9, d=256)
    G = 128
    x1 = xi.gen_next_layer_x(w, xi.gen_x(w), 1)
    acc_bits = xi.gen_x(w)
    starts = [8, 3, 0]
    new = np.stack([x1[b, starts[b]] for b in range(3)])[:, None, :]
    delta = xq.alloc_cache(3, 9, 256, G, 2)
    xq.xq_cl_delta_quantize(delta, bits_to_torch(new), bits_to_torch(acc_bits), starts)
    torch.cuda.synchronize()
    for b in range(3):
        d_ref = xo.cl_delta_rows(new[b], acc_bits[b, starts[b]:starts[b] + 1])
        c, s, z = xo.quantize_rows(d_ref, G, 2)
        assert np.array_equal(delta.codes[b, starts[b]].cpu().numpy(), xo.pack_rows(c, 2)[0])
        assert np.array_equal(torch_to_bits(delta.scale)[b, starts[b]], s[0])
        assert np.array_equal(torch_to_bits(delta.zero)[b, starts[b]], z[0])


def test_full_size_llama2_7b_bulk_append(xq):
    """The benchmark's quantise workload (B=8, T=4096, d=4096, 3-bit, G=128), every byte."""
    w = xi.C2
    x = xi.gen_x(w)
    cache = xq.alloc_cache(w.B, w.L, w.d, w.G, w.bits)
    xq.xq_quantize_append(cache, bits_to_torch(x), [0] * w.B)
    torch.cuda.synchronize()
    gc, gs, gz = cache.codes.cpu().numpy(), torch_to_bits(cache.scale), torch_to_bits(cache.zero)
    for b in range(w.B):                                  # one sequence at a time keeps host memory small
        packed, scale, zero = _oracle_rows(x[b], w.G, w.bits)
        assert np.array_equal(gs[b], scale) and np.array_equal(gz[b], zero), b
        assert np.array_equal(gc[b], packed), b
