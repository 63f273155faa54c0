"""GPU parity of the cross-layer path of grouped-query models, Sec. 3.3.2 of arxiv 2508.10395:
xq_cl_latent_delta_project, xq_prepare_upproject and xq_cl_accumulate_latent against the oracle.

Tolerances.  The projection and the up-projection accumulate in fp32 on the matrix cores, the
oracle in double.  With A = sum of |terms| of an output, the fp32 result lies within A * 2^-16 of
the exact sum (bound: (n/16 MFMA accumulations + n/G rescalings + 3) * 2^-23 * A for n <= 2048
contraction indices; observed errors are far smaller), so the stored bf16 is a correct rounding of
a number that close to the exact one: |stored - exact| <= half a bf16 ulp + A * 2^-16.  The share
of elements that differ from the oracle's bits at all is checked to be small."""
import numpy as np
import pytest
import torch

import xq_inputs as xi
from oracle import xq_oracle as xo
from tests.util import bits_to_torch, rel_errors, torch_to_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def xq():
    import paper_2508_10395_amd as m
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    m.load_library()
    return m


def bf(x):
    return xi.from_bf16_bits(x)


def bits(x):
    return xi.to_bf16_bits(np.asarray(x, np.float32))


def _ulp(v):
    return 2.0 ** (np.floor(np.log2(np.maximum(np.abs(v), 1e-30))) - 7)


def _subspace(rng, d, n_lat):
    """U_kv^T [n_lat][d]: orthonormal columns from a QR (the offline SVD's left factor has the
    same property); bf16 as stored."""
    u, _ = np.linalg.qr(rng.standard_normal((d, n_lat)))
    return bits(u.T)


def _check_rounded(got_bits, exact, absum, ref_bits, max_mismatch):
    g = bf(got_bits).astype(np.float64)
    assert np.all(np.abs(g - exact) <= 0.5 * _ulp(exact) * 1.0001 + absum * 2.0 ** -16)
    mismatch = float(np.mean(got_bits != ref_bits))
    assert mismatch <= max_mismatch, mismatch
    return mismatch


@pytest.mark.parametrize("B,T,cap,d,n_lat", [(1, 1, 5, 256, 64), (8, 1, 300, 512, 256), (3, 17, 64, 384, 96)])
def test_delta_projection_matches_oracle(xq, B, T, cap, d, n_lat):
    rng = np.random.default_rng(100 * B + T)
    ut = _subspace(rng, d, n_lat)
    acc = bits(rng.standard_normal((B, cap, d)))
    start = [int(v) for v in rng.integers(0, cap - T + 1, size=B)]
    rows = np.stack([acc[b, start[b]:start[b] + T] for b in range(B)])           # [B][T][d]
    x = bits(bf(rows) + 0.2 * rng.standard_normal((B, T, d)))
    out = torch.full((B, T, n_lat), 7.0, dtype=torch.bfloat16, device="cuda")
    xq.xq_cl_latent_delta_project(bits_to_torch(x), bits_to_torch(acc), bits_to_torch(ut), start, out=out)
    torch.cuda.synchronize()
    ref = xo.project_delta_rows(x, rows, ut)
    delta = bf(x).astype(np.float64) - bf(rows).astype(np.float64)
    exact = delta @ bf(ut).astype(np.float64).T
    absum = np.abs(delta) @ np.abs(bf(ut)).astype(np.float64).T
    _check_rounded(torch_to_bits(out), exact, absum, ref, 0.01)


def test_delta_projection_of_an_unchanged_input_is_zero_and_empty_is_a_noop(xq):
    rng = np.random.default_rng(3)
    ut = _subspace(rng, 256, 64)
    acc = bits(rng.standard_normal((2, 9, 256)))
    out = xq.xq_cl_latent_delta_project(bits_to_torch(acc[:, 4:6]), bits_to_torch(acc), bits_to_torch(ut), [4, 4])
    torch.cuda.synchronize()
    assert not np.any(bf(torch_to_bits(out)))
    e = xq.xq_cl_latent_delta_project(torch.empty((2, 0, 256), dtype=torch.bfloat16, device="cuda"),
                                      bits_to_torch(acc), bits_to_torch(ut), [0, 0])
    assert e.shape == (2, 0, 64)


def _accumulate_case(xq, B, cap, d, n_lat, G, b, lens, seed, sample_rows=None, outlier=True):
    rng = np.random.default_rng(seed)
    if n_lat <= d and d * n_lat <= 1 << 20:
        ut = _subspace(rng, d, n_lat)
    else:                                           # large, or wider than the hidden size: near-orthonormal rows
        ut = bits(rng.standard_normal((n_lat, d)) * d ** -0.5)
    acc0 = torch.randn((B, cap, d), generator=torch.Generator().manual_seed(seed)).to(torch.bfloat16)
    lat = torch.randn((B, cap, n_lat), generator=torch.Generator().manual_seed(seed + 1)) * 0.3
    if outlier:
        lat[..., 0] *= 20.0                                                     # the latent space keeps an outlier channel
    cache = xq.alloc_cache(B, cap, n_lat, G, b)
    xq.xq_quantize_append(cache, lat.to(torch.bfloat16).cuda(), [0] * B)
    uprep = xq.xq_prepare_upproject(d, G, b, bits_to_torch(ut))
    acc = acc0.cuda()
    xq.xq_cl_accumulate_latent(acc, cache, uprep, lens)
    torch.cuda.synchronize()
    got = torch_to_bits(acc)
    a0 = torch_to_bits(acc0)
    gp, gs, gz = cache.codes.cpu().numpy(), torch_to_bits(cache.scale), torch_to_bits(cache.zero)
    lat_bits = torch_to_bits(lat.to(torch.bfloat16))             # the seeded latent rows, as both sides got them
    utf = bf(ut).astype(np.float64)
    worst = 0.0
    for s in range(B):
        n = lens[s]
        assert np.array_equal(got[s, n:], a0[s, n:]), "rows at or past len must not change"
        if n == 0 or (sample_rows is not None and s >= 3):
            continue
        rows = np.arange(n) if sample_rows is None else np.unique(np.minimum(sample_rows, n - 1))
        codes, sc, ze = xo.quantize_rows(bf(lat_bits[s, rows]), G, b)           # the oracle's own cache rows
        assert np.array_equal(gp[s, rows], xo.pack_rows(codes, b))
        assert np.array_equal(gs[s, rows], sc) and np.array_equal(gz[s, rows], ze)
        ref = xo.cl_accumulate_latent_rows(np.ascontiguousarray(a0[s, rows]), codes, sc, ze, ut, G)
        dq = xo.dequantize_rows(codes, sc, ze, G).astype(np.float64)
        exact = bf(a0[s, rows]).astype(np.float64) + dq @ utf
        absum = np.abs(bf(a0[s, rows])).astype(np.float64) + np.abs(dq) @ np.abs(utf)
        worst = max(worst, _check_rounded(got[s, rows], exact, absum, ref, 0.01))
    return worst


@pytest.mark.parametrize("bits_,G", [(2, 64), (2, 128), (3, 64), (3, 128), (4, 64), (4, 128)])
def test_accumulate_latent_formats(xq, bits_, G):
    _accumulate_case(xq, B=3, cap=300, d=512, n_lat=256, G=G, b=bits_, lens=[300, 257, 31], seed=10 * bits_ + G)


@pytest.mark.parametrize("d,n_lat", [(256, 128), (1024, 128), (256, 1024), (768, 384)])
def test_accumulate_latent_shapes(xq, d, n_lat):
    """One slab and several, one column block of the hidden size and several, ragged and empty
    sequences, a sequence ending exactly on a tile boundary."""
    _accumulate_case(xq, B=4, cap=520, d=d, n_lat=n_lat, G=128, b=3, lens=[520, 0, 256, 1], seed=d + n_lat)


def test_accumulate_latent_all_empty_is_a_noop(xq):
    _accumulate_case(xq, B=2, cap=40, d=256, n_lat=128, G=64, b=4, lens=[0, 0], seed=1)


def test_two_layers_chain_like_the_oracle(xq):
    """Two cross-layer steps end to end on the GPU (project the delta of every cached token,
    quantise, merge) against the same chain in the oracle; the approximation X^ must also get
    closer to the true input, which is the point of caching the delta."""
    rng = np.random.default_rng(77)
    B, L, d, n_lat, G, b = 2, 130, 512, 256, 128, 4
    ut = _subspace(rng, d, n_lat)
    utf = bf(ut).astype(np.float64)
    base = rng.standard_normal((B, L, d))
    acc_bits = bits(base)
    acc = bits_to_torch(acc_bits)
    acc_ref = acc_bits.copy()
    uprep = xq.xq_prepare_upproject(d, G, b, bits_to_torch(ut))
    x_prev = base
    for layer in (1, 2):
        x_true = x_prev + 0.3 * (rng.standard_normal((B, L, n_lat)) @ utf)       # the change lives in the subspace
        xb = bits(x_true)
        lat = xq.xq_cl_latent_delta_project(bits_to_torch(xb), acc, bits_to_torch(ut), [0] * B)
        cache = xq.alloc_cache(B, L, n_lat, G, b)
        xq.xq_quantize_append(cache, lat, [0] * B)
        before = np.abs(bf(xb).astype(np.float64) - bf(torch_to_bits(acc)).astype(np.float64)).mean()
        # the oracle's own chain: it starts from the same seeded accumulator and keeps its own afterwards
        lat_ref = xo.project_delta_rows(xb, acc_ref, ut)
        qc, qs, qz = xo.quantize_rows(bf(lat_ref), G, b)
        xo.cl_accumulate_latent_rows(acc_ref.reshape(B * L, d), qc.reshape(B * L, n_lat), qs.reshape(B * L, -1),
                                     qz.reshape(B * L, -1), ut, G)
        xq.xq_cl_accumulate_latent(acc, cache, uprep, [L] * B)
        torch.cuda.synchronize()
        got = bf(torch_to_bits(acc)).astype(np.float64)
        after = np.abs(bf(xb).astype(np.float64) - got).mean()
        assert after < 0.35 * before
        # a latent value that rounds the other way on the GPU moves a code by one step, so the
        # two chains are compared by norm, not bit for bit
        normwise, _ = rel_errors(got.reshape(B * L, d), bf(acc_ref).astype(np.float64).reshape(B * L, d))
        assert normwise.max() < 0.02
        x_prev = x_true


def test_full_size_llama3_8b_accumulate_sampled_rows(xq):
    """Config 4's shape: B=16, L=8192, d=4096, latent width 2048 (2 d / g), 2-bit, group 64; the
    oracle redoes sampled rows of three sequences."""
    w = xi.C4
    n_lat = 2 * w.Hkv * w.hd
    lens = [w.L] * w.B
    lens[1], lens[2] = w.L - 300, 1
    worst = _accumulate_case(xq, B=w.B, cap=w.L, d=w.d, n_lat=n_lat, G=w.G, b=w.bits, lens=lens, seed=4,
                             sample_rows=np.array([0, 1, 255, 256, 4095, 7891, 7892, 8191]))
    print(f"c4 up-projecting accumulate: share of elements off by one bf16 ulp {worst:.2e}")


@pytest.mark.parametrize("B,T,cap,d,n_lat", [(1, 300, 400, 256, 256), (3, 17, 64, 384, 256), (4, 700, 900, 512, 512),
                                             (2, 256, 256, 128, 256)])
def test_bulk_delta_projection_matches_oracle(xq, B, T, cap, d, n_lat):
    """The matrix-core route of the delta projection: x U - acc U summed in one fp32 accumulator.  Its
    accumulation error is relative to sum (|x| + |acc|) |U|, so that is the sum the bound uses; T = 17 makes
    the 256-row tiles straddle sequences, whose accumulator rows start at different offsets."""
    rng = np.random.default_rng(1000 * B + T)
    ut = bits(rng.standard_normal((n_lat, d)) * d ** -0.5)
    acc = bits(rng.standard_normal((B, cap, d)))
    start = [int(v) for v in rng.integers(0, cap - T + 1, size=B)]
    rows = np.stack([acc[b, start[b]:start[b] + T] for b in range(B)])           # [B][T][d]
    x = bits(bf(rows) + 0.2 * rng.standard_normal((B, T, d)))
    proj = xq.xq_prepare_projection(bits_to_torch(ut))
    out = torch.full((B, T, n_lat), 7.0, dtype=torch.bfloat16, device="cuda")
    xq.xq_cl_latent_delta_project_bulk(bits_to_torch(x), bits_to_torch(acc), proj, n_lat, start, out=out)
    small = xq.xq_cl_latent_delta_project(bits_to_torch(x), bits_to_torch(acc), bits_to_torch(ut), start)
    torch.cuda.synchronize()
    ref = xo.project_delta_rows(x, rows, ut)
    uf = np.abs(bf(ut)).astype(np.float64).T
    exact = (bf(x).astype(np.float64) - bf(rows).astype(np.float64)) @ bf(ut).astype(np.float64).T
    absum = (np.abs(bf(x)).astype(np.float64) + np.abs(bf(rows)).astype(np.float64)) @ uf
    mismatch = _check_rounded(torch_to_bits(out), exact, absum, ref, 0.01)
    assert np.mean(torch_to_bits(out) != torch_to_bits(small)) <= 0.01            # two routes to the same sum
    print(f"bulk delta projection B={B} T={T}: share of elements off the oracle's bits {mismatch:.2e}")


def test_bulk_delta_projection_edge_cases(xq):
    rng = np.random.default_rng(8)
    d, n_lat = 256, 256
    ut = bits(rng.standard_normal((n_lat, d)) * d ** -0.5)
    proj = xq.xq_prepare_projection(bits_to_torch(ut))
    acc = bits(rng.standard_normal((2, 300, d)))
    # an unchanged input: x U and acc U cancel up to the fp32 accumulation error of either sum
    out = xq.xq_cl_latent_delta_project_bulk(bits_to_torch(acc[:, 10:290]), bits_to_torch(acc), proj, n_lat, [10, 10])
    torch.cuda.synchronize()
    absum = 2.0 * np.abs(bf(acc[:, 10:290])).astype(np.float64) @ np.abs(bf(ut)).astype(np.float64).T
    assert np.all(np.abs(bf(torch_to_bits(out)).astype(np.float64)) <= absum * 2.0 ** -16)
    e = xq.xq_cl_latent_delta_project_bulk(torch.empty((2, 0, d), dtype=torch.bfloat16, device="cuda"), bits_to_torch(acc),
                                           proj, n_lat, [0, 0])
    assert e.shape == (2, 0, n_lat)
    with pytest.raises(xq.XQError):                                               # rows past the accumulator's capacity
        xq.xq_cl_latent_delta_project_bulk(bits_to_torch(acc[:, :100]), bits_to_torch(acc), proj, n_lat, [0, 201])
