"""GPU parity of xq_remat_attn_prefill (causal attention of the T newest tokens of every
sequence, scores and weighted sums on the matrix cores) against the oracle, which attends each
query over the prefix ending at its own row."""
import numpy as np
import pytest
import torch

import xq_inputs as xi
from oracle import xq_oracle as xo
from tests.util import assert_cache_equals, bits_to_torch, oracle_cache, rel_errors

pytestmark = pytest.mark.gpu

TOL = 2e-3


@pytest.fixture(scope="module")
def xq():
    import paper_2508_10395_amd as m
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    m.load_library()
    return m


def table(n_pos, hd=128, base=10000.0):
    inv = base ** (-np.arange(hd // 2, dtype=np.float64) * 2.0 / hd)
    ang = np.arange(n_pos, dtype=np.float64)[:, None] * inv[None, :]
    return np.stack([np.cos(ang), np.sin(ang)], axis=-1).astype(np.float32)


def gen_queries(w, T, seed):
    """[B][T][Hq][hd] bf16 bits with the scale of the workload's decode queries."""
    rng = np.random.default_rng(seed)
    q1 = xi.from_bf16_bits(xi.gen_q(w)).astype(np.float64)
    return xi.to_bf16_bits((rng.standard_normal((w.B, T, w.Hq, w.hd)) * q1.std()).astype(np.float32))


def _run(xq, w, T, bits, G, lens, triples=None, dense=False, rope=None, pos0=None, seed=0):
    x, (wk, wv) = xi.gen_x(w), xi.gen_weights(w)
    q = gen_queries(w, T, seed)
    attn = xq.XQAttn(w.Hq, w.Hkv, w.hd, w.hd ** -0.5)
    if triples is None:
        triples = [(b, t, h) for b in range(w.B) for t in range(T) for h in range(w.Hq)]
    common = dict(q_bf16=q, Wk=wk, Wv=wv, Hq=w.Hq, Hkv=w.Hkv, hd=w.hd, softmax_scale=w.hd ** -0.5, lens=lens,
                  triples=triples)
    gk = {}
    if rope is not None:
        common.update(rope_cos_sin=rope, pos0=pos0)
        gk = dict(rope_cos_sin=torch.from_numpy(rope).cuda(), pos0=pos0)
    if dense:
        wprep = xq.xq_prepare_weights(attn, w.d, 128, 16, bits_to_torch(wk), bits_to_torch(wv))
        out = xq.xq_remat_attn_prefill(attn, bits_to_torch(q), wprep, lens, acc_bf16=bits_to_torch(x), **gk)
        torch.cuda.synchronize()
        ref = xo.prefill_attn_triples(acc_bf16=x, **common)
    else:
        cache = xq.alloc_cache(w.B, w.L, w.d, G, bits)
        xq.xq_quantize_append(cache, bits_to_torch(x), [0] * w.B)
        wprep = xq.xq_prepare_weights(attn, w.d, G, bits, bits_to_torch(wk), bits_to_torch(wv))
        out = xq.xq_remat_attn_prefill(attn, bits_to_torch(q), wprep, lens, xcache=cache, **gk)
        torch.cuda.synchronize()
        seqs = [b for b, _, _ in triples]
        packed, scale, zero = oracle_cache(x, G, bits, seqs=seqs)               # the oracle's own cache
        assert_cache_equals(cache, packed, scale, zero, w.L, seqs=seqs)
        ref = xo.prefill_attn_triples(packed=packed, scale=scale, zero=zero, G=G, bits=bits, **common)
    got = out.cpu().numpy()
    sel = np.array([got[b, t, h] for b, t, h in triples])
    normwise, maxwise = rel_errors(sel, ref)
    assert np.all(np.isfinite(got)), w.name
    assert normwise.max() <= TOL and maxwise <= TOL, (w.name, T, float(normwise.max()), float(maxwise))
    return float(normwise.max())


@pytest.mark.parametrize("T", [1, 5, 32, 45])
def test_prefill_mha_ragged(xq, T):
    """One KV head per query head: T queries per head; 45 needs two passes of 32 query rows.  Lengths
    put the query rows inside a chunk, across a chunk boundary and across a tile boundary."""
    w = xi.C2.scaled(B=4, L=600, d=512, Hq=4, Hkv=4, n_outlier=5)
    _run(xq, w, T, 3, 128, lens=[600, 257 + T // 2, T, 512], seed=T)


@pytest.mark.parametrize("bits,G", [(2, 64), (2, 128), (4, 64), (4, 128), (8, 64), (8, 128)])
def test_prefill_formats(xq, bits, G):
    w = xi.C2.scaled(B=2, L=300, d=512, Hq=4, Hkv=4, n_outlier=5)
    _run(xq, w, 7, bits, G, lens=[300, 40], seed=bits + G)


@pytest.mark.parametrize("T", [1, 3, 16])
def test_prefill_gqa(xq, T):
    """4 query heads per KV head: 4 T query rows per KV head (64 at T = 16: two passes)."""
    w = xi.C4.scaled(B=2, L=300, d=768, Hq=8, Hkv=2)
    _run(xq, w, T, 2, 64, lens=[300, 130], seed=T)


@pytest.mark.parametrize("Hq,T,dense", [(8, 5, False), (6, 11, False), (10, 7, False), (6, 9, True)])
def test_prefill_gqa_groups_of_128(xq, Hq, T, dense):
    """4, 3 and 5 query heads per KV head with groups of 128 (and from the accumulator): the epilogue of the
    16x16x32 kernels takes the (token, head) rows 16 at a time -- 20, 33, 35 and 27 rows, so the last pass is
    ragged and a pass straddles query tokens; lengths put the rows across a tile boundary."""
    w = xi.C4.scaled(B=2, L=600, d=512, Hq=Hq, Hkv=2)
    _run(xq, w, T, 3, 128, lens=[600, 253 + T], seed=Hq + T, dense=dense)


def test_prefill_dense_source_and_rope(xq):
    w3 = xi.C3.scaled(B=2, L=330, d=512, Hq=4, Hkv=4)
    _run(xq, w3, 9, 0, 0, lens=[330, 100], dense=True)
    _run(xq, w3, 9, 0, 0, lens=[330, 100], dense=True, rope=table(500), pos0=[3, 150])
    w = xi.C2.scaled(B=2, L=300, d=512, Hq=4, Hkv=4, n_outlier=5)
    _run(xq, w, 20, 3, 128, lens=[300, 281], rope=table(1200), pos0=[0, 900])


def test_single_query_agrees_with_the_decode_entry_point(xq):
    w = xi.C2.scaled(B=3, L=400, d=512, Hq=4, Hkv=4, n_outlier=5)
    x, (wk, wv), q = xi.gen_x(w), xi.gen_weights(w), xi.gen_q(w)
    attn = xq.XQAttn(w.Hq, w.Hkv, w.hd, w.hd ** -0.5)
    cache = xq.alloc_cache(w.B, w.L, w.d, 128, 3)
    xq.xq_quantize_append(cache, bits_to_torch(x), [0] * w.B)
    wprep = xq.xq_prepare_weights(attn, w.d, 128, 3, bits_to_torch(wk), bits_to_torch(wv))
    lens = [400, 33, 256]
    dec = xq.xq_remat_attn_decode(attn, bits_to_torch(q), wprep, lens, xcache=cache).cpu().numpy()
    pre = xq.xq_remat_attn_prefill(attn, bits_to_torch(q).reshape(w.B, 1, w.Hq, w.hd).contiguous(), wprep, lens,
                                   xcache=cache).cpu().numpy()[:, 0]
    normwise, maxwise = rel_errors(pre.reshape(-1, w.hd), dec.reshape(-1, w.hd))
    assert normwise.max() < 2e-4 and maxwise < 2e-4


def test_prefill_argument_errors(xq):
    w = xi.C2.scaled(B=2, L=64, d=256, Hq=2, Hkv=2, n_outlier=0)
    attn = xq.XQAttn(w.Hq, w.Hkv, w.hd, w.hd ** -0.5)
    cache = xq.alloc_cache(2, 64, 256, 128, 3)
    wprep = xq.xq_prepare_weights(attn, 256, 128, 3, bits_to_torch(xi.gen_weights(w)[0]), bits_to_torch(xi.gen_weights(w)[1]))
    q = torch.zeros((2, 5, 2, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(xq.XQError):
        xq.xq_remat_attn_prefill(attn, q, wprep, [64, 4], xcache=cache)          # fewer rows than queries
    with pytest.raises(xq.XQError):
        xq.xq_remat_attn_prefill(attn, q, wprep, [64, 65], xcache=cache)         # past the capacity
    with pytest.raises(xq.XQError):
        xq.xq_remat_attn_prefill(attn, q, wprep, [64, 64], xcache=cache, workspace=torch.empty(64, dtype=torch.uint8, device="cuda"))


def test_full_size_llama2_7b_chunk_of_32_sampled(xq):
    """Config 2 at full size with a chunk of 32 new tokens per sequence; the oracle redoes sampled
    (sequence, query, head) triples, among them the first and the last query of the chunk."""
    w = xi.C2
    T = 32
    rng = np.random.default_rng(2)
    triples = [(0, 0, 0), (w.B - 1, T - 1, w.Hq - 1)] + [(int(rng.integers(w.B)), int(rng.integers(T)), int(rng.integers(w.Hq)))
                                                         for _ in range(6)]
    worst = _run(xq, w, T, w.bits, w.G, [w.L] * w.B, triples=triples)
    print(f"c2 prefill chunk of 32, sampled triples: worst norm-wise rel err {worst:.2e}")


def test_full_size_chunk_of_128_sampled(xq):
    """Config 2's layer at full hidden size and context, two sequences, a chunk of 128 new tokens each (four
    passes of 32 query rows per tile).  Sampled queries: the first and the last of the chunk and the two
    either side of a pass boundary, three heads each."""
    w = xi.C2.scaled(B=2)
    T = 128
    triples = [(b, t, h) for t in (0, 31, 32, T - 1) for b, h in ((0, 0), (1, w.Hq - 1), (1, 13))]
    worst = _run(xq, w, T, w.bits, w.G, [w.L, w.L - 77], triples=triples, seed=128)
    print(f"c2 shape, prefill chunk of 128, sampled triples: worst norm-wise rel err {worst:.2e}")


def test_full_size_long_context_chunk_of_512_sampled(xq):
    """Config 5's 512-token chunk attending causally over the whole 32768-row context (2-bit, group 128, d=4096,
    32 heads), one sequence of the four: 16 passes of 32 query rows per tile, 128 tiles, the last two tiles cut
    by the causal mask.  The oracle redoes the first and the last query of the chunk on three heads each."""
    w = xi.C5.scaled(B=1)
    T = 512
    triples = [(0, t, h) for t in (0, T - 1) for h in (0, 17, w.Hq - 1)]
    worst = _run(xq, w, T, w.bits, w.G, [w.L], triples=triples, seed=512)
    print(f"c5 shape, prefill chunk of 512, sampled triples: worst norm-wise rel err {worst:.2e}")


def test_prefill_maximum_batch(xq):
    """The largest batch any call accepts (128 sequences), ragged, three queries each."""
    w = xi.C2.scaled(B=128, L=96, d=256, Hq=2, Hkv=2, n_outlier=2)
    lens = [3 + (7 * b) % 94 for b in range(w.B)]
    rng = np.random.default_rng(5)
    triples = [(int(rng.integers(w.B)), int(rng.integers(3)), int(rng.integers(w.Hq))) for _ in range(40)] + [(127, 2, 1), (0, 0, 0)]
    _run(xq, w, 3, 3, 128, lens=lens, triples=triples)
