"""GPU parity of xq_remat_attn_decode_rope (rotary embedding of the rematerialised keys) against
the oracle."""
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


def _check(got, ref, what):
    normwise, maxwise = rel_errors(got, ref)
    assert np.all(np.isfinite(got)), what
    assert normwise.max() <= TOL and maxwise <= TOL, (what, float(normwise.max()), float(maxwise))
    return float(normwise.max())


def _run(xq, w, bits, G, lens, pos0, n_pos, pairs=None, dense=False):
    x, (wk, wv), q = xi.gen_x(w), xi.gen_weights(w), xi.gen_q(w)
    tab = table(n_pos, w.hd)
    attn = xq.XQAttn(w.Hq, w.Hkv, w.hd, w.hd ** -0.5)
    t_tab = torch.from_numpy(tab).cuda()
    if pairs is None:
        pairs = [(b, h) for b in range(w.B) for h in range(w.Hq)]
    common = dict(q_bf16=q, Wk=wk, Wv=wv, Hq=w.Hq, Hkv=w.Hkv, hd=w.hd, softmax_scale=w.hd ** -0.5, lens=lens,
                  pairs=pairs, rope_cos_sin=tab, pos0=pos0)
    if dense:
        wprep = xq.xq_prepare_weights(attn, w.d, 128, 16, bits_to_torch(wk), bits_to_torch(wv))
        out = xq.xq_remat_attn_decode(attn, bits_to_torch(q), wprep, lens, acc_bf16=bits_to_torch(x),
                                      rope_cos_sin=t_tab, pos0=pos0)
        ref = xo.remat_attn_pairs(acc_bf16=x, **common)
    else:
        cache = xq.alloc_cache(w.B, w.L, w.d, G, bits)
        xq.xq_quantize_append(cache, bits_to_torch(x), [0] * w.B)
        wprep = xq.xq_prepare_weights(attn, w.d, G, bits, bits_to_torch(wk), bits_to_torch(wv))
        out = xq.xq_remat_attn_decode(attn, bits_to_torch(q), wprep, lens, xcache=cache, rope_cos_sin=t_tab, pos0=pos0)
        seqs = [b for b, _ in pairs]
        packed, scale, zero = oracle_cache(x, G, bits, seqs=seqs)               # the oracle's own cache
        assert_cache_equals(cache, packed, scale, zero, w.L, seqs=seqs)
        ref = xo.remat_attn_pairs(packed=packed, scale=scale, zero=zero, G=G, bits=bits, **common)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    return _check(np.array([got[b, h] for b, h in pairs]), ref, w.name)


@pytest.mark.parametrize("bits,G", [(2, 64), (3, 128), (4, 128)])
def test_rope_coded_ragged_with_offsets(xq, bits, G):
    w = xi.C2.scaled(B=4, L=600, d=512, Hq=4, Hkv=4, n_outlier=5)
    _run(xq, w, bits, G, lens=[600, 257, 1, 512], pos0=[0, 1000, 7, 88], n_pos=1300)


def test_rope_gqa_and_dense_source(xq):
    w = xi.C4.scaled(B=2, L=300, d=768, Hq=8, Hkv=2)
    _run(xq, w, 2, 64, lens=[300, 130], pos0=[0, 0], n_pos=300)
    w3 = xi.C3.scaled(B=2, L=330, d=512, Hq=4, Hkv=4)
    _run(xq, w3, 0, 0, lens=[330, 100], pos0=[3, 0], n_pos=400, dense=True)


def test_identity_table_changes_nothing_and_errors_are_caught(xq):
    w = xi.C2.scaled(B=2, L=300, d=512, Hq=4, Hkv=4, n_outlier=5)
    x, (wk, wv), q = xi.gen_x(w), xi.gen_weights(w), xi.gen_q(w)
    attn = xq.XQAttn(w.Hq, w.Hkv, w.hd, w.hd ** -0.5)
    cache = xq.alloc_cache(2, w.L, w.d, 128, 3)
    xq.xq_quantize_append(cache, bits_to_torch(x), [0, 0])
    wprep = xq.xq_prepare_weights(attn, w.d, 128, 3, bits_to_torch(wk), bits_to_torch(wv))
    ident = torch.zeros((300, 64, 2), dtype=torch.float32, device="cuda")
    ident[..., 0] = 1.0
    a = xq.xq_remat_attn_decode(attn, bits_to_torch(q), wprep, [300, 300], xcache=cache).cpu().numpy()
    b = xq.xq_remat_attn_decode(attn, bits_to_torch(q), wprep, [300, 300], xcache=cache, rope_cos_sin=ident).cpu().numpy()
    assert np.array_equal(a, b)
    with pytest.raises(xq.XQError):     # positions run past the table
        xq.xq_remat_attn_decode(attn, bits_to_torch(q), wprep, [300, 300], xcache=cache, rope_cos_sin=ident, pos0=[0, 1])


def test_rope_full_size_llama2_7b_sampled_pairs(xq):
    w = xi.C2
    worst = _run(xq, w, w.bits, w.G, [w.L] * w.B, pos0=[0] * w.B, n_pos=w.L, pairs=xi.sample_pairs(w, 8))
    print(f"c2 with rope, sampled pairs: worst norm-wise rel err {worst:.2e}")
