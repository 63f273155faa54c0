"""xq_remat_attn_decode_static -- the decode entry point that allocates nothing (its workspace is a buffer built
into the library) -- against xq_remat_attn_decode with a caller workspace, through the C ABI: two calls in a row,
the second on a smaller input, so that what the first call left in the shared buffer must not matter."""
import numpy as np
import pytest
import torch

import xq_inputs as xi
from tests.util import bits_to_torch, rel_errors

pytestmark = pytest.mark.gpu

TOL = 2e-3


@pytest.fixture(scope="module")
def xq():
    import paper_2508_10395_amd as m
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    m.load_library()
    return m


def _pair_of_calls(xq, w, bits, G, lens, dense=False):
    x, (wk, wv), q = xi.gen_x(w), xi.gen_weights(w), xi.gen_q(w)
    attn = xq.XQAttn(w.Hq, w.Hkv, w.hd, w.hd ** -0.5)
    qd = bits_to_torch(q)
    if dense:
        src = dict(acc_bf16=bits_to_torch(x))
        wprep = xq.xq_prepare_weights(attn, w.d, 128, 16, bits_to_torch(wk), bits_to_torch(wv))
    else:
        cache = xq.alloc_cache(w.B, w.L, w.d, G, bits)
        xq.xq_quantize_append(cache, bits_to_torch(x), [0] * w.B)
        src = dict(xcache=cache)
        wprep = xq.xq_prepare_weights(attn, w.d, G, bits, bits_to_torch(wk), bits_to_torch(wv))
    ref = xq.xq_remat_attn_decode(attn, qd, wprep, lens, **src)
    out = torch.full((w.B, w.Hq, w.hd), float("nan"), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    xq.xq_remat_attn_decode_static(attn, qd, wprep, lens, out=out, **src)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before                     # (torch's view: the binding allocated nothing)
    got, want = out.cpu().numpy(), ref.cpu().numpy()
    assert np.all(np.isfinite(got))
    normwise, maxwise = rel_errors(got.reshape(-1, w.hd), want.reshape(-1, w.hd))
    assert normwise.max() <= TOL and maxwise <= TOL, (float(normwise.max()), float(maxwise))
    assert np.array_equal(got, want)                                   # same kernels, same order of operations


def test_static_workspace_two_calls_second_smaller(xq):
    big = xi.C2.scaled(B=4, L=1500, d=1024, Hq=8, Hkv=8, n_outlier=10)
    _pair_of_calls(xq, big, 3, 128, lens=[1500, 1024, 77, 1300])
    small = xi.C2.scaled(B=2, L=300, d=512, Hq=4, Hkv=4, n_outlier=5)
    _pair_of_calls(xq, small, 3, 128, lens=[300, 33])
    # other format, grouped-query heads (matrix-core epilogue), then the accumulator source
    gqa = xi.C4.scaled(B=2, L=700, d=768, Hq=8, Hkv=2)
    _pair_of_calls(xq, gqa, 2, 64, lens=[700, 130])
    _pair_of_calls(xq, xi.C3.scaled(B=2, L=330, d=512, Hq=4, Hkv=4), 0, 0, lens=[330, 100], dense=True)


def test_static_workspace_refuses_what_does_not_fit(xq):
    """Config 4's batch, heads and context (B=16, 32 query heads, 8192 rows, group 64) need 69 MB of softmax
    partials alone, more than the built-in buffer: refused on the host, nothing is launched.  (Hidden size 128
    keeps this test's own cache small.)"""
    w = xi.C4
    attn = xq.XQAttn(w.Hq, w.Hkv, w.hd, w.hd ** -0.5)
    assert xq.xq_remat_attn_workspace_bytes(attn, w.B, w.L, 128, w.G) > xq.XQ_STATIC_SCRATCH_BYTES
    cache = xq.alloc_cache(w.B, w.L, 128, w.G, w.bits)
    q = torch.zeros((w.B, w.Hq, w.hd), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros((w.B, w.Hq, w.hd), dtype=torch.float32, device="cuda")
    wprep = torch.zeros(xq.xq_prepared_weights_bytes(attn, 128, w.G, w.bits), dtype=torch.uint8, device="cuda")
    with pytest.raises(xq.XQError, match="workspace"):
        xq.xq_remat_attn_decode_static(attn, q, wprep, [w.L] * w.B, xcache=cache, out=out)
