"""The decode step (append one token, attend) captured into a HIP graph and replayed: the library only
enqueues kernels on the caller's stream and allocates nothing, so a serving loop can capture it.  Every
replay is checked against the eager result on the same inputs, with eager work between the replays."""
import numpy as np
import pytest
import torch

import xq_inputs as xi
from tests.util import bits_to_torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def xq():
    import paper_2508_10395_amd as m
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    m.load_library()
    return m


def test_decode_step_replays_from_a_graph(xq):
    w = xi.C2.scaled(B=2, L=520, d=512, Hq=4, Hkv=4, n_outlier=5)
    x, (wk, wv) = xi.gen_x(w), xi.gen_weights(w)
    attn = xq.XQAttn(w.Hq, w.Hkv, w.hd, w.hd ** -0.5)
    wprep = xq.xq_prepare_weights(attn, w.d, 128, 3, bits_to_torch(wk), bits_to_torch(wv))
    xt = bits_to_torch(x)
    L0 = 500                                             # tokens cached before the captured step
    lens = [L0 + 1] * w.B

    def fresh_cache():
        c = xq.alloc_cache(w.B, w.L, w.d, 128, 3)
        xq.xq_quantize_append(c, xt[:, :L0].contiguous(), [0] * w.B)
        return c

    # static buffers of the captured step
    cache = fresh_cache()
    x_new = torch.empty((w.B, 1, w.d), dtype=torch.bfloat16, device="cuda")
    q = torch.empty((w.B, w.Hq, w.hd), dtype=torch.bfloat16, device="cuda")
    out = torch.empty((w.B, w.Hq, w.hd), dtype=torch.float32, device="cuda")
    ws = torch.empty(xq.xq_remat_attn_workspace_bytes(attn, w.B, w.L, w.d, 128), dtype=torch.uint8, device="cuda")

    def step(c, xn, qq, o):
        xq.xq_quantize_append(c, xn, [L0] * w.B)
        xq.xq_remat_attn_decode(attn, qq, wprep, lens, xcache=c, out=o, workspace=ws)

    x_new.copy_(xt[:, L0:L0 + 1])
    q.copy_(torch.randn(q.shape, device="cuda").to(torch.bfloat16))
    step(cache, x_new, q, out)                           # warm-up outside the capture (first-use set-up of the launches)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(cache, x_new, q, out)
    gen = torch.Generator(device="cuda").manual_seed(3)
    for rep in range(4):
        x_new.copy_(xt[:, L0 + 1 + rep:L0 + 2 + rep])    # a different token and query every time
        q.copy_(torch.randn(q.shape, device="cuda", generator=gen).to(torch.bfloat16))
        graph.replay()
        torch.cuda.synchronize()
        got = out.clone()
        # eager reference on a separate cache and output, which is also the eager work between replays
        ref_cache = fresh_cache()
        ref_out = torch.empty_like(out)
        step(ref_cache, x_new, q, ref_out)
        torch.cuda.synchronize()
        assert torch.equal(got, ref_out), rep
        assert torch.equal(cache.codes[:, L0], ref_cache.codes[:, L0]) and torch.equal(cache.scale[:, L0], ref_cache.scale[:, L0])
