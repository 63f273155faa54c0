"""GPU parity of the per-channel path (groups along the token axis with a bf16 residual window,
Sec. 3.3.1 of arxiv 2508.10395) against the oracle: the block quantiser bit for bit, the
attention within the tolerance of the fused kernels."""
import numpy as np
import pytest
import torch

import xq_inputs as xi
from oracle import xq_oracle as xo
from tests.util import bits_to_torch, rel_errors, torch_to_bits

pytestmark = pytest.mark.gpu

TOL = 2e-3


@pytest.fixture(scope="module")
def xq():
    import paper_2508_10395_amd as m
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    m.load_library()
    return m


def bf(x):
    return xi.from_bf16_bits(x)


def _rows(seed, B, rows, d):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((B, rows, d)).astype(np.float32)
    x[..., 0] *= 50.0                                   # the latent space's outlier channel
    x[..., 5] = 1.25                                    # a constant channel: zero scale
    x[:, :, 7] = np.where(np.arange(rows)[None, :] % 2 == 0, -0.0, 0.0)   # zeros of both signs
    return xi.to_bf16_bits(x)


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
@pytest.mark.parametrize("G,d", [(64, 128), (128, 1024), (128, 1536), (64, 4096)])
def test_block_quantiser_bit_exact(xq, bits, G, d):
    B, nblk, cap = 3, 2, 5 * G
    x = _rows(bits * 1000 + d, B, nblk * G, d)
    cache = xq.alloc_cache_per_channel(B, cap, d, G, bits)
    cache.codes.fill_(0xAB)
    block0 = [0, 3, 1]
    xq.xq_quantize_blocks_per_channel(cache, bits_to_torch(x), block0)
    torch.cuda.synchronize()
    codes, scale, zero = xo.quantize_blocks_per_channel(bf(x), G, bits)
    packed = xo.pack_rows(codes, bits)
    got_c, got_s, got_z = cache.codes.cpu().numpy(), torch_to_bits(cache.scale), torch_to_bits(cache.zero)
    for b in range(B):
        r0 = block0[b] * G
        assert np.array_equal(got_c[b, r0:r0 + nblk * G], packed[b])
        assert np.array_equal(got_s[b, block0[b]:block0[b] + nblk], scale[b])
        assert np.array_equal(got_z[b, block0[b]:block0[b] + nblk], zero[b])
        untouched = np.ones(cap, bool)
        untouched[r0:r0 + nblk * G] = False
        assert np.all(got_c[b, untouched] == 0xAB)      # rows of other blocks are not written


def test_block_quantiser_noop_and_errors(xq):
    cache = xq.alloc_cache_per_channel(2, 256, 256, 128, 3)
    xq.xq_quantize_blocks_per_channel(cache, torch.empty((2, 0, 256), dtype=torch.bfloat16, device="cuda"), [0, 0])
    x = torch.zeros((2, 128, 256), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(xq.XQError):
        xq.xq_quantize_blocks_per_channel(cache, x, [0, 2])                  # past the capacity
    with pytest.raises(xq.XQError):
        xq.xq_quantize_blocks_per_channel(xq.alloc_cache_per_channel(2, 256, 192, 64, 3),
                                          torch.zeros((2, 64, 192), dtype=torch.bfloat16, device="cuda"), [0, 0])
