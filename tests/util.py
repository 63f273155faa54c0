"""Helpers shared by the tests: bf16-bit <-> torch conversions and error metrics."""
import numpy as np
import torch


def bits_to_torch(bits_u16, device="cuda"):
    """numpy uint16 bf16 bit patterns -> torch.bfloat16 tensor on `device`."""
    t = torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16)).view(torch.bfloat16)
    return t.to(device)


def torch_to_bits(t):
    """torch.bfloat16 tensor -> numpy uint16 bit patterns (host)."""
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def rel_errors(got, ref):
    """Per-row norm-wise relative error and the global max-wise relative error."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    normwise = np.linalg.norm(got - ref, axis=-1) / np.linalg.norm(ref, axis=-1)
    maxwise = np.abs(got - ref).max() / np.abs(ref).max()
    return normwise, maxwise


def oracle_cache(x_bits, G, bits, seqs=None, cap=None):
    """The oracle's own per-token cache of x ([B][L][d] bf16 bits): packed codes [B][cap][d bits/8],
    scale and zero bf16 bits [B][cap][d/G].  Only the sequences in `seqs` are quantised (all of them
    if None); the others and the rows past L stay zero."""
    import xq_inputs as xi
    from oracle import xq_oracle as xo
    B, L, d = x_bits.shape
    cap = L if cap is None else cap
    packed = np.zeros((B, cap, d * bits // 8), np.uint8)
    scale = np.zeros((B, cap, d // G), np.uint16)
    zero = np.zeros((B, cap, d // G), np.uint16)
    for b in (range(B) if seqs is None else sorted(set(seqs))):
        c, s, z = xo.quantize_rows(xi.from_bf16_bits(x_bits[b]), G, bits)
        packed[b, :L], scale[b, :L], zero[b, :L] = xo.pack_rows(c, bits), s, z
    return packed, scale, zero


def assert_cache_equals(cache, packed, scale, zero, rows, seqs=None):
    """The GPU library's cache holds the oracle's bytes on the first `rows` rows of the sequences in
    `seqs` (all if None)."""
    gc, gs, gz = cache.codes.cpu().numpy(), torch_to_bits(cache.scale), torch_to_bits(cache.zero)
    for b in (range(gc.shape[0]) if seqs is None else sorted(set(seqs))):
        assert np.array_equal(gc[b, :rows], packed[b, :rows]), ("codes", b)
        assert np.array_equal(gs[b, :rows], scale[b, :rows]), ("scale", b)
        assert np.array_equal(gz[b, :rows], zero[b, :rows]), ("zero", b)


def oracle_cache_per_channel(x_bits, G, bits, lens, seqs=None):
    """The oracle's own per-channel cache of x ([B][L][d] bf16 bits) for sequences of lens[b] rows: the
    complete blocks of G tokens quantised per channel (packed codes [B][cap][d bits/8], scale and zero bf16
    bits [B][cap/G][d], cap = L rounded up to whole blocks) and the bf16 window [B][G][d] holding the
    rows after the last complete block.  Only the sequences in `seqs` are filled (all if None)."""
    import xq_inputs as xi
    from oracle import xq_oracle as xo
    B, L, d = x_bits.shape
    cap = (L + G - 1) // G * G
    packed = np.zeros((B, cap, d * bits // 8), np.uint8)
    scale = np.zeros((B, cap // G, d), np.uint16)
    zero = np.zeros((B, cap // G, d), np.uint16)
    tail = np.zeros((B, G, d), np.uint16)
    for b in (range(B) if seqs is None else sorted(set(seqs))):
        nblk, rem = divmod(lens[b], G)
        if nblk:
            c, s, z = xo.quantize_blocks_per_channel(xi.from_bf16_bits(x_bits[b, :nblk * G]), G, bits)
            packed[b, :nblk * G], scale[b, :nblk], zero[b, :nblk] = xo.pack_rows(c, bits), s, z
        tail[b, :rem] = x_bits[b, nblk * G:lens[b]]
    return packed, scale, zero, tail


def assert_cache_per_channel_equals(cache, packed, scale, zero, G, lens, seqs=None):
    """The GPU library's per-channel cache holds the oracle's bytes on the complete blocks."""
    gc, gs, gz = cache.codes.cpu().numpy(), torch_to_bits(cache.scale), torch_to_bits(cache.zero)
    for b in (range(gc.shape[0]) if seqs is None else sorted(set(seqs))):
        nblk = lens[b] // G
        assert np.array_equal(gc[b, :nblk * G], packed[b, :nblk * G]), ("codes", b)
        assert np.array_equal(gs[b, :nblk], scale[b, :nblk]), ("scale", b)
        assert np.array_equal(gz[b, :nblk], zero[b, :nblk]), ("zero", b)
