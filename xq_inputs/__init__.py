"""Seeded synthetic inputs shaped like the paper's Llama-class decode workloads.

This module only draws random tensors and lays them out; it contains none of
the method's arithmetic (no quantiser, no matmul, no softmax).  Both the CPU
oracle's tests and the GPU tests take their inputs from here, so the two sides
see identical bits.  bf16 tensors are returned as uint16 bit patterns.

Workloads (one decoder layer unless stated), after the five benchmark configs:

  c1  B=1  L=512   d=256  Hq=Hkv=2   4-bit G=128, 4 outlier channels x20
  c2  B=8  L=4096  d=4096 Hq=Hkv=32  3-bit G=128, 1% outlier channels x30   (Llama-2-7B shaped)
  c3  B=8  L=8192  d=4096 Hq=Hkv=32  cross-layer: base 4-bit, deltas 2-bit, 32 layers
  c4  B=16 L=8192  d=4096 Hq=32 Hkv=8 2-bit G=64, outliers as c2            (Llama-3-8B shaped, GQA)
  c5  B=4  L=32768 d=4096 Hq=Hkv=32  2-bit G=128, outliers as c2            (long context)

X ~ N(0,1) with the outlier channels multiplied by their factor, W ~ N(0, 1/d)
(second argument = variance), q ~ N(0,1), cross-layer steps
X_l = bf16(X_{l-1} + N(0, 0.1)).  Everything is rounded to bf16 (RNE).
"""
from dataclasses import dataclass, replace

import numpy as np

SEED0 = 0x5851F42D4C957F2D

T_X, T_WK, T_WV, T_Q, T_OUTLIER, T_DELTA = 0, 1, 2, 3, 4, 100


@dataclass(frozen=True)
class Workload:
    name: str
    cfg_id: int
    B: int
    L: int          # context attended at the decode step (rows in the cache after the append)
    d: int
    Hq: int
    Hkv: int
    hd: int
    bits: int
    G: int
    n_outlier: int
    outlier_factor: float
    layers: int = 1
    delta_bits: int = 0
    delta_var: float = 0.0

    def scaled(self, **kw):
        return replace(self, **kw)


C1 = Workload("c1_small_mha", 1, 1, 512, 256, 2, 2, 128, 4, 128, 4, 20.0)
C2 = Workload("c2_llama2_7b", 2, 8, 4096, 4096, 32, 32, 128, 3, 128, 41, 30.0)
C3 = Workload("c3_xquant_cl", 3, 8, 8192, 4096, 32, 32, 128, 4, 128, 0, 1.0,
              layers=32, delta_bits=2, delta_var=0.1)
C4 = Workload("c4_llama3_8b_gqa", 4, 16, 8192, 4096, 32, 8, 128, 2, 64, 41, 30.0)
C5 = Workload("c5_long_context", 5, 4, 32768, 4096, 32, 32, 128, 2, 128, 41, 30.0)

WORKLOADS = {w.cfg_id: w for w in (C1, C2, C3, C4, C5)}


def _rng(cfg_id, tensor_id):
    seed = (SEED0 ^ (cfg_id << 32) ^ tensor_id) & ((1 << 64) - 1)
    return np.random.Generator(np.random.Philox(key=seed))


def to_bf16_bits(x_f32):
    """fp32 array -> bf16 bit patterns, round-to-nearest-even (finite values)."""
    u = np.ascontiguousarray(x_f32, np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def from_bf16_bits(bits):
    return (np.ascontiguousarray(bits, np.uint16).astype(np.uint32) << 16).view(np.float32)


def _normal_bf16(rng, shape, std, col_scale=None, chunk_rows=4096):
    """N(0, std^2) rounded to bf16; optional per-last-axis multiplier."""
    shape = tuple(shape)
    ncols = shape[-1]
    nrows = int(np.prod(shape[:-1])) if len(shape) > 1 else 1
    out = np.empty((nrows, ncols), np.uint16)
    for r0 in range(0, nrows, chunk_rows):
        r1 = min(nrows, r0 + chunk_rows)
        blk = rng.standard_normal((r1 - r0, ncols), dtype=np.float32)
        if std != 1.0:
            blk *= np.float32(std)
        if col_scale is not None:
            blk *= col_scale
        out[r0:r1] = to_bf16_bits(blk)
    return out.reshape(shape)


def outlier_channels(w):
    """Seeded choice of which hidden channels carry the outlier factor."""
    if w.n_outlier == 0:
        return np.zeros(0, np.int64)
    return np.sort(_rng(w.cfg_id, T_OUTLIER).choice(w.d, size=w.n_outlier, replace=False))


def gen_x(w, rows=None):
    """Layer input X as bf16 bits, [B][rows][d] (rows defaults to L)."""
    rows = w.L if rows is None else rows
    col = np.ones(w.d, np.float32)
    col[outlier_channels(w)] = w.outlier_factor
    return _normal_bf16(_rng(w.cfg_id, T_X), (w.B, rows, w.d), 1.0,
                        col_scale=None if w.n_outlier == 0 else col)


def gen_weights(w, layer=0):
    """(Wk, Wv) bf16 bits, each [d][Hkv*hd], entries ~ N(0, 1/d)."""
    std = float(w.d) ** -0.5
    wk = _normal_bf16(_rng(w.cfg_id, T_WK + 1000 * layer), (w.d, w.Hkv * w.hd), std)
    wv = _normal_bf16(_rng(w.cfg_id, T_WV + 1000 * layer), (w.d, w.Hkv * w.hd), std)
    return wk, wv


def gen_q(w, layer=0):
    """Decode queries, bf16 bits [B][Hq][hd], ~ N(0,1)."""
    return _normal_bf16(_rng(w.cfg_id, T_Q + 1000 * layer), (w.B, w.Hq, w.hd), 1.0)


def gen_next_layer_x(w, x_prev_bits, layer):
    """True input of layer `layer` >= 1: bf16(X_{layer-1} + N(0, delta_var))."""
    rng = _rng(w.cfg_id, T_DELTA + layer)
    flat = x_prev_bits.reshape(-1, w.d)
    out = np.empty_like(flat)
    std = np.float32(np.sqrt(w.delta_var))
    for r0 in range(0, flat.shape[0], 4096):
        r1 = min(flat.shape[0], r0 + 4096)
        step = rng.standard_normal((r1 - r0, w.d), dtype=np.float32) * std
        out[r0:r1] = to_bf16_bits(from_bf16_bits(flat[r0:r1]) + step)
    return out.reshape(x_prev_bits.shape)


def sample_pairs(w, n, seed_tag=7):
    """Seeded (b, q-head) sample: always head 0 and the last head, and for GQA
    all query heads of one KV head; the rest drawn without replacement."""
    fixed = [(0, 0), (w.B - 1, w.Hq - 1)]
    g = w.Hq // w.Hkv
    if g > 1:
        fixed += [(0, g + j) for j in range(g)]
    allp = [(b, h) for b in range(w.B) for h in range(w.Hq)]
    rng = _rng(w.cfg_id, 10_000 + seed_tag)
    order = rng.permutation(len(allp))
    out = list(dict.fromkeys(fixed))
    for i in order:
        if len(out) >= n:
            break
        if allp[i] not in out:
            out.append(allp[i])
    return out[:max(n, len(fixed))]
