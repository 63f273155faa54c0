"""ctypes binding of libxquant.so: argument marshalling only.

Each function has the name and meaning of the C entry point declared in
include/xquant.h.  Tensors are torch CUDA (ROCm) tensors; the calls enqueue work on
torch's current stream and return without synchronising.  There is no fallback:
if the library is missing or a call fails, an exception is raised.
"""
import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

XQ_MAX_BATCH = 128
SYMBOLS = [
    "xq_status_string", "xq_version", "xq_codes_row_bytes", "xq_meta_row_elems",
    "xq_quantize_append", "xq_cl_delta_quantize", "xq_cl_accumulate",
    "xq_prepared_weights_bytes", "xq_prepare_weights",
    "xq_remat_attn_workspace_bytes", "xq_remat_attn_decode", "xq_remat_attn_decode_static",
    "xq_latent_project", "xq_prepare_weights_latent", "xq_remat_attn_decode_latent",
    "xq_remat_attn_decode_rope",
    "xq_prepared_weights_latent_bytes", "xq_remat_attn_latent_workspace_bytes",
    "xq_cl_latent_delta_project", "xq_cl_latent_delta_project_bulk", "xq_prepared_upproject_bytes", "xq_prepare_upproject",
    "xq_cl_accumulate_latent_workspace_bytes", "xq_cl_accumulate_latent",
    "xq_remat_attn_prefill_workspace_bytes", "xq_remat_attn_prefill",
    "xq_quantize_blocks_per_channel",
    "xq_remat_attn_per_channel_workspace_bytes", "xq_per_channel_terms_bytes", "xq_remat_attn_decode_per_channel",
    "xq_prepared_weights_pairs_bytes", "xq_prepare_weights_pairs",
    "xq_remat_attn_latent_per_channel_workspace_bytes", "xq_remat_attn_decode_latent_per_channel",
    "xq_prepared_projection_bytes", "xq_prepare_projection", "xq_latent_project_bulk",
]


class XQError(RuntimeError):
    pass


class _QFmt(C.Structure):
    _fields_ = [("d", C.c_int32), ("group", C.c_int32), ("bits", C.c_int32)]


class _Cache(C.Structure):
    _fields_ = [("codes", C.c_void_p), ("scale", C.c_void_p), ("zero", C.c_void_p),
                ("B", C.c_int32), ("cap", C.c_int32), ("fmt", _QFmt)]


class _Attn(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("softmax_scale", C.c_float)]


def lib_path():
    return os.path.join(_HERE, "libxquant.so")


def load_library():
    """Load the built library.  It is built first if it was never built or if its recorded source digest does
    not match the sources in the tree, so a stale library is never the one under test."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    from . import build as _build
    if _build.needs_build():
        _build.build(force=True)
    lib = C.CDLL(path)
    lib.xq_status_string.restype = C.c_char_p
    lib.xq_status_string.argtypes = [C.c_int]
    lib.xq_version.restype = C.c_int
    for name in ("xq_codes_row_bytes", "xq_meta_row_elems"):
        getattr(lib, name).restype = C.c_size_t
        getattr(lib, name).argtypes = [C.POINTER(_QFmt)]
    lib.xq_quantize_append.restype = C.c_int
    lib.xq_quantize_append.argtypes = [C.POINTER(_Cache), C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.c_void_p]
    lib.xq_cl_delta_quantize.restype = C.c_int
    lib.xq_cl_delta_quantize.argtypes = [C.POINTER(_Cache), C.c_void_p, C.c_void_p, C.c_int32,
                                         C.POINTER(C.c_int32), C.c_void_p]
    lib.xq_cl_accumulate.restype = C.c_int
    lib.xq_cl_accumulate.argtypes = [C.c_void_p, C.POINTER(_Cache), C.POINTER(C.c_int32), C.c_int32, C.c_void_p]
    lib.xq_prepared_weights_bytes.restype = C.c_size_t
    lib.xq_prepared_weights_bytes.argtypes = [C.POINTER(_Attn), C.c_int32, C.c_int32, C.c_int32]
    lib.xq_prepare_weights.restype = C.c_int
    lib.xq_prepare_weights.argtypes = [C.POINTER(_Attn), C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.xq_remat_attn_workspace_bytes.restype = C.c_size_t
    lib.xq_remat_attn_workspace_bytes.argtypes = [C.POINTER(_Attn), C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    lib.xq_remat_attn_decode.restype = C.c_int
    lib.xq_remat_attn_decode.argtypes = [C.POINTER(_Attn), C.c_void_p, C.POINTER(_Cache), C.c_void_p,
                                         C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                         C.POINTER(C.c_int32), C.c_void_p, C.c_void_p, C.c_size_t,
                                         C.c_void_p]
    lib.xq_remat_attn_decode_static.restype = C.c_int
    lib.xq_remat_attn_decode_static.argtypes = [C.POINTER(_Attn), C.c_void_p, C.POINTER(_Cache), C.c_void_p,
                                                C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                                C.POINTER(C.c_int32), C.c_void_p, C.c_void_p]
    lib.xq_remat_attn_decode_rope.restype = C.c_int
    lib.xq_remat_attn_decode_rope.argtypes = [C.POINTER(_Attn), C.c_void_p, C.POINTER(_Cache), C.c_void_p,
                                              C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                              C.POINTER(C.c_int32), C.c_void_p, C.c_int32, C.POINTER(C.c_int32),
                                              C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.xq_prepared_weights_latent_bytes.restype = C.c_size_t
    lib.xq_prepared_weights_latent_bytes.argtypes = [C.POINTER(_Attn), C.c_int32, C.c_int32, C.c_int32]
    lib.xq_remat_attn_latent_workspace_bytes.restype = C.c_size_t
    lib.xq_remat_attn_latent_workspace_bytes.argtypes = [C.POINTER(_Attn), C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    lib.xq_latent_project.restype = C.c_int
    lib.xq_latent_project.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                      C.c_void_p]
    lib.xq_prepare_weights_latent.restype = C.c_int
    lib.xq_prepare_weights_latent.argtypes = [C.POINTER(_Attn), C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.xq_remat_attn_decode_latent.restype = C.c_int
    lib.xq_remat_attn_decode_latent.argtypes = [C.POINTER(_Attn), C.c_void_p, C.POINTER(_Cache), C.c_void_p,
                                                C.POINTER(C.c_int32), C.c_void_p, C.c_void_p, C.c_size_t,
                                                C.c_void_p]
    lib.xq_cl_latent_delta_project_bulk.restype = C.c_int
    lib.xq_cl_latent_delta_project_bulk.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                                    C.POINTER(C.c_int32), C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.xq_cl_latent_delta_project.restype = C.c_int
    lib.xq_cl_latent_delta_project.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                               C.POINTER(C.c_int32), C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.xq_prepared_upproject_bytes.restype = C.c_size_t
    lib.xq_prepared_upproject_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    lib.xq_prepare_upproject.restype = C.c_int
    lib.xq_prepare_upproject.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                         C.c_size_t, C.c_void_p]
    lib.xq_cl_accumulate_latent_workspace_bytes.restype = C.c_size_t
    lib.xq_cl_accumulate_latent_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    lib.xq_cl_accumulate_latent.restype = C.c_int
    lib.xq_cl_accumulate_latent.argtypes = [C.c_void_p, C.POINTER(_Cache), C.c_int32, C.c_void_p,
                                            C.POINTER(C.c_int32), C.c_void_p, C.c_size_t, C.c_void_p]
    lib.xq_remat_attn_prefill_workspace_bytes.restype = C.c_size_t
    lib.xq_remat_attn_prefill_workspace_bytes.argtypes = [C.POINTER(_Attn), C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                                          C.c_int32]
    lib.xq_remat_attn_prefill.restype = C.c_int
    lib.xq_remat_attn_prefill.argtypes = [C.POINTER(_Attn), C.c_void_p, C.c_int32, C.POINTER(_Cache), C.c_void_p,
                                          C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.POINTER(C.c_int32),
                                          C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.c_void_p, C.c_void_p,
                                          C.c_size_t, C.c_void_p]
    lib.xq_quantize_blocks_per_channel.restype = C.c_int
    lib.xq_quantize_blocks_per_channel.argtypes = [C.POINTER(_Cache), C.c_void_p, C.c_int32, C.POINTER(C.c_int32),
                                                   C.c_void_p]
    lib.xq_remat_attn_per_channel_workspace_bytes.restype = C.c_size_t
    lib.xq_remat_attn_per_channel_workspace_bytes.argtypes = [C.POINTER(_Attn), C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    lib.xq_remat_attn_decode_per_channel.restype = C.c_int
    lib.xq_per_channel_terms_bytes.restype = C.c_size_t
    lib.xq_per_channel_terms_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    lib.xq_remat_attn_decode_per_channel.argtypes = [C.POINTER(_Attn), C.c_void_p, C.POINTER(_Cache), C.c_void_p,
                                                     C.POINTER(C.c_int32), C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                                     C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.xq_prepared_weights_pairs_bytes.restype = C.c_size_t
    lib.xq_prepared_weights_pairs_bytes.argtypes = [C.POINTER(_Attn), C.c_int32, C.c_int32, C.c_int32]
    lib.xq_prepare_weights_pairs.restype = C.c_int
    lib.xq_prepare_weights_pairs.argtypes = [C.POINTER(_Attn), C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                             C.c_size_t, C.c_void_p]
    lib.xq_remat_attn_latent_per_channel_workspace_bytes.restype = C.c_size_t
    lib.xq_remat_attn_latent_per_channel_workspace_bytes.argtypes = [C.POINTER(_Attn), C.c_int32, C.c_int32, C.c_int32,
                                                                     C.c_int32, C.c_int32]
    lib.xq_remat_attn_decode_latent_per_channel.restype = C.c_int
    lib.xq_remat_attn_decode_latent_per_channel.argtypes = [C.POINTER(_Attn), C.c_void_p, C.POINTER(_Cache), C.c_void_p,
                                                            C.POINTER(_Cache), C.c_void_p, C.c_void_p, C.c_void_p,
                                                            C.POINTER(C.c_int32), C.c_void_p, C.c_int64, C.c_void_p,
                                                            C.c_void_p, C.c_size_t, C.c_int32,
                                                            C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.xq_prepared_projection_bytes.restype = C.c_size_t
    lib.xq_prepared_projection_bytes.argtypes = [C.c_int32, C.c_int32]
    lib.xq_prepare_projection.restype = C.c_int
    lib.xq_prepare_projection.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.xq_latent_project_bulk.restype = C.c_int
    lib.xq_latent_project_bulk.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    _LIB = lib
    return lib


@dataclass
class XQCache:
    """Caller-owned quantised cache: codes u8 [B][cap][d*bits/8], scale/zero bf16 [B][cap][d/group]."""
    codes: torch.Tensor
    scale: torch.Tensor
    zero: torch.Tensor
    B: int
    cap: int
    d: int
    group: int
    bits: int

    def c_struct(self):
        return _Cache(self.codes.data_ptr(), self.scale.data_ptr(), self.zero.data_ptr(),
                      self.B, self.cap, _QFmt(self.d, self.group, self.bits))


@dataclass
class XQAttn:
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    softmax_scale: float

    def c_struct(self):
        return _Attn(self.n_q_heads, self.n_kv_heads, self.head_dim, self.softmax_scale)


def alloc_cache(B, cap, d, group, bits, device="cuda"):
    rb = d * bits // 8
    return XQCache(torch.zeros((B, cap, rb), dtype=torch.uint8, device=device),
                   torch.zeros((B, cap, d // group), dtype=torch.bfloat16, device=device),
                   torch.zeros((B, cap, d // group), dtype=torch.bfloat16, device=device),
                   B, cap, d, group, bits)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status, what):
    if status != 0:
        msg = load_library().xq_status_string(status).decode()
        raise XQError(f"{what}: {msg} ({status})")


def _i32(vals, n):
    vals = [int(v) for v in vals]
    if len(vals) != n:
        raise XQError(f"expected {n} per-sequence integers, got {len(vals)}")
    return (C.c_int32 * n)(*vals)


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def xq_version():
    return load_library().xq_version()


def xq_status_string(status):
    return load_library().xq_status_string(status).decode()


def xq_codes_row_bytes(d, group, bits):
    return load_library().xq_codes_row_bytes(C.byref(_QFmt(d, group, bits)))


def xq_meta_row_elems(d, group, bits):
    return load_library().xq_meta_row_elems(C.byref(_QFmt(d, group, bits)))


def xq_quantize_append(cache, x_bf16, start):
    """x_bf16 [B][T][d] bf16; rows start[b]..start[b]+T-1 of the cache are written."""
    assert x_bf16.dtype == torch.bfloat16 and x_bf16.is_contiguous() and x_bf16.dim() == 3
    T = x_bf16.shape[1]
    cs = cache.c_struct()
    _check(load_library().xq_quantize_append(C.byref(cs), _ptr(x_bf16), T, _i32(start, cache.B), _stream()),
           "xq_quantize_append")


def xq_cl_delta_quantize(delta, x_bf16, acc_bf16, start):
    assert x_bf16.dtype == torch.bfloat16 and x_bf16.is_contiguous() and x_bf16.dim() == 3
    assert acc_bf16.dtype == torch.bfloat16 and acc_bf16.is_contiguous()
    T = x_bf16.shape[1]
    cs = delta.c_struct()
    _check(load_library().xq_cl_delta_quantize(C.byref(cs), _ptr(x_bf16), _ptr(acc_bf16), T,
                                               _i32(start, delta.B), _stream()), "xq_cl_delta_quantize")


def xq_cl_accumulate(acc_bf16, src, lens, init):
    assert acc_bf16.dtype == torch.bfloat16 and acc_bf16.is_contiguous()
    cs = src.c_struct()
    _check(load_library().xq_cl_accumulate(_ptr(acc_bf16), C.byref(cs), _i32(lens, src.B),
                                           1 if init else 0, _stream()), "xq_cl_accumulate")


def xq_prepared_weights_bytes(attn, d, group, src_bits):
    a = attn.c_struct()
    return load_library().xq_prepared_weights_bytes(C.byref(a), d, group, src_bits)


def xq_prepare_weights(attn, d, group, src_bits, Wk, Wv, out=None):
    """Returns the prepared-weights buffer (uint8 tensor) for xq_remat_attn_decode."""
    assert Wk.dtype == torch.bfloat16 and Wv.dtype == torch.bfloat16
    assert Wk.is_contiguous() and Wv.is_contiguous()
    nbytes = xq_prepared_weights_bytes(attn, d, group, src_bits)
    if nbytes == 0:
        raise XQError("xq_prepare_weights: unsupported combination")
    if out is None:
        out = torch.empty(nbytes, dtype=torch.uint8, device=Wk.device)
    a = attn.c_struct()
    _check(load_library().xq_prepare_weights(C.byref(a), d, group, src_bits, _ptr(Wk), _ptr(Wv), _ptr(out),
                                             out.numel(), _stream()), "xq_prepare_weights")
    return out


def _walk_of(xcache, d):
    """(d, group) to size the attention workspace with: the cache's own, except that an 8-bit cache is walked as
    4-bit groups of 128 nibbles over twice the width; group 0 for the accumulator source."""
    if xcache is None:
        return d, 0
    return (2 * xcache.d, 128) if xcache.bits == 8 else (xcache.d, xcache.group)


def xq_remat_attn_workspace_bytes(attn, B, max_len, d, group):
    """group = the X cache's group size, or 0 when the bf16 accumulator is the source."""
    a = attn.c_struct()
    return load_library().xq_remat_attn_workspace_bytes(C.byref(a), B, max_len, d, group)


def xq_remat_attn_decode(attn, q_bf16, wprep, lens, *, xcache=None, acc_bf16=None, out=None, workspace=None,
                         rope_cos_sin=None, pos0=None):
    """Attention output fp32 [B][Hq][head_dim] over the first lens[b] cached rows.  With rope_cos_sin
    (fp32 [n_pos][head_dim/2][2]) the call is xq_remat_attn_decode_rope: keys rotated, row t of sequence b
    at position pos0[b] + t."""
    assert q_bf16.dtype == torch.bfloat16 and q_bf16.is_contiguous()
    if xcache is not None:
        B, cap, d = xcache.B, xcache.cap, xcache.d
        cs = xcache.c_struct()
        cptr = C.byref(cs)
    else:
        assert acc_bf16.dtype == torch.bfloat16 and acc_bf16.is_contiguous() and acc_bf16.dim() == 3
        B, cap, d = acc_bf16.shape
        cptr = None
    lens = [int(v) for v in lens]
    a = attn.c_struct()
    need = xq_remat_attn_workspace_bytes(attn, B, max(lens) if lens else 1, *_walk_of(xcache, d))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q_bf16.device)
    if out is None:
        out = torch.empty((B, attn.n_q_heads, attn.head_dim), dtype=torch.float32, device=q_bf16.device)
    if rope_cos_sin is not None:
        assert rope_cos_sin.dtype == torch.float32 and rope_cos_sin.is_contiguous() and rope_cos_sin.dim() == 3
        pos0 = [0] * B if pos0 is None else pos0
        _check(load_library().xq_remat_attn_decode_rope(C.byref(a), _ptr(q_bf16), cptr, _ptr(acc_bf16), B, cap, d,
                                                        _ptr(wprep), _i32(lens, B), _ptr(rope_cos_sin),
                                                        rope_cos_sin.shape[0], _i32(pos0, B), _ptr(out),
                                                        _ptr(workspace), workspace.numel(), _stream()),
               "xq_remat_attn_decode_rope")
        return out
    _check(load_library().xq_remat_attn_decode(C.byref(a), _ptr(q_bf16), cptr, _ptr(acc_bf16), B, cap, d,
                                               _ptr(wprep), _i32(lens, B), _ptr(out), _ptr(workspace),
                                               workspace.numel(), _stream()), "xq_remat_attn_decode")
    return out


XQ_STATIC_SCRATCH_BYTES = 32 << 20


def xq_remat_attn_decode_static(attn, q_bf16, wprep, lens, *, xcache=None, acc_bf16=None, out):
    """xq_remat_attn_decode with the library's built-in workspace: the call allocates nothing, so `out` is
    the caller's (fp32 [B][Hq][head_dim])."""
    assert q_bf16.dtype == torch.bfloat16 and q_bf16.is_contiguous()
    assert out.dtype == torch.float32 and out.is_contiguous()
    if xcache is not None:
        B, cap, d = xcache.B, xcache.cap, xcache.d
        cs = xcache.c_struct()
        cptr = C.byref(cs)
    else:
        assert acc_bf16.dtype == torch.bfloat16 and acc_bf16.is_contiguous() and acc_bf16.dim() == 3
        B, cap, d = acc_bf16.shape
        cptr = None
    a = attn.c_struct()
    _check(load_library().xq_remat_attn_decode_static(C.byref(a), _ptr(q_bf16), cptr, _ptr(acc_bf16), B, cap, d,
                                                      _ptr(wprep), _i32([int(v) for v in lens], B), _ptr(out),
                                                      _stream()), "xq_remat_attn_decode_static")
    return out


def xq_prepared_weights_latent_bytes(attn, r, group, src_bits):
    a = attn.c_struct()
    return load_library().xq_prepared_weights_latent_bytes(C.byref(a), r, group, src_bits)


def xq_remat_attn_latent_workspace_bytes(attn, B, max_len, r, group):
    a = attn.c_struct()
    return load_library().xq_remat_attn_latent_workspace_bytes(C.byref(a), B, max_len, r, group)


def xq_latent_project(x_bf16, Ut_bf16, out=None):
    """x [..., d] bf16 times U (given transposed, [n_lat][d]) -> [..., n_lat] bf16."""
    assert x_bf16.dtype == torch.bfloat16 and x_bf16.is_contiguous()
    assert Ut_bf16.dtype == torch.bfloat16 and Ut_bf16.is_contiguous() and Ut_bf16.dim() == 2
    d = x_bf16.shape[-1]
    n_lat = Ut_bf16.shape[0]
    assert Ut_bf16.shape[1] == d
    M = x_bf16.numel() // d
    if out is None:
        out = torch.empty((*x_bf16.shape[:-1], n_lat), dtype=torch.bfloat16, device=x_bf16.device)
    _check(load_library().xq_latent_project(_ptr(x_bf16), _ptr(Ut_bf16), M, d, n_lat, _ptr(out), _stream()),
           "xq_latent_project")
    return out


def xq_prepare_weights_latent(attn, r, group, src_bits, Wfk, Wfv, out=None):
    """Prepared stream for a latent cache [X Uk | X Uv]; Wfk, Wfv [r][Hkv*hd] = S B^T of the two SVDs."""
    assert Wfk.dtype == torch.bfloat16 and Wfv.dtype == torch.bfloat16
    assert Wfk.is_contiguous() and Wfv.is_contiguous()
    nbytes = xq_prepared_weights_latent_bytes(attn, r, group, src_bits)
    if nbytes == 0:
        raise XQError("xq_prepare_weights_latent: unsupported combination")
    if out is None:
        out = torch.empty(nbytes, dtype=torch.uint8, device=Wfk.device)
    a = attn.c_struct()
    _check(load_library().xq_prepare_weights_latent(C.byref(a), r, group, src_bits, _ptr(Wfk), _ptr(Wfv), _ptr(out),
                                                    out.numel(), _stream()), "xq_prepare_weights_latent")
    return out


def xq_remat_attn_decode_latent(attn, q_bf16, wprep, lens, latent, out=None, workspace=None):
    """As xq_remat_attn_decode for a latent cache (fmt.d = 2r) and a stream from xq_prepare_weights_latent."""
    assert q_bf16.dtype == torch.bfloat16 and q_bf16.is_contiguous()
    lens = [int(v) for v in lens]
    a = attn.c_struct()
    cs = latent.c_struct()
    need = xq_remat_attn_latent_workspace_bytes(attn, latent.B, max(lens) if lens else 1, latent.d // 2, latent.group)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q_bf16.device)
    if out is None:
        out = torch.empty((latent.B, attn.n_q_heads, attn.head_dim), dtype=torch.float32, device=q_bf16.device)
    _check(load_library().xq_remat_attn_decode_latent(C.byref(a), _ptr(q_bf16), C.byref(cs), _ptr(wprep),
                                                      _i32(lens, latent.B), _ptr(out), _ptr(workspace),
                                                      workspace.numel(), _stream()), "xq_remat_attn_decode_latent")
    return out


def xq_cl_latent_delta_project(x_bf16, acc_bf16, Ut_bf16, start, out=None):
    """(x - acc rows start[b]+t) U_kv for x [B][T][d], acc [B][cap][d], Ut = U_kv transposed [n_lat][d]
    -> [B][T][n_lat] bf16."""
    for t in (x_bf16, acc_bf16, Ut_bf16):
        assert t.dtype == torch.bfloat16 and t.is_contiguous()
    B, T, d = x_bf16.shape
    assert acc_bf16.dim() == 3 and acc_bf16.shape[0] == B and acc_bf16.shape[2] == d
    n_lat = Ut_bf16.shape[0]
    assert Ut_bf16.shape[1] == d
    if out is None:
        out = torch.empty((B, T, n_lat), dtype=torch.bfloat16, device=x_bf16.device)
    _check(load_library().xq_cl_latent_delta_project(_ptr(x_bf16), _ptr(acc_bf16), _ptr(Ut_bf16), B, T,
                                                     acc_bf16.shape[1], _i32(start, B), d, n_lat, _ptr(out),
                                                     _stream()), "xq_cl_latent_delta_project")
    return out


def xq_cl_latent_delta_project_bulk(x_bf16, acc_bf16, proj, n_lat, start, out=None):
    """The same for prefill-sized T, on the matrix cores; proj = xq_prepare_projection(Ut)."""
    for t in (x_bf16, acc_bf16):
        assert t.dtype == torch.bfloat16 and t.is_contiguous()
    B, T, d = x_bf16.shape
    assert acc_bf16.dim() == 3 and acc_bf16.shape[0] == B and acc_bf16.shape[2] == d
    if out is None:
        out = torch.empty((B, T, n_lat), dtype=torch.bfloat16, device=x_bf16.device)
    _check(load_library().xq_cl_latent_delta_project_bulk(_ptr(x_bf16), _ptr(acc_bf16), _ptr(proj), B, T,
                                                          acc_bf16.shape[1], _i32(start, B), d, n_lat, _ptr(out),
                                                          _stream()), "xq_cl_latent_delta_project_bulk")
    return out


def xq_prepared_upproject_bytes(d, n_lat, group, src_bits):
    return load_library().xq_prepared_upproject_bytes(d, n_lat, group, src_bits)


def xq_prepare_upproject(d, group, src_bits, Ut_bf16, out=None):
    """Prepared stream of U_kv^T (Ut [n_lat][d] bf16) for xq_cl_accumulate_latent."""
    assert Ut_bf16.dtype == torch.bfloat16 and Ut_bf16.is_contiguous() and Ut_bf16.shape[1] == d
    n_lat = Ut_bf16.shape[0]
    nbytes = xq_prepared_upproject_bytes(d, n_lat, group, src_bits)
    if nbytes == 0:
        raise XQError("xq_prepare_upproject: unsupported combination")
    if out is None:
        out = torch.empty(nbytes, dtype=torch.uint8, device=Ut_bf16.device)
    _check(load_library().xq_prepare_upproject(d, n_lat, group, src_bits, _ptr(Ut_bf16), _ptr(out), out.numel(),
                                               _stream()), "xq_prepare_upproject")
    return out


def xq_cl_accumulate_latent_workspace_bytes(B, max_len, n_lat, group):
    return load_library().xq_cl_accumulate_latent_workspace_bytes(B, max_len, n_lat, group)


def xq_cl_accumulate_latent(acc_bf16, delta, uprep, lens, workspace=None):
    """acc [B][cap][d] += dequant(delta cache, fmt.d = n_lat) U_kv^T on rows t < lens[b], in place."""
    assert acc_bf16.dtype == torch.bfloat16 and acc_bf16.is_contiguous() and acc_bf16.dim() == 3
    assert acc_bf16.shape[0] == delta.B and acc_bf16.shape[1] == delta.cap
    lens = [int(v) for v in lens]
    cs = delta.c_struct()
    need = xq_cl_accumulate_latent_workspace_bytes(delta.B, max(max(lens), 1) if lens else 1, delta.d, delta.group)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=acc_bf16.device)
    _check(load_library().xq_cl_accumulate_latent(_ptr(acc_bf16), C.byref(cs), acc_bf16.shape[2], _ptr(uprep),
                                                  _i32(lens, delta.B), _ptr(workspace), workspace.numel(),
                                                  _stream()), "xq_cl_accumulate_latent")


def xq_remat_attn_prefill_workspace_bytes(attn, B, T, max_len, d, group):
    a = attn.c_struct()
    return load_library().xq_remat_attn_prefill_workspace_bytes(C.byref(a), B, T, max_len, d, group)


def xq_remat_attn_prefill(attn, q_bf16, wprep, lens, *, xcache=None, acc_bf16=None, out=None, workspace=None,
                          rope_cos_sin=None, pos0=None):
    """Causal attention of the T newest cache rows of every sequence: q [B][T][Hq][head_dim] bf16 ->
    fp32 [B][T][Hq][head_dim]; lens[b] counts the valid rows including the T new ones."""
    assert q_bf16.dtype == torch.bfloat16 and q_bf16.is_contiguous() and q_bf16.dim() == 4
    T = q_bf16.shape[1]
    if xcache is not None:
        B, cap, d = xcache.B, xcache.cap, xcache.d
        cs = xcache.c_struct()
        cptr = C.byref(cs)
    else:
        assert acc_bf16.dtype == torch.bfloat16 and acc_bf16.is_contiguous() and acc_bf16.dim() == 3
        B, cap, d = acc_bf16.shape
        cptr = None
    lens = [int(v) for v in lens]
    a = attn.c_struct()
    need = xq_remat_attn_prefill_workspace_bytes(attn, B, T, max(lens) if lens else 1, *_walk_of(xcache, d))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q_bf16.device)
    if out is None:
        out = torch.empty((B, T, attn.n_q_heads, attn.head_dim), dtype=torch.float32, device=q_bf16.device)
    rope_ptr, n_pos, p0 = None, 0, None
    if rope_cos_sin is not None:
        assert rope_cos_sin.dtype == torch.float32 and rope_cos_sin.is_contiguous() and rope_cos_sin.dim() == 3
        rope_ptr, n_pos = _ptr(rope_cos_sin), rope_cos_sin.shape[0]
        p0 = _i32([0] * B if pos0 is None else pos0, B)
    _check(load_library().xq_remat_attn_prefill(C.byref(a), _ptr(q_bf16), T, cptr, _ptr(acc_bf16), B, cap, d,
                                                _ptr(wprep), _i32(lens, B), rope_ptr, n_pos, p0, _ptr(out),
                                                _ptr(workspace), workspace.numel(), _stream()),
           "xq_remat_attn_prefill")
    return out


def alloc_cache_per_channel(B, cap, d, group, bits, device="cuda"):
    """Per-channel cache: codes as alloc_cache, scale / zero [B][cap/group][d]."""
    assert cap % group == 0
    return XQCache(torch.zeros((B, cap, d * bits // 8), dtype=torch.uint8, device=device),
                   torch.zeros((B, cap // group, d), dtype=torch.bfloat16, device=device),
                   torch.zeros((B, cap // group, d), dtype=torch.bfloat16, device=device),
                   B, cap, d, group, bits)


def xq_quantize_blocks_per_channel(cache, x_bf16, block0):
    """x [B][nblk*group][d] bf16 -> blocks block0[b] .. of the per-channel cache."""
    assert x_bf16.dtype == torch.bfloat16 and x_bf16.is_contiguous() and x_bf16.dim() == 3
    assert x_bf16.shape[0] == cache.B and x_bf16.shape[2] == cache.d and x_bf16.shape[1] % cache.group == 0
    cs = cache.c_struct()
    _check(load_library().xq_quantize_blocks_per_channel(C.byref(cs), _ptr(x_bf16), x_bf16.shape[1] // cache.group,
                                                         _i32(block0, cache.B), _stream()),
           "xq_quantize_blocks_per_channel")


def xq_remat_attn_per_channel_workspace_bytes(attn, B, max_len, d, group):
    a = attn.c_struct()
    return load_library().xq_remat_attn_per_channel_workspace_bytes(C.byref(a), B, max_len, d, group)


def xq_per_channel_terms_bytes(B, cap, d, group, col_blocks):
    return load_library().xq_per_channel_terms_bytes(B, cap, d, group, col_blocks)


def alloc_per_channel_terms(cache, col_blocks):
    """A buffer for the per-block terms of `cache` (col_blocks = n_kv_heads, or n_kv_heads / 2 for the latent
    variant); pass it as `terms` with terms_valid=False after a block was completed, True otherwise."""
    n = xq_per_channel_terms_bytes(cache.B, cache.cap, cache.d, cache.group, col_blocks)
    if n == 0:
        raise XQError("xq_per_channel_terms_bytes: unsupported combination")
    return torch.empty(n, dtype=torch.uint8, device=cache.codes.device)


def _terms_args(terms):
    if terms is None:
        return None, 0
    assert terms.dtype == torch.uint8 and terms.is_contiguous()
    return _ptr(terms), terms.numel()


def xq_remat_attn_decode_per_channel(attn, q_bf16, cache, tail_bf16, lens, wprep_coded, wprep_dense, out=None,
                                     workspace=None, terms=None, terms_valid=False):
    """Decode attention from a per-channel cache plus the bf16 residual window [B][group][d]."""
    assert q_bf16.dtype == torch.bfloat16 and q_bf16.is_contiguous()
    assert tail_bf16.dtype == torch.bfloat16 and tail_bf16.is_contiguous()
    assert tuple(tail_bf16.shape) == (cache.B, cache.group, cache.d)
    lens = [int(v) for v in lens]
    a = attn.c_struct()
    cs = cache.c_struct()
    need = xq_remat_attn_per_channel_workspace_bytes(attn, cache.B, max(lens) if lens else 1, cache.d, cache.group)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q_bf16.device)
    if out is None:
        out = torch.empty((cache.B, attn.n_q_heads, attn.head_dim), dtype=torch.float32, device=q_bf16.device)
    _check(load_library().xq_remat_attn_decode_per_channel(C.byref(a), _ptr(q_bf16), C.byref(cs), _ptr(tail_bf16),
                                                           _i32(lens, cache.B), _ptr(wprep_coded), _ptr(wprep_dense),
                                                           *_terms_args(terms), int(bool(terms_valid)),
                                                           _ptr(out), _ptr(workspace), workspace.numel(), _stream()),
           "xq_remat_attn_decode_per_channel")
    return out


def xq_prepared_weights_pairs_bytes(attn, r, group, src_bits):
    a = attn.c_struct()
    return load_library().xq_prepared_weights_pairs_bytes(C.byref(a), r, group, src_bits)


def xq_prepare_weights_pairs(attn, r, group, src_bits, Wf, out=None):
    """Prepared stream of one fused latent matrix Wf [r][Hkv*hd] bf16 with a pair of KV heads per "head"."""
    assert Wf.dtype == torch.bfloat16 and Wf.is_contiguous()
    nbytes = xq_prepared_weights_pairs_bytes(attn, r, group, src_bits)
    if nbytes == 0:
        raise XQError("xq_prepare_weights_pairs: unsupported combination")
    if out is None:
        out = torch.empty(nbytes, dtype=torch.uint8, device=Wf.device)
    a = attn.c_struct()
    _check(load_library().xq_prepare_weights_pairs(C.byref(a), r, group, src_bits, _ptr(Wf), _ptr(out), out.numel(),
                                                   _stream()), "xq_prepare_weights_pairs")
    return out


def xq_remat_attn_latent_per_channel_workspace_bytes(attn, B, max_len, r, k_group, v_group):
    a = attn.c_struct()
    return load_library().xq_remat_attn_latent_per_channel_workspace_bytes(C.byref(a), B, max_len, r, k_group, v_group)


def xq_remat_attn_decode_latent_per_channel(attn, q_bf16, kcache, ktail_bf16, vcache, wk_coded, wk_dense, wv_coded, lens,
                                            out=None, workspace=None, terms=None, terms_valid=False, k0_f16=None,
                                            wk_row0=None):
    """Decode attention from a per-channel X Uk cache (+ bf16 window) and a per-token X Uv cache (Sec. 3.3.1).
    k0_f16 [B][stride] float16 with wk_row0 [Hkv*hd] bfloat16: the outlier channel of X Uk kept in fp16 (App. B)."""
    k0_stride = 0
    if k0_f16 is not None:
        assert k0_f16.dtype == torch.float16 and k0_f16.is_contiguous() and k0_f16.dim() == 2 and k0_f16.shape[0] == kcache.B
        assert wk_row0 is not None and wk_row0.dtype == torch.bfloat16 and wk_row0.is_contiguous()
        assert wk_row0.numel() == attn.n_kv_heads * attn.head_dim
        k0_stride = k0_f16.shape[1]
    assert q_bf16.dtype == torch.bfloat16 and q_bf16.is_contiguous()
    assert ktail_bf16.dtype == torch.bfloat16 and ktail_bf16.is_contiguous()
    assert tuple(ktail_bf16.shape) == (kcache.B, kcache.group, kcache.d)
    lens = [int(v) for v in lens]
    a = attn.c_struct()
    ks, vs = kcache.c_struct(), vcache.c_struct()
    need = xq_remat_attn_latent_per_channel_workspace_bytes(attn, kcache.B, max(lens) if lens else 1, kcache.d,
                                                            kcache.group, vcache.group)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q_bf16.device)
    if out is None:
        out = torch.empty((kcache.B, attn.n_q_heads, attn.head_dim), dtype=torch.float32, device=q_bf16.device)
    _check(load_library().xq_remat_attn_decode_latent_per_channel(
        C.byref(a), _ptr(q_bf16), C.byref(ks), _ptr(ktail_bf16), C.byref(vs), _ptr(wk_coded), _ptr(wk_dense),
        _ptr(wv_coded), _i32(lens, kcache.B), _ptr(k0_f16), k0_stride, _ptr(wk_row0), *_terms_args(terms),
        int(bool(terms_valid)), _ptr(out), _ptr(workspace),
        workspace.numel(), _stream()),
        "xq_remat_attn_decode_latent_per_channel")
    return out


def xq_prepare_projection(Ut_bf16, out=None):
    """Prepared stream of U (given transposed, [n_lat][d] bf16) for xq_latent_project_bulk."""
    assert Ut_bf16.dtype == torch.bfloat16 and Ut_bf16.is_contiguous() and Ut_bf16.dim() == 2
    n_lat, d = Ut_bf16.shape
    nbytes = load_library().xq_prepared_projection_bytes(d, n_lat)
    if nbytes == 0:
        raise XQError("xq_prepare_projection: unsupported shape")
    if out is None:
        out = torch.empty(nbytes, dtype=torch.uint8, device=Ut_bf16.device)
    _check(load_library().xq_prepare_projection(d, n_lat, _ptr(Ut_bf16), _ptr(out), out.numel(), _stream()),
           "xq_prepare_projection")
    return out


def xq_latent_project_bulk(x_bf16, proj, n_lat, out=None):
    """x [..., d] bf16 times U through the matrix cores -> [..., n_lat] bf16 (proj from xq_prepare_projection)."""
    assert x_bf16.dtype == torch.bfloat16 and x_bf16.is_contiguous()
    d = x_bf16.shape[-1]
    M = x_bf16.numel() // d
    if out is None:
        out = torch.empty((*x_bf16.shape[:-1], n_lat), dtype=torch.bfloat16, device=x_bf16.device)
    _check(load_library().xq_latent_project_bulk(_ptr(x_bf16), _ptr(proj), M, d, n_lat, _ptr(out), _stream()),
           "xq_latent_project_bulk")
    return out
