"""CPU checks of the C-ABI library: it loads, exports every symbol the header
declares, and rejects bad arguments on the host without touching a GPU."""
import ctypes as C
import os
import re

import pytest

import paper_2508_10395_amd as xq
from paper_2508_10395_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "xquant.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(xq_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = xq.load_library()
    declared = _declared_symbols()
    assert len(declared) >= 11
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(B.SYMBOLS) == declared
    assert xq.xq_version() >= 100
    assert xq.xq_status_string(0) == "ok" and "argument" in xq.xq_status_string(-1)


def test_format_queries():
    assert xq.xq_codes_row_bytes(4096, 128, 3) == 1536
    assert xq.xq_codes_row_bytes(4096, 64, 2) == 1024
    assert xq.xq_meta_row_elems(4096, 64, 2) == 64
    assert xq.xq_meta_row_elems(4096, 100, 2) == 0
    a = xq.XQAttn(32, 32, 128, 0.1)
    assert xq.xq_remat_attn_workspace_bytes(a, 8, 4096, 4096, 0) == 8 * 32 * 128 * 130 * 4
    assert xq.xq_remat_attn_workspace_bytes(a, 8, 4097, 4096, 0) == 8 * 32 * 136 * 130 * 4
    assert xq.xq_remat_attn_workspace_bytes(a, 8, 4096, 4096, 128) == 8 * 32 * 128 * 130 * 4 + 8 * 16 * 33 * 512
    assert xq.xq_remat_attn_workspace_bytes(a, 8, 4096, 4096, 32) == 0
    assert xq.xq_prepared_weights_bytes(a, 4096, 128, 3) > 2 * 4096 * 4096 * 2
    assert xq.xq_prepared_weights_bytes(a, 4096, 128, 5) == 0
    assert xq.xq_prepared_weights_bytes(xq.XQAttn(32, 32, 64, 0.1), 4096, 128, 3) == 0


def _cache(codes=16, scale=16, zero=16, B_=1, cap=8, d=256, group=128, bits=4):
    return B._Cache(codes, scale, zero, B_, cap, B._QFmt(d, group, bits))


def test_argument_errors_are_reported_before_any_launch():
    lib = xq.load_library()
    one = (C.c_int32 * 1)(0)
    x = C.c_void_p(32)
    st = C.c_void_p(0)
    INVALID, UNSUPPORTED, WORKSPACE = -1, -2, -3
    assert lib.xq_quantize_append(None, x, 1, one, st) == INVALID
    assert lib.xq_quantize_append(C.byref(_cache(codes=0)), x, 1, one, st) == INVALID
    assert lib.xq_quantize_append(C.byref(_cache(codes=8)), x, 1, one, st) == INVALID          # misaligned
    assert lib.xq_quantize_append(C.byref(_cache()), None, 1, one, st) == INVALID
    assert lib.xq_quantize_append(C.byref(_cache()), x, -1, one, st) == INVALID
    assert lib.xq_quantize_append(C.byref(_cache()), x, 9, one, st) == INVALID                 # start+T > cap
    assert lib.xq_quantize_append(C.byref(_cache()), x, 1, (C.c_int32 * 1)(8), st) == INVALID
    assert lib.xq_quantize_append(C.byref(_cache(bits=5)), x, 1, one, st) == UNSUPPORTED
    assert lib.xq_quantize_append(C.byref(_cache(group=32)), x, 1, one, st) == UNSUPPORTED
    assert lib.xq_quantize_append(C.byref(_cache(d=200, group=100)), x, 1, one, st) == UNSUPPORTED
    assert lib.xq_quantize_append(C.byref(_cache(d=200)), x, 1, one, st) == INVALID            # group does not divide d
    assert lib.xq_quantize_append(C.byref(_cache(B_=129)), x, 1, one, st) == UNSUPPORTED
    assert lib.xq_quantize_append(C.byref(_cache()), x, 0, one, st) == 0                       # T = 0: no-op
    assert lib.xq_quantize_append(C.byref(_cache()), None, 0, one, st) == 0
    assert lib.xq_cl_delta_quantize(C.byref(_cache()), x, None, 1, one, st) == INVALID
    assert lib.xq_cl_accumulate(None, C.byref(_cache()), one, 0, st) == INVALID
    assert lib.xq_cl_accumulate(x, C.byref(_cache()), (C.c_int32 * 1)(9), 0, st) == INVALID    # len > cap
    assert lib.xq_cl_accumulate(x, C.byref(_cache()), (C.c_int32 * 1)(0), 0, st) == 0          # nothing to do

    a = B._Attn(4, 2, 128, 0.1)
    bad_hd = B._Attn(4, 2, 64, 0.1)
    bad_ratio = B._Attn(5, 2, 128, 0.1)
    assert lib.xq_prepare_weights(C.byref(bad_hd), 256, 128, 4, x, x, x, 1 << 30, st) == UNSUPPORTED
    assert lib.xq_prepare_weights(C.byref(bad_ratio), 256, 128, 4, x, x, x, 1 << 30, st) == INVALID
    assert lib.xq_prepare_weights(C.byref(a), 256, 128, 5, x, x, x, 1 << 30, st) == UNSUPPORTED
    assert lib.xq_prepare_weights(C.byref(a), 256, 128, 8, x, x, x, 16, st) == WORKSPACE     # 8-bit caches are served
    assert lib.xq_prepare_weights(C.byref(a), 256, 128, 4, x, x, x, 16, st) == WORKSPACE
    cache = _cache()
    ok_len = (C.c_int32 * 1)(8)
    args = lambda **kw: dict(dict(a=C.byref(a), q=x, xc=C.byref(cache), acc=None, B=1, cap=8, d=256, w=x,
                                  len=ok_len, out=x, ws=x, wsb=1 << 30), **kw)

    def call(**kw):
        k = args(**kw)
        return lib.xq_remat_attn_decode(k["a"], k["q"], k["xc"], k["acc"], k["B"], k["cap"], k["d"], k["w"],
                                        k["len"], k["out"], k["ws"], k["wsb"], st)

    assert call(acc=x) == INVALID                       # both sources given
    assert call(xc=None) == INVALID                     # no source
    assert call(len=(C.c_int32 * 1)(0)) == INVALID      # empty sequence
    assert call(len=(C.c_int32 * 1)(9)) == INVALID      # longer than the cache
    assert call(wsb=64) == WORKSPACE
    assert call(xc=C.byref(_cache(bits=8)), wsb=64) == WORKSPACE      # 8-bit caches are served (walked nibble by nibble)
    assert call(xc=C.byref(_cache(bits=5))) == UNSUPPORTED
    assert call(a=C.byref(bad_hd)) == UNSUPPORTED
    assert call(out=None) == INVALID


def test_argument_errors_of_the_widened_entry_points():
    """Latent cache, cross-layer GQA and prefill entry points: every host-side check fires before a launch."""
    lib = xq.load_library()
    x = C.c_void_p(32)
    st = C.c_void_p(0)
    one = (C.c_int32 * 1)(0)
    INVALID, UNSUPPORTED, WORKSPACE = -1, -2, -3
    a = B._Attn(4, 2, 128, 0.1)
    # prefill: T rows must exist, B*T bounded, workspace checked, size query
    cache = _cache()
    pre = lambda T, ln, wsb=1 << 30, xc=cache: lib.xq_remat_attn_prefill(
        C.byref(a), x, T, C.byref(xc), None, 1, 8, 256, x, (C.c_int32 * 1)(ln), None, 0, None, x, x, wsb, st)
    assert pre(0, 8) == INVALID
    assert pre(5, 4) == INVALID                         # fewer rows than queries
    assert pre(2, 9) == INVALID                         # longer than the cache
    assert pre(2, 8, wsb=64) == WORKSPACE
    assert pre(2, 8, xc=_cache(bits=8), wsb=64) == WORKSPACE
    assert lib.xq_remat_attn_prefill(C.byref(a), x, 2, C.byref(cache), None, 1, 8, 256, x, (C.c_int32 * 1)(8), x, 4,
                                     None, x, x, 1 << 30, st) == INVALID        # table without positions
    at = xq.XQAttn(4, 2, 128, 0.1)
    assert xq.xq_remat_attn_prefill_workspace_bytes(at, 2, 3, 257, 256, 0) == 2 * 3 * 4 * 2 * 130 * 4
    assert xq.xq_remat_attn_prefill_workspace_bytes(at, 2, 0, 257, 256, 0) == 0
    # latent projection and its cross-layer variant
    assert lib.xq_latent_project(x, x, 4, 200, 64, x, st) == UNSUPPORTED
    assert lib.xq_latent_project(x, x, -1, 256, 64, x, st) == INVALID
    assert lib.xq_latent_project(None, x, 0, 256, 64, x, st) == 0               # no rows: nothing is read
    assert xq.load_library().xq_prepared_projection_bytes(4096, 2048) == 4096 * 2048 * 2
    assert xq.load_library().xq_prepared_projection_bytes(4096, 2048 + 128) == 0             # n_lat not a multiple of 256
    assert lib.xq_prepare_projection(512, 256, x, x, 16, st) == WORKSPACE
    assert lib.xq_prepare_projection(512, 200, x, x, 1 << 30, st) == UNSUPPORTED
    assert lib.xq_latent_project_bulk(x, x, 0, 512, 256, x, st) == 0
    assert lib.xq_latent_project_bulk(None, x, 4, 512, 256, x, st) == INVALID
    assert lib.xq_latent_project_bulk(x, x, 1 << 22, 4096, 256, x, st) == UNSUPPORTED        # rows beyond 32-bit byte offsets
    dp = lambda **kw: lib.xq_cl_latent_delta_project(*[dict(dict(x=x, acc=x, ut=x, B=1, T=1, cap=8, start=one, d=256,
                                                                 n=64, out=x, st=st), **kw)[k]
                                                       for k in ("x", "acc", "ut", "B", "T", "cap", "start", "d", "n", "out", "st")])
    assert dp(acc=None) == INVALID
    assert dp(start=(C.c_int32 * 1)(8)) == INVALID      # start + T > cap
    assert dp(d=200) == UNSUPPORTED
    assert dp(n=48) == UNSUPPORTED
    assert dp(T=0, x=None) == 0
    dpb = lambda **kw: lib.xq_cl_latent_delta_project_bulk(*[dict(dict(x=x, acc=x, proj=x, B=1, T=1, cap=8, start=one, d=256,
                                                                       n=256, out=x, st=st), **kw)[k]
                                                             for k in ("x", "acc", "proj", "B", "T", "cap", "start", "d", "n", "out", "st")])
    assert dpb(acc=None) == INVALID
    assert dpb(start=(C.c_int32 * 1)(8)) == INVALID     # start + T > cap
    assert dpb(n=64) == UNSUPPORTED                     # the matrix-core route needs whole 256-column blocks
    assert dpb(cap=1 << 21, d=4096) == UNSUPPORTED      # accumulator beyond 32-bit byte offsets
    assert dpb(T=0, x=None) == 0
    # up-projection stream and accumulate
    assert xq.xq_prepared_upproject_bytes(4096, 2048, 64, 2) > 2048 * 4096 * 2
    assert xq.xq_prepared_upproject_bytes(4096 + 128, 2048, 64, 2) == 0         # d not a multiple of 256
    assert xq.xq_prepared_upproject_bytes(4096, 2048, 64, 16) == 0
    assert lib.xq_prepare_upproject(512, 256, 128, 3, x, x, 16, st) == WORKSPACE
    assert lib.xq_prepare_upproject(512, 256, 128, 3, None, x, 1 << 30, st) == INVALID
    lat = _cache(d=256, group=128, bits=3)
    acc_lat = lambda ln, d=512, ws=x, wsb=1 << 30: lib.xq_cl_accumulate_latent(x, C.byref(lat), d, x, (C.c_int32 * 1)(ln),
                                                                                ws, wsb, st)
    assert acc_lat(9) == INVALID
    assert acc_lat(0) == 0                              # nothing to do
    assert acc_lat(8, d=384) == UNSUPPORTED
    assert acc_lat(8, wsb=16) == WORKSPACE
    assert acc_lat(8, ws=None) == INVALID
    assert xq.xq_cl_accumulate_latent_workspace_bytes(2, 300, 256, 128) == 2 * 2 * 3 * 256 * 2
    # latent attention
    la = B._Attn(4, 2, 128, 0.1)
    lc = _cache(d=512, group=128, bits=3)
    lat_call = lambda attn=la, c=lc, ln=8, wsb=1 << 30: lib.xq_remat_attn_decode_latent(
        C.byref(attn), x, C.byref(c), x, (C.c_int32 * 1)(ln), x, x, wsb, st)
    assert lat_call(ln=0) == INVALID
    assert lat_call(wsb=16) == WORKSPACE
    assert lat_call(attn=B._Attn(3, 3, 128, 0.1), c=_cache(d=768, group=128, bits=3)) == UNSUPPORTED   # odd number of KV heads
    assert lat_call(c=_cache(d=384, group=128, bits=3)) == UNSUPPORTED          # latent width not a multiple of 256
    # one sequence's rows are addressed with 32-bit byte offsets
    assert lib.xq_remat_attn_decode(C.byref(la), x, None, x, 1, 1 << 20, 4096, x, (C.c_int32 * 1)(8), x, x, 1 << 30, st) == UNSUPPORTED
    assert lib.xq_remat_attn_decode(C.byref(la), x, C.byref(_cache(cap=1 << 23, d=4096, group=128, bits=4)), None, 0, 0, 0, x,
                                    (C.c_int32 * 1)(8), x, x, 1 << 30, st) == UNSUPPORTED
    # per-channel cache: block quantiser and attention
    pc = lambda **kw: _cache(**dict(dict(cap=256, d=256, group=128, bits=3), **kw))
    qb = lambda c, nblk=1, b0=0, xx=x: lib.xq_quantize_blocks_per_channel(C.byref(c), xx, nblk, (C.c_int32 * 1)(b0), st)
    assert qb(pc(), nblk=0) == 0
    assert qb(pc(), nblk=1, b0=2) == INVALID                                    # past the capacity
    assert qb(pc(), xx=None) == INVALID
    assert qb(pc(cap=200)) == INVALID                                           # capacity not a whole number of blocks
    assert qb(pc(group=32)) == UNSUPPORTED
    assert qb(pc(d=192)) == UNSUPPORTED
    pa = lambda c=None, ln=130, tail=x, wsb=1 << 30, terms=None, tb=0: lib.xq_remat_attn_decode_per_channel(
        C.byref(la), x, C.byref(c if c is not None else pc()), tail, (C.c_int32 * 1)(ln), x, x, terms, tb, 0, x, x, wsb, st)
    assert pa(ln=0) == INVALID
    assert pa(ln=400) == INVALID                                                # three blocks do not fit a cache of two
    assert pa(tail=None) == INVALID
    assert pa(wsb=64) == WORKSPACE
    assert pa(c=pc(bits=8)) == UNSUPPORTED
    assert pa(terms=x, tb=64) == WORKSPACE                                      # a terms buffer too small for the cache
    assert xq.xq_per_channel_terms_bytes(1, 256, 256, 128, 2) > 0
    assert xq.xq_per_channel_terms_bytes(1, 200, 256, 128, 2) == 0              # capacity not a whole number of blocks
    assert xq.xq_per_channel_terms_bytes(1, 256, 256, 32, 2) == 0
    assert xq.xq_remat_attn_per_channel_workspace_bytes(xq.XQAttn(4, 2, 128, 0.1), 1, 300, 256, 32) == 0
    assert xq.xq_remat_attn_per_channel_workspace_bytes(xq.XQAttn(4, 2, 128, 0.1), 1, 300, 256, 128) > 0
    # latent keys per channel, latent values per token
    at2 = xq.XQAttn(4, 2, 128, 0.1)
    assert xq.xq_prepared_weights_pairs_bytes(at2, 256, 128, 3) > 256 * 256 * 2
    assert xq.xq_prepared_weights_pairs_bytes(at2, 256, 0, 16) == 256 * 256 * 2                 # the dense stream: no correction slabs
    assert xq.xq_prepared_weights_pairs_bytes(xq.XQAttn(3, 3, 128, 0.1), 384, 128, 3) == 0     # odd number of KV heads
    assert lib.xq_prepare_weights_pairs(C.byref(la), 256, 128, 3, x, x, 16, st) == WORKSPACE
    assert lib.xq_prepare_weights_pairs(C.byref(la), 256, 128, 3, None, x, 1 << 30, st) == INVALID
    kc, vc = pc(d=256), _cache(cap=256, d=256, group=64, bits=2)
    lp = lambda k=kc, v=vc, ln=130, wsb=1 << 30, terms=None, tb=0, k0=None, k0s=0, w0=None: \
        lib.xq_remat_attn_decode_latent_per_channel(C.byref(la), x, C.byref(k), x, C.byref(v), x, x, x, (C.c_int32 * 1)(ln),
                                                    k0, k0s, w0, terms, tb, 0, x, x, wsb, st)
    assert lp(ln=0) == INVALID
    assert lp(ln=300) == INVALID                                                # longer than the value cache
    assert lp(v=_cache(cap=256, d=512, group=64, bits=2)) == INVALID            # widths differ
    assert lp(wsb=64) == WORKSPACE
    assert lp(k=pc(d=256, bits=8)) == UNSUPPORTED
    assert lp(terms=x, tb=64) == WORKSPACE
    assert lp(k0=x, k0s=256, w0=None) == INVALID                                # the fp16 channel without its weight row
    assert lp(k0=x, k0s=100, w0=x) == INVALID                                   # fewer fp16 values than tokens
    assert xq.xq_remat_attn_latent_per_channel_workspace_bytes(at2, 1, 300, 256, 128, 64) > 0
    assert xq.xq_remat_attn_latent_per_channel_workspace_bytes(at2, 1, 300, 256, 128, 32) == 0


def test_binding_has_no_cpu_fallback():
    src = open(os.path.join(ROOT, "paper_2508_10395_amd", "binding.py")).read()
    assert "oracle" not in src
    with pytest.raises(OSError):
        C.CDLL(os.path.join(ROOT, "paper_2508_10395_amd", "does_not_exist.so"))
