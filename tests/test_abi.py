"""CPU-side checks of the C ABI: the library loads, exports every symbol hlq.h declares, and
rejects bad arguments with the documented status before touching the GPU."""
import ctypes as C
import os
import re

import pytest

import paper_2406_15102_amd as hlq
from paper_2406_15102_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "hlq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hlq_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    declared = _declared_symbols()
    assert "hlq_linear_backward" in declared and "hlq_compress_act" in declared
    l = hlq.lib()
    for name in declared:
        assert hasattr(l, name), "libhlq.so does not export %s" % name
    assert declared == binding.exported_symbols()


def test_version_and_status_strings():
    assert hlq.hlq_version() >= 100
    assert hlq.hlq_status_str(0) == "HLQ_OK"
    for code, word in [(1, "NULL"), (2, "SHAPE"), (3, "BLOCK"), (4, "RANK"), (5, "DTYPE"), (6, "WORKSPACE"),
                       (7, "LAUNCH")]:
        assert word in hlq.hlq_status_str(code)
    assert "unknown" in hlq.hlq_status_str(99)


def test_workspace_bytes():
    n = hlq.hlq_workspace_bytes(4096, 4096, 11008, 16, 8)
    # codes of G and W, bf16 compressed G and X, plus small vectors
    assert n >= 4096 * 11008 * 2 + (11008 + 4096) * 2048 * 2
    assert hlq.hlq_workspace_bytes(4096, 4096, 11008, 16, 8, True) < n
    assert hlq.hlq_workspace_bytes(4096, 4096, 11000, 16, 8) == 0      # d_out % B
    assert hlq.hlq_workspace_bytes(4096, 4096, 11008, 24, 8) == 0      # bad block
    assert hlq.hlq_quantize_w_workspace_bytes(11008, 4096) > 0


FAKE = C.c_void_p(0x10000)   # non-null, 16-aligned; never dereferenced because validation fails first


def _bw(G=FAKE, X=FAKE, W=FAKE, N=256, d_in=256, d_out=256, B=16, r=8, dX=FAKE, dW=FAKE):
    return hlq.lib().hlq_linear_backward(G, X, W, N, d_in, d_out, B, r, 0, dX, dW, None)


def test_linear_backward_rejects_bad_arguments_without_a_gpu():
    assert _bw(G=None) == 1 and _bw(dX=None) == 1 and _bw(W=None) == 1
    assert _bw(B=8) == 3 and _bw(B=48) == 3 and _bw(B=128) == 3
    assert _bw(r=0) == 4 and _bw(r=3) == 4 and _bw(r=32) == 4
    assert _bw(N=0) == 2 and _bw(N=250) == 2            # empty / not a multiple of B
    assert _bw(d_out=250) == 2 and _bw(d_out=65536 + 64) == 2
    assert _bw(d_in=100) == 2                            # d_in % 8
    assert _bw(N=16, r=1) == 2                           # compressed token axis not a multiple of 8
    assert _bw(N=1 << 22, d_out=4096) == 2               # random-stream counter would overflow


def test_ex_rejects_bad_arguments_without_a_gpu():
    f = hlq.lib().hlq_linear_backward_ex
    ok = dict(N=256, d_in=256, d_out=256, B=16, r=8)

    def call(G=FAKE, X=FAKE, Xh=None, W=FAKE, dt=0, dX=FAKE, dW=FAKE, ws=FAKE, wsb=1 << 30, **kw):
        a = dict(ok, **kw)
        return f(G, X, Xh, W, a["N"], a["d_in"], a["d_out"], a["B"], a["r"], 0, dt, dX, dW, ws, wsb, None)

    assert call(dt=7) == 5
    assert call(X=FAKE, Xh=FAKE) == 1 and call(X=None, Xh=None) == 1     # exactly one of X / XhatT
    assert call(dX=None, dW=None) == 1
    assert call(wsb=1000) == 6                                            # workspace too small
    assert call(ws=C.c_void_p(0x10010)) == 6                              # workspace misaligned
    assert call(G=C.c_void_p(0x10004)) == 2                               # tensor misaligned


def test_stage_entry_points_reject_bad_arguments_without_a_gpu():
    l = hlq.lib()
    assert l.hlq_quantize_g(None, 16, 256, 16, 0, 0, 4, FAKE, FAKE, None, None) == 1
    assert l.hlq_quantize_g(FAKE, 16, 250, 16, 0, 0, 4, FAKE, FAKE, None, None) == 2
    assert l.hlq_quantize_g(FAKE, 16, 256, 20, 0, 0, 4, FAKE, FAKE, None, None) == 3
    assert l.hlq_quantize_g(FAKE, 16, 256, 16, 0, 9, 4, FAKE, FAKE, None, None) == 5
    assert l.hlq_quantize_g(FAKE, 16, 256, 16, 0, 0, 5, FAKE, FAKE, None, None) == 5      # bits must be 4 or 8
    assert l.hlq_quantize_w(FAKE, 256, 256, 16, 0, 0, 4, FAKE, FAKE, None, None, 0, None) == 1
    assert l.hlq_quantize_w(FAKE, 256, 256, 16, 0, 0, 4, FAKE, FAKE, None, FAKE, 16, None) == 6
    assert l.hlq_quantize_w(FAKE, 256, 100, 16, 0, 0, 4, FAKE, FAKE, None, FAKE, 1 << 20, None) == 2
    assert l.hlq_int8_gemm_nt(FAKE, FAKE, 64, 64, 40, None, None, 1.0, 1, FAKE, None, None, 0, None) == 2   # K % 16
    assert l.hlq_int8_gemm_nt(FAKE, FAKE, 64, 62, 64, None, None, 1.0, 1, FAKE, None, None, 0, None) == 2   # Nn % 4
    assert l.hlq_int8_gemm_nt(FAKE, FAKE, 64, 64, 64, None, None, 1.0, 1, None, None, None, 0, None) == 1
    assert l.hlq_int8_gemm_nt(FAKE, FAKE, 64, 64, 131072 + 16, None, None, 1.0, 1, FAKE, None, None, 0, None) == 2   # int32 range
    assert l.hlq_quantize_g(FAKE, 16, 48, 16, 0, 0, 0x104, FAKE, FAKE, None, None) == 2     # packed rows: d_out % 32
    assert l.hlq_quantize_w(FAKE, 48, 256, 16, 0, 0, 0x104, FAKE, FAKE, None, FAKE, 1 << 20, None) == 2
    assert l.hlq_int4_gemm_nt(FAKE, FAKE, 64, 64, 48, None, None, 1.0, 1, FAKE, None, None, 0, None) == 2   # K % 32
    assert l.hlq_int4_gemm_nt(FAKE, FAKE, 64, 64, 1 << 18, None, None, 1.0, 1, FAKE, None, None, 0, None) == 2
    assert l.hlq_int4_gemm_nt(FAKE, None, 64, 64, 64, None, None, 1.0, 1, FAKE, None, None, 0, None) == 1
    assert l.hlq_hla_project(FAKE, 250, 64, 16, 8, 0, FAKE, None, None) == 2
    assert l.hlq_hla_project(FAKE, 256, 64, 16, 5, 0, FAKE, None, None) == 4
    assert l.hlq_compress_act(FAKE, 256, 64, 16, 8, 0, None, None) == 1
    assert l.hlq_hla_project_basis(FAKE, 256, 64, 16, 8, 2, 0, FAKE, None, None) == 4                       # unknown basis
    assert l.hlq_hla_project_basis(FAKE, 250, 64, 16, 8, 1, 0, FAKE, None, None) == 2
    assert l.hlq_bf16_gemm_nt(FAKE, FAKE, 64, 64, 36, 1.0, 0, FAKE, None, 0, None) == 2                     # K % 8
    W256 = C.c_void_p(0x10000)
    assert l.hlq_hla_quantize(FAKE, 256, 64, 16, 2, 0, 2, 0, FAKE, FAKE, None, W256, 1 << 20, None) == 4   # r % 4
    assert l.hlq_hla_quantize(FAKE, 256, 64, 16, 8, 0, 1, 0, FAKE, FAKE, None, W256, 1 << 20, None) == 2   # stream id
    assert l.hlq_hla_quantize(FAKE, 16, 64, 16, 8, 0, 2, 0, FAKE, FAKE, None, W256, 1 << 20, None) == 2    # Kc % 16
    assert l.hlq_hla_quantize(FAKE, 256, 64, 16, 8, 0, 2, 0, FAKE, FAKE, None, W256, 16, None) == 6
    assert l.hlq_compress_act_int8(FAKE, 256, 64, 16, 8, 0, 0, None, FAKE, W256, 1 << 20, None) == 1


def test_mode_entry_point_rejects_bad_arguments_without_a_gpu():
    f = hlq.lib().hlq_linear_backward_mode

    def call(X=FAKE, Xc=None, sXc=None, flags=0, N=256, r=8, wsb=1 << 30):
        return f(FAKE, X, Xc, sXc, FAKE, N, 256, 256, 16, r, 0, 0, flags, FAKE, FAKE, FAKE, wsb, None)

    assert call(flags=64) == 2                                  # unknown flag
    assert call(flags=2, r=2) == 4                              # integer g_w path needs r % 4 == 0
    assert call(flags=2, N=16, r=8) == 2                        # compressed token axis % 16
    assert call(X=None, Xc=FAKE, sXc=None, flags=2) == 1        # int8 codes need their scales
    assert call(X=None, Xc=FAKE, sXc=FAKE, flags=0) == 1        # bf16 XhatT takes no scales
    assert call(flags=2, wsb=1000) == 6
    assert hlq.hlq_workspace_bytes_mode(4096, 4096, 11008, 16, 8, False, 2) < hlq.hlq_workspace_bytes(4096, 4096, 11008, 16, 8)
    assert hlq.hlq_workspace_bytes_mode(4096, 4096, 11008, 16, 8, False, 0) == hlq.hlq_workspace_bytes(4096, 4096, 11008, 16, 8)
    assert hlq.hlq_workspace_bytes_mode(4096, 4096, 11008, 16, 2, False, 2) == 0


def test_binding_refuses_cpu_tensors():
    import torch
    t = torch.zeros(16, 256, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        hlq.hlq_quantize_g(t, 16, 0, torch.zeros(16, 256, dtype=torch.int8), torch.zeros(16))


def test_cached_weight_entry_point_without_a_gpu():
    l = hlq.lib()
    assert l.hlq_weight_code_bits(256, 0) == 0x104 and l.hlq_weight_code_bits(48, 0) == 4
    assert l.hlq_weight_code_bits(256, 1) == 8 and l.hlq_weight_code_bits(256, 4) == 4
    f = l.hlq_linear_backward_cached

    def call(WqT=FAKE, sW=FAKE, dX=FAKE, dW=FAKE, **kw):
        a = dict(N=256, d_in=256, d_out=256, B=16, r=8, flags=0)
        a.update(kw)
        return f(FAKE, FAKE, None, None, WqT, sW, a["N"], a["d_in"], a["d_out"], a["B"], a["r"], 0, 0, a["flags"], dX, dW,
                 FAKE, 1 << 30, None)

    assert call(WqT=None) == 1 and call(sW=None) == 1            # dX wanted: the codes and their scales are needed
    assert call(WqT=C.c_void_p(0x10004)) == 2                    # misaligned codes
    assert call(d_out=250) == 2 and call(B=20) == 3 and call(flags=64) == 2


def test_convolution_entry_points_without_a_gpu():
    l = hlq.lib()

    def geom(**kw):
        a = dict(Nb=4, H=8, W=8, C=16, O=32, kh=3, kw=3, stride_h=1, stride_w=1, pad_h=1, pad_w=1, dil_h=1, dil_w=1)
        a.update(kw)
        return hlq.hlq_conv_geom(**a)

    assert hlq.hlq_conv_sizes(geom()) == (8, 8, 256, 144)
    assert hlq.hlq_conv_sizes(geom(stride_h=2, stride_w=2)) == (4, 4, 64, 144)
    assert hlq.hlq_conv_sizes(geom(H=7, W=9, kh=3, kw=2, stride_h=2, pad_h=0, dil_w=2)) == (3, 9, 108, 96)
    assert hlq.hlq_conv_sizes(geom(kh=1, kw=1, pad_h=0, pad_w=0)) == (8, 8, 256, 16)
    v = C.c_int64()
    for bad in (geom(stride_h=0), geom(pad_w=-1), geom(dil_h=0), geom(C=0), geom(H=2, pad_h=0, kh=5), geom(Nb=0)):
        assert l.hlq_conv_sizes(C.byref(bad), C.byref(v), None, None, None) == 2
    assert l.hlq_conv_sizes(None, None, None, None, None) == 1
    g = geom()
    assert l.hlq_im2col(None, C.byref(g), 0, FAKE, None) == 1 and l.hlq_im2col(FAKE, C.byref(g), 7, FAKE, None) == 5
    assert l.hlq_im2col(FAKE, C.byref(g), 0, C.c_void_p(0x10002), None) == 2
    assert l.hlq_col2im(FAKE, C.byref(g), 0, None, None) == 1 and l.hlq_col2im(FAKE, None, 0, FAKE, None) == 1
    f = l.hlq_conv2d_backward

    def call(g, G=FAKE, X=FAKE, W=FAKE, B=16, r=8, flags=0, dX=FAKE, dW=FAKE, wsb=1 << 40):
        return f(G, X, W, C.byref(g), B, r, 0, 0, flags, dX, dW, FAKE, wsb, None)

    assert call(g, G=None) == 1 and call(g, dX=None, dW=None) == 1 and call(g, X=None) == 1 and call(g, W=None) == 1
    assert call(g, B=20) == 3 and call(g, r=3) == 4 and call(g, flags=64) == 2
    assert call(geom(O=40)) == 2                                 # d_out = O must be whole Hadamard blocks
    assert call(geom(Nb=1, H=5, W=5)) == 2                       # N = 25 positions: not whole blocks of tokens
    assert call(geom(C=3)) == 2                                  # I = 27: rows of the column matrix must be 16-byte multiples
    assert call(g, wsb=1000) == 6
    # workspace: the column gradient on top of the linear pass's own; the column matrix too when the
    # channels do not divide among the lanes; nothing extra for a pointwise kernel
    inner = hlq.hlq_workspace_bytes_mode(256, 144, 32, 16, 8, False, 0)
    assert hlq.hlq_conv_workspace_bytes(g, 16, 8, 0) == inner + 256 * 144 * 2
    g4 = geom(C=4, kh=2, kw=2, pad_h=0, pad_w=0, stride_h=2, stride_w=2)          # N = 64, I = 16
    assert hlq.hlq_conv_workspace_bytes(g4, 16, 8, 0) == hlq.hlq_workspace_bytes_mode(64, 16, 32, 16, 8, False, 0) + 2 * 64 * 16 * 2
    assert l.hlq_conv_compress_act(FAKE, C.byref(g4), 16, 8, 0, 0, FAKE, None, None) == 2      # 4 channels, 8 per lane
    assert l.hlq_conv_compress_act(FAKE, C.byref(g), 16, 8, 0, 0, None, None, None) == 1
    assert l.hlq_conv_compress_act(FAKE, C.byref(g), 16, 8, 5, 0, FAKE, None, None) == 4       # unknown basis
    assert l.hlq_conv_compress_act(FAKE, C.byref(g), 16, 3, 0, 0, FAKE, None, None) == 4
    assert l.hlq_conv_compress_act_int8(FAKE, C.byref(g), 16, 2, 0, 0, 0, FAKE, FAKE, None, FAKE, 1 << 20, None) == 4
    assert l.hlq_conv_compress_act_int8(FAKE, C.byref(g), 16, 8, 0, 0, 0, FAKE, FAKE, None, FAKE, 16, None) == 6
    p = geom(kh=1, kw=1, pad_h=0, pad_w=0)
    assert hlq.hlq_conv_workspace_bytes(p, 16, 8, 0) == hlq.hlq_workspace_bytes_mode(256, 16, 32, 16, 8, False, 0)
    assert hlq.hlq_conv_workspace_bytes(geom(O=40), 16, 8, 0) == 0


def test_products_entry_point_without_a_gpu():
    l = hlq.lib()
    f = l.hlq_backward_products

    def call(Gq=FAKE, sG=FAKE, WqT=FAKE, sW=FAKE, bits=0x104, Gh=FAKE, sGh=None, Xh=FAKE, sXh=None, N=256, I=256, O=256,
             Kc=128, B=16, dt=0, dX=FAKE, dW=FAKE):
        return f(Gq, sG, WqT, sW, bits, Gh, sGh, Xh, sXh, N, I, O, Kc, B, dt, dX, dW, None, 0, None)

    assert call(Gq=None) == 1 and call(dW=None) == 1 and call(sGh=FAKE) == 1      # int8 projections come with both scales
    assert call(bits=5) == 2 and call(bits=0x304) == 2                             # storage, without a rounding bit
    assert call(O=48) == 2                                                         # packed codes need d_out % 32 == 0
    assert call(B=20) == 3 and call(dt=9) == 5
    assert call(Kc=12) == 2 and call(sGh=FAKE, sXh=FAKE, Kc=24) == 2               # 16-byte rows of either operand kind
    assert hlq.hlq_backward_products_workspace_bytes(50176, 432, 96, 25088, 0x104) > 0    # few tiles, long reduction
    assert hlq.hlq_backward_products_workspace_bytes(4096, 4096, 11008, 2048, 0x104) == 0
    assert hlq.hlq_backward_products_workspace_bytes(4096, 4096, 11008, 2048, 7) == 0


def test_set_workspace_rejects_and_bounds_the_plain_call_without_a_gpu():
    """A registered workspace is used or refused, never replaced by an allocation: with one that is
    too small the plain 12-argument call comes back with HLQ_ERR_WORKSPACE before anything is launched."""
    sw = hlq.lib().hlq_set_workspace
    try:
        assert sw(C.c_void_p(0x10010), 1 << 20) == 6            # not 256-byte aligned
        assert sw(FAKE, 0) == 6                                 # a pointer without a size
        assert sw(FAKE, 1000) == 0
        assert _bw() == 6                                       # 1000 bytes cannot hold this layer's scratch
        f = hlq.lib().hlq_linear_backward_ex                    # the same through a NULL workspace argument
        assert f(FAKE, FAKE, None, FAKE, 256, 256, 256, 16, 8, 0, 0, FAKE, FAKE, None, 0, None) == 6
        assert _bw(B=8) == 3                                    # argument checks still come first
    finally:
        assert sw(None, 0) == 0                                 # withdrawn: back to the library-owned scratch


def test_static_scratch_entry_point_rejects_bad_arguments_without_a_gpu():
    f = hlq.lib().hlq_quantize_w_static

    def call(W=FAKE, d_out=256, d_in=256, B=16, dt=0, bits=4, WqT=FAKE, sW=FAKE):
        return f(W, d_out, d_in, B, 0, dt, bits, WqT, sW, None)

    assert call(W=None) == 1 and call(WqT=None) == 1 and call(sW=None) == 1
    assert call(B=8) == 3 and call(dt=5) == 5 and call(bits=3) == 5
    assert call(d_in=100) == 2 and call(d_out=250) == 2
    assert call(d_in=65536 + 8, d_out=64) == 6                  # beyond the static array: refused, not allocated


def test_binding_refuses_mismatched_tensors():
    """The binding checks element type and element count of every tensor against the gradient's: an
    fp32 weight beside a bf16 gradient, or a tensor shorter than the stated sizes, must not reach
    the library (which sees only pointers)."""
    import torch
    g = torch.empty((32, 64), dtype=torch.bfloat16)
    x = torch.empty((32, 16), dtype=torch.bfloat16)
    w32 = torch.empty((64, 16), dtype=torch.float32)
    with pytest.raises(TypeError):
        binding._expect_backward(g, x, w32, None, None, 32, 16, 64)
    w = torch.empty((64, 8), dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        binding._expect_backward(g, x, w, None, None, 32, 16, 64)
    with pytest.raises(TypeError):
        binding._expect_store(torch.empty((16, 16), dtype=torch.bfloat16), None, 16, 16, binding.HLQ_FLAG_GW_INT8)
    binding._expect_backward(g, x, torch.empty((64, 16), dtype=torch.bfloat16), None, None, 32, 16, 64)
