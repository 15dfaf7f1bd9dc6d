"""ctypes binding of ``libhlq.so`` -- argument marshalling only.

Each function has the name and argument order of its C entry point in ``include/hlq.h``;
tensors are torch CUDA (ROCm) tensors whose ``data_ptr()`` is handed over together with the
current torch stream.  Nothing is computed here, and there is no fallback: if the HIP library
has not been built, importing the entry points raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhlq.so")

HLQ_BF16, HLQ_F32 = 0, 1
HLQ_OK = 0
HLQ_FLAG_GX_8BIT, HLQ_FLAG_GW_INT8, HLQ_FLAG_GX_UNPACKED, HLQ_FLAG_GW_SEQUENCY = 1, 2, 4, 8
HLQ_BASIS_NATURAL, HLQ_BASIS_SEQUENCY = 0, 1
HLQ_BITS_ROUND_MANTISSA = HLQ_BASIS_ROUND_MANTISSA = 0x200
HLQ_FLAG_ROUND_MANTISSA = 16
HLQ_FLAG_SEPARATE_PRODUCTS = 32
HLQ_FLAG_XC_INT4 = 64
HLQ_BITS_4, HLQ_BITS_8, HLQ_BITS_4_PACKED = 4, 8, 0x104



class hlq_conv_geom(C.Structure):
    """Geometry of a convolution layer, field for field the C struct of the same name."""
    _fields_ = [(n, C.c_int32) for n in ("Nb", "H", "W", "C", "O", "kh", "kw", "stride_h", "stride_w", "pad_h",
                                           "pad_w", "dil_h", "dil_w")]


_GEOM_P = C.POINTER(hlq_conv_geom)

_EXPORTS = {
    "hlq_status_str": (C.c_char_p, [C.c_int]),
    "hlq_version": (C.c_int, []),
    "hlq_workspace_bytes": (C.c_size_t, [C.c_int64, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int]),
    "hlq_set_workspace": (C.c_int, [C.c_void_p, C.c_size_t]),
    "hlq_set_option": (C.c_int, [C.c_int, C.c_int]),
    "hlq_quantize_w_static": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_uint64, C.c_int, C.c_int, C.c_void_p,
                                        C.c_void_p, C.c_void_p]),
    "hlq_linear_backward": (C.c_int, [C.c_void_p] * 3 + [C.c_int64] * 3 + [C.c_int, C.c_int, C.c_uint64]
                            + [C.c_void_p] * 3),
    "hlq_linear_backward_ex": (C.c_int, [C.c_void_p] * 4 + [C.c_int64] * 3 + [C.c_int, C.c_int, C.c_uint64, C.c_int]
                               + [C.c_void_p] * 3 + [C.c_size_t, C.c_void_p]),
    "hlq_compress_act": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_void_p,
                                   C.c_void_p]),
    "hlq_quantize_g": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_uint64, C.c_int, C.c_int, C.c_void_p,
                                 C.c_void_p, C.c_void_p, C.c_void_p]),
    "hlq_quantize_w_workspace_bytes": (C.c_size_t, [C.c_int64, C.c_int64]),
    "hlq_quantize_w": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_uint64, C.c_int, C.c_int, C.c_void_p,
                                 C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "hlq_hla_quantize_workspace_bytes": (C.c_size_t, [C.c_int64]),
    "hlq_hla_quantize": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_uint64, C.c_int, C.c_int,
                                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "hlq_compress_act_int8": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_uint64, C.c_int,
                                        C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "hlq_compress_act_int4": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_uint64, C.c_int,
                                        C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "hlq_workspace_bytes_mode": (C.c_size_t, [C.c_int64, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int]),
    "hlq_linear_backward_mode": (C.c_int, [C.c_void_p] * 5 + [C.c_int64] * 3 + [C.c_int, C.c_int, C.c_uint64, C.c_int,
                                           C.c_int] + [C.c_void_p] * 3 + [C.c_size_t, C.c_void_p]),
    "hlq_weight_code_bits": (C.c_int, [C.c_int64, C.c_int]),
    "hlq_linear_backward_cached": (C.c_int, [C.c_void_p] * 6 + [C.c_int64] * 3 + [C.c_int, C.c_int, C.c_uint64, C.c_int,
                                             C.c_int] + [C.c_void_p] * 3 + [C.c_size_t, C.c_void_p]),
    "hlq_int8_gemm_nt": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p,
                                   C.c_float, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "hlq_int4_gemm_nt": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p,
                                   C.c_float, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "hlq_gemm_workspace_bytes": (C.c_size_t, [C.c_int, C.c_int64, C.c_int64, C.c_int64]),
    "hlq_hla_project": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_void_p,
                                  C.c_void_p, C.c_void_p]),
    "hlq_hla_project_basis": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p,
                                        C.c_void_p, C.c_void_p]),
    "hlq_hla_quantize_basis": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_uint64, C.c_int,
                                         C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "hlq_bf16_gemm_nt": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_float, C.c_int,
                                   C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "hlq_mfma_probe": (C.c_int, [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]),
    "hlq_backward_products_workspace_bytes": (C.c_size_t, [C.c_int64] * 4 + [C.c_int, C.c_int]),
    "hlq_backward_products_plan": (C.c_int, [C.c_int64] * 4 + [C.c_int, C.c_int, C.c_size_t, C.POINTER(C.c_int)]),
    "hlq_backward_products": (C.c_int, [C.c_void_p] * 4 + [C.c_int] + [C.c_void_p] * 4 + [C.c_int64] * 4
                              + [C.c_int, C.c_int] + [C.c_void_p] * 3 + [C.c_size_t, C.c_void_p]),
    "hlq_conv_sizes": (C.c_int, [_GEOM_P] + [C.POINTER(C.c_int64)] * 4),
    "hlq_im2col": (C.c_int, [C.c_void_p, _GEOM_P, C.c_int, C.c_void_p, C.c_void_p]),
    "hlq_col2im": (C.c_int, [C.c_void_p, _GEOM_P, C.c_int, C.c_void_p, C.c_void_p]),
    "hlq_conv_compress_act": (C.c_int, [C.c_void_p, _GEOM_P, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                        C.c_void_p]),
    "hlq_conv_compress_act_int8": (C.c_int, [C.c_void_p, _GEOM_P, C.c_int, C.c_int, C.c_int, C.c_uint64, C.c_int,
                                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "hlq_conv_workspace_bytes": (C.c_size_t, [_GEOM_P, C.c_int, C.c_int, C.c_int, C.c_int]),
    "hlq_conv2d_backward": (C.c_int, [C.c_void_p] * 3 + [_GEOM_P, C.c_int, C.c_int, C.c_uint64, C.c_int, C.c_int]
                            + [C.c_void_p] * 3 + [C.c_size_t, C.c_void_p]),
}

_lib = None


class HlqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s" % (where, lib().hlq_status_str(status).decode()))


def exported_symbols():
    """Names every build of the library must export (one per declaration in hlq.h)."""
    return sorted(_EXPORTS)


def lib() -> C.CDLL:
    """Load the HIP library; raises if it has not been built (there is no other code path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "HIP library %s not built: run `python -m paper_2406_15102_amd.build` "
                "(there is no CPU fallback)" % LIB_PATH)
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in _EXPORTS.items():
            fn = getattr(l, name)
            fn.restype = res
            fn.argtypes = args
        _lib = l
    return _lib


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return HLQ_BF16
    if t.dtype == torch.float32:
        return HLQ_F32
    raise TypeError("tensor dtype must be bfloat16 or float32, got %s" % t.dtype)


def _ptr(t, dtype=None):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("tensor must live on the GPU")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous (dense row-major)")
    if dtype is not None and t.dtype != dtype:
        raise TypeError("expected %s, got %s" % (dtype, t.dtype))
    return C.c_void_p(t.data_ptr())


def _expect(name, t, shape, dtype):
    """Refuse a tensor whose element type or element count is not what the C call will read or
    write: the library sees only a pointer and would run past the end (or read bf16 bits as fp32)."""
    if t is None:
        return
    if t.dtype != dtype:
        raise TypeError("%s must be %s like the gradient, got %s" % (name, dtype, t.dtype))
    n = 1
    for d in shape:
        n *= int(d)
    if t.numel() != n:
        raise ValueError("%s must hold %s = %d elements, has %d" % (name, "x".join(str(int(d)) for d in shape), n, t.numel()))


def _expect_backward(G, X, W, dX, dW, N, d_in, d_out):
    dt = G.dtype
    _expect("G", G, (N, d_out), dt)
    _expect("X", X, (N, d_in), dt)
    _expect("W", W, (d_out, d_in), dt)
    _expect("dX", dX, (N, d_in), dt)
    _expect("dW", dW, (d_out, d_in), dt)


def _expect_store(Xc, sXc, d_in, Kc, flags):
    if Xc is None:
        return
    if flags & HLQ_FLAG_XC_INT4:
        _expect("Xc", Xc, (d_in, Kc // 2), torch.uint8)
        _expect("sXc", sXc, (d_in,), torch.float32)
    elif flags & HLQ_FLAG_GW_INT8:
        _expect("Xc", Xc, (d_in, Kc), torch.int8)
        _expect("sXc", sXc, (d_in,), torch.float32)
    else:
        _expect("Xc", Xc, (d_in, Kc), torch.bfloat16)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status: int, where: str):
    if status != HLQ_OK:
        raise HlqError(status, where)


def hlq_version() -> int:
    return int(lib().hlq_version())


def hlq_status_str(status: int) -> str:
    return lib().hlq_status_str(status).decode()


def hlq_workspace_bytes(N, d_in, d_out, B, r, x_is_compressed=False) -> int:
    return int(lib().hlq_workspace_bytes(N, d_in, d_out, B, r, int(bool(x_is_compressed))))


HLQ_OPT_PERSISTENT_PRODUCTS = 1
HLQ_OPT_SHARED_G_READ = 2
HLQ_OPT_DIRECT_TO_LDS = 3
HLQ_OPT_PLAN_TILE = 4
HLQ_OPT_PLAN_SPLITS = 5
HLQ_OPT_TAIL_TILES = 6
HLQ_OPT_FRONT_INTERLEAVE = 7


def hlq_set_option(option, value):
    _check(lib().hlq_set_option(int(option), int(value)), "hlq_set_option")


def hlq_set_workspace(workspace):
    """Register `workspace` (a uint8 CUDA tensor the caller keeps alive) as the scratch of every call
    on the current device that passes none; None withdraws it."""
    if workspace is None:
        _check(lib().hlq_set_workspace(None, 0), "hlq_set_workspace")
    else:
        _check(lib().hlq_set_workspace(_ptr(workspace), _nbytes(workspace)), "hlq_set_workspace")


def hlq_linear_backward(G, X, W, B, r, seed, dX, dW):
    """dX, dW <- HLQ backward of one bf16 layer (registered or library-owned workspace)."""
    N, d_out = G.shape
    d_in = W.shape[1]
    for t in (G, X, W, dX, dW):
        _ptr(t, torch.bfloat16)
    assert X.shape == (N, d_in) and W.shape == (d_out, d_in) and dX.shape == (N, d_in) and dW.shape == (d_out, d_in)
    _check(lib().hlq_linear_backward(_ptr(G), _ptr(X), _ptr(W), N, d_in, d_out, B, r, seed, _ptr(dX), _ptr(dW),
                                     _stream()), "hlq_linear_backward")


def hlq_linear_backward_ex(G, X, XhatT, W, N, d_in, d_out, B, r, seed, dX, dW, workspace=None):
    """Full-option call; any of X / XhatT / W / dX / dW may be None as hlq.h allows."""
    dt = _dt(G)
    _expect_backward(G, X, W, dX, dW, N, d_in, d_out)
    _expect_store(XhatT, None, d_in, N // B * r, 0)
    ws_ptr, ws_bytes = (None, 0) if workspace is None else (_ptr(workspace), workspace.numel() * workspace.element_size())
    _check(lib().hlq_linear_backward_ex(_ptr(G), _ptr(X), _ptr(XhatT), _ptr(W), N, d_in, d_out, B, r, seed, dt,
                                        _ptr(dX), _ptr(dW), ws_ptr, ws_bytes, _stream()), "hlq_linear_backward_ex")


def hlq_compress_act(X, B, r, XhatT):
    N, d_in = X.shape
    _check(lib().hlq_compress_act(_ptr(X), N, d_in, B, r, _dt(X), _ptr(XhatT, torch.bfloat16), _stream()),
           "hlq_compress_act")


def _codes_ptr(t):
    if t.dtype not in (torch.int8, torch.uint8):
        raise TypeError("codes must be int8 (or uint8 for packed codes), got %s" % t.dtype)
    return _ptr(t)


def hlq_quantize_g(G, B, seed, Gq, sG, coeff=None, bits=4):
    N, d_out = G.shape
    _check(lib().hlq_quantize_g(_ptr(G), N, d_out, B, seed, _dt(G), bits, _codes_ptr(Gq), _ptr(sG, torch.float32),
                                _ptr(coeff, torch.float32), _stream()), "hlq_quantize_g")


def hlq_quantize_w_workspace_bytes(d_out, d_in) -> int:
    return int(lib().hlq_quantize_w_workspace_bytes(d_out, d_in))


def hlq_quantize_w(W, B, seed, WqT, sW, workspace, coeffT=None, bits=4):
    d_out, d_in = W.shape
    _check(lib().hlq_quantize_w(_ptr(W), d_out, d_in, B, seed, _dt(W), bits, _codes_ptr(WqT), _ptr(sW, torch.float32),
                                _ptr(coeffT, torch.float32), _ptr(workspace),
                                workspace.numel() * workspace.element_size(), _stream()), "hlq_quantize_w")


def hlq_quantize_w_static(W, B, seed, WqT, sW, bits=4):
    """hlq_quantize_w on the library's static scratch (no workspace, nothing allocated)."""
    d_out, d_in = W.shape
    _check(lib().hlq_quantize_w_static(_ptr(W), d_out, d_in, B, seed, _dt(W), bits, _codes_ptr(WqT),
                                       _ptr(sW, torch.float32), _stream()), "hlq_quantize_w_static")


def _ws(workspace):
    return (None, 0) if workspace is None else (_ptr(workspace), workspace.numel() * workspace.element_size())


def hlq_gemm_workspace_bytes(kind, M, Nn, K) -> int:
    return int(lib().hlq_gemm_workspace_bytes(kind, M, Nn, K))


def hlq_int8_gemm_nt(A, Bm, sA, sB, alpha, C_out=None, acc=None, workspace=None):
    M, K = A.shape
    Nn = Bm.shape[0]
    out_dt = _dt(C_out) if C_out is not None else HLQ_F32
    wp, wb = _ws(workspace)
    _check(lib().hlq_int8_gemm_nt(_ptr(A, torch.int8), _ptr(Bm, torch.int8), M, Nn, K, _ptr(sA, torch.float32),
                                  _ptr(sB, torch.float32), float(alpha), out_dt, _ptr(C_out), _ptr(acc, torch.int32),
                                  wp, wb, _stream()), "hlq_int8_gemm_nt")


def hlq_int4_gemm_nt(A4, Bm4, sA, sB, alpha, C_out=None, acc=None, workspace=None):
    """A4 [M, K/2], Bm4 [Nn, K/2] uint8: 4-bit codes, two to a byte."""
    M, Kb = A4.shape
    Nn = Bm4.shape[0]
    out_dt = _dt(C_out) if C_out is not None else HLQ_F32
    wp, wb = _ws(workspace)
    _check(lib().hlq_int4_gemm_nt(_ptr(A4, torch.uint8), _ptr(Bm4, torch.uint8), M, Nn, 2 * Kb, _ptr(sA, torch.float32),
                                  _ptr(sB, torch.float32), float(alpha), out_dt, _ptr(C_out), _ptr(acc, torch.int32),
                                  wp, wb, _stream()), "hlq_int4_gemm_nt")


def hlq_hla_project(T, B, r, ThatT, coeffT=None):
    N, D = T.shape
    _check(lib().hlq_hla_project(_ptr(T), N, D, B, r, _dt(T), _ptr(ThatT, torch.bfloat16),
                                 _ptr(coeffT, torch.float32), _stream()), "hlq_hla_project")


def hlq_bf16_gemm_nt(A, Bm, alpha, C_out, workspace=None):
    M, K = A.shape
    Nn = Bm.shape[0]
    wp, wb = _ws(workspace)
    _check(lib().hlq_bf16_gemm_nt(_ptr(A, torch.bfloat16), _ptr(Bm, torch.bfloat16), M, Nn, K, float(alpha),
                                  _dt(C_out), _ptr(C_out), wp, wb, _stream()), "hlq_bf16_gemm_nt")


def hlq_mfma_probe(kind, blocks, iters, sink):
    _check(lib().hlq_mfma_probe(kind, blocks, iters, _ptr(sink, torch.float32), _stream()), "hlq_mfma_probe")


def _nbytes(t):
    return t.numel() * t.element_size()


def hlq_hla_quantize_workspace_bytes(D) -> int:
    return int(lib().hlq_hla_quantize_workspace_bytes(D))


def hlq_hla_quantize(T, B, r, seed, tensor, TqT, sT, workspace, coeffT=None):
    N, D = T.shape
    _check(lib().hlq_hla_quantize(_ptr(T), N, D, B, r, seed, tensor, _dt(T), _ptr(TqT, torch.int8),
                                  _ptr(sT, torch.float32), _ptr(coeffT, torch.float32), _ptr(workspace),
                                  _nbytes(workspace), _stream()), "hlq_hla_quantize")


def hlq_compress_act_int8(X, B, r, seed, XqT, sX, workspace):
    N, d_in = X.shape
    _check(lib().hlq_compress_act_int8(_ptr(X), N, d_in, B, r, seed, _dt(X), _ptr(XqT, torch.int8),
                                       _ptr(sX, torch.float32), _ptr(workspace), _nbytes(workspace), _stream()),
           "hlq_compress_act_int8")


def hlq_compress_act_int4(X, B, r, seed, Xq4T, sX, workspace):
    N, d_in = X.shape
    _check(lib().hlq_compress_act_int4(_ptr(X), N, d_in, B, r, seed, _dt(X), _ptr(Xq4T, torch.uint8),
                                       _ptr(sX, torch.float32), _ptr(workspace), _nbytes(workspace), _stream()),
           "hlq_compress_act_int4")


def hlq_workspace_bytes_mode(N, d_in, d_out, B, r, x_is_compressed=False, flags=0) -> int:
    return int(lib().hlq_workspace_bytes_mode(N, d_in, d_out, B, r, int(bool(x_is_compressed)), flags))


def hlq_linear_backward_mode(G, X, Xc, sXc, W, N, d_in, d_out, B, r, seed, flags, dX, dW, workspace=None):
    """hlq_linear_backward_ex with HLQ_FLAG_GX_8BIT / HLQ_FLAG_GW_INT8."""
    _expect_backward(G, X, W, dX, dW, N, d_in, d_out)
    _expect_store(Xc, sXc, d_in, N // B * r, flags)
    ws_ptr, ws_bytes = (None, 0) if workspace is None else (_ptr(workspace), _nbytes(workspace))
    _check(lib().hlq_linear_backward_mode(_ptr(G), _ptr(X), _ptr(Xc), _ptr(sXc, torch.float32), _ptr(W), N, d_in,
                                          d_out, B, r, seed, _dt(G), flags, _ptr(dX), _ptr(dW), ws_ptr, ws_bytes,
                                          _stream()), "hlq_linear_backward_mode")


def hlq_weight_code_bits(d_out, flags) -> int:
    return int(lib().hlq_weight_code_bits(d_out, flags))


def hlq_linear_backward_cached(G, X, Xc, sXc, WqT, sW, N, d_in, d_out, B, r, seed, flags, dX, dW, workspace=None):
    """hlq_linear_backward_mode with the weight codes of hlq_quantize_w handed over."""
    _expect_backward(G, X, None, dX, dW, N, d_in, d_out)
    _expect_store(Xc, sXc, d_in, N // B * r, flags)
    ws_ptr, ws_bytes = (None, 0) if workspace is None else (_ptr(workspace), _nbytes(workspace))
    _check(lib().hlq_linear_backward_cached(_ptr(G), _ptr(X), _ptr(Xc), _ptr(sXc, torch.float32), _ptr(WqT),
                                            _ptr(sW, torch.float32), N, d_in, d_out, B, r, seed, _dt(G), flags,
                                            _ptr(dX), _ptr(dW), ws_ptr, ws_bytes, _stream()),
           "hlq_linear_backward_cached")


def hlq_hla_project_basis(T, B, r, basis, ThatT, coeffT=None):
    N, D = T.shape
    _check(lib().hlq_hla_project_basis(_ptr(T), N, D, B, r, basis, _dt(T), _ptr(ThatT, torch.bfloat16),
                                       _ptr(coeffT, torch.float32), _stream()), "hlq_hla_project_basis")


def hlq_hla_quantize_basis(T, B, r, basis, seed, tensor, TqT, sT, workspace, coeffT=None):
    N, D = T.shape
    _check(lib().hlq_hla_quantize_basis(_ptr(T), N, D, B, r, basis, seed, tensor, _dt(T), _ptr(TqT, torch.int8),
                                        _ptr(sT, torch.float32), _ptr(coeffT, torch.float32), _ptr(workspace),
                                        _nbytes(workspace), _stream()), "hlq_hla_quantize_basis")


def hlq_conv_sizes(geom):
    """-> (Ho, Wo, N, I) of the geometry."""
    v = [C.c_int64() for _ in range(4)]
    _check(lib().hlq_conv_sizes(C.byref(geom), *[C.byref(x) for x in v]), "hlq_conv_sizes")
    return tuple(int(x.value) for x in v)


def hlq_im2col(X, geom, cols):
    _check(lib().hlq_im2col(_ptr(X), C.byref(geom), _dt(X), _ptr(cols, X.dtype), _stream()), "hlq_im2col")


def hlq_col2im(cols, geom, dX):
    _check(lib().hlq_col2im(_ptr(cols), C.byref(geom), _dt(cols), _ptr(dX, cols.dtype), _stream()), "hlq_col2im")


def hlq_conv_compress_act(X, geom, B, r, basis, XhatT, coeffT=None):
    _check(lib().hlq_conv_compress_act(_ptr(X), C.byref(geom), B, r, basis, _dt(X), _ptr(XhatT, torch.bfloat16),
                                       _ptr(coeffT, torch.float32), _stream()), "hlq_conv_compress_act")


def hlq_conv_compress_act_int8(X, geom, B, r, basis, seed, XqT, sX, workspace, coeffT=None):
    _check(lib().hlq_conv_compress_act_int8(_ptr(X), C.byref(geom), B, r, basis, seed, _dt(X), _ptr(XqT, torch.int8),
                                            _ptr(sX, torch.float32), _ptr(coeffT, torch.float32), _ptr(workspace),
                                            _nbytes(workspace), _stream()), "hlq_conv_compress_act_int8")


def hlq_conv_workspace_bytes(geom, B, r, dtype, flags=0) -> int:
    return int(lib().hlq_conv_workspace_bytes(C.byref(geom), B, r, dtype, flags))


def hlq_conv2d_backward(G, X, Wt, geom, B, r, seed, flags, dX, dW, workspace=None):
    """Channels-last G [Nb, Ho, Wo, O], X [Nb, H, W, C], Wt [O, kh, kw, C] -> dX, dW of the same layouts."""
    ws_ptr, ws_bytes = (None, 0) if workspace is None else (_ptr(workspace), _nbytes(workspace))
    _check(lib().hlq_conv2d_backward(_ptr(G), _ptr(X), _ptr(Wt), C.byref(geom), B, r, seed, _dt(G), flags, _ptr(dX),
                                     _ptr(dW), ws_ptr, ws_bytes, _stream()), "hlq_conv2d_backward")


def hlq_backward_products_workspace_bytes(N, d_in, d_out, Kc, gx_bits, gw_int8=False) -> int:
    return int(lib().hlq_backward_products_workspace_bytes(N, d_in, d_out, Kc, gx_bits, int(bool(gw_int8))))


def hlq_backward_products_plan(N, d_in, d_out, Kc, gx_bits, gw_int8=False, workspace_bytes=1 << 28):
    """-> (tile_x, tile_w, splits_w, w_first, persistent): the layout hlq_backward_products would choose."""
    plan = (C.c_int * 5)()
    _check(lib().hlq_backward_products_plan(N, d_in, d_out, Kc, gx_bits, int(bool(gw_int8)), workspace_bytes, plan),
           "hlq_backward_products_plan")
    return tuple(int(v) for v in plan)


def hlq_backward_products(Gq, sG, WqT, sW, gx_bits, GhatT, sGhat, XhatT, sXhat, B, dX, dW, workspace=None):
    """Both matrix products of the pass in one launch, from the stored codes and projections."""
    N, d_in = dX.shape
    d_out, Kc = GhatT.shape
    ws_ptr, ws_bytes = (None, 0) if workspace is None else (_ptr(workspace), _nbytes(workspace))
    _check(lib().hlq_backward_products(_codes_ptr(Gq), _ptr(sG, torch.float32), _codes_ptr(WqT), _ptr(sW, torch.float32),
                                       gx_bits, _ptr(GhatT), _ptr(sGhat, torch.float32), _ptr(XhatT),
                                       _ptr(sXhat, torch.float32), N, d_in, d_out, Kc, B, _dt(dX), _ptr(dX), _ptr(dW),
                                       ws_ptr, ws_bytes, _stream()), "hlq_backward_products")
