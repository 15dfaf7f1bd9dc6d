"""ctypes front-end of ``hlq_oracle.c`` -- TEST INFRASTRUCTURE, not product code.

Every function takes and returns numpy arrays (fp32 inputs; bf16 data is passed
widened to fp32, which is exact) and calls straight into the C file next to it.
Section/equation references are those of arXiv 2406.15102.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hlq_oracle.c")
_LIB = os.path.join(_HERE, "libhlq_oracle.so")

TENSOR_G, TENSOR_W, TENSOR_XHAT, TENSOR_GHAT = 0, 1, 2, 3   # random-stream ids of the four quantised operands

__all__ = [
    "TENSOR_G", "TENSOR_W", "TENSOR_XHAT", "TENSOR_GHAT", "linear_backward_mode",
    "build", "num_threads", "hadamard", "coeff_f32", "coeff_f64", "transform_rows",
    "transform_cols", "stream_key", "rand_word", "rand_byte", "quantize_one", "quantize_rows",
    "int_gemm_nt", "dequant", "hla_f32", "hla_f64", "round_bf16", "gemm_nt_f64",
    "linear_backward", "BASIS_NATURAL", "BASIS_SEQUENCY", "basis_rows", "ROUND_COUNTER", "ROUND_MANTISSA",
    "quantize_one_mantissa", "conv_out_size", "im2col", "col2im", "conv2d_backward", "pack_nibbles",
]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over independent rows, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        i8p, f32p, f64p, i32p = (C.POINTER(C.c_int8), C.POINTER(C.c_float), C.POINTER(C.c_double),
                                 C.POINTER(C.c_int32))
        lib.hlqo_num_threads.restype = C.c_int
        lib.hlqo_hadamard.argtypes = [C.c_int, i8p]
        lib.hlqo_coeff_f32.argtypes = [C.c_int, f32p, C.c_long, C.c_int, f32p]
        lib.hlqo_coeff_f64.argtypes = [C.c_int, f32p, C.c_long, C.c_int, f64p]
        lib.hlqo_transform_rows.argtypes = [f32p, C.c_long, C.c_long, C.c_int, f32p]
        lib.hlqo_transform_cols.argtypes = [f32p, C.c_long, C.c_long, C.c_int, f32p]
        lib.hlqo_stream_key.argtypes = [C.c_uint64, C.c_uint32]
        lib.hlqo_stream_key.restype = C.c_uint64
        lib.hlqo_rand_word.argtypes = [C.c_uint64, C.c_uint32]
        lib.hlqo_rand_word.restype = C.c_uint32
        lib.hlqo_rand_byte.argtypes = [C.c_uint64, C.c_long, C.c_long, C.c_long]
        lib.hlqo_rand_byte.restype = C.c_uint32
        lib.hlqo_quantize_one.argtypes = [C.c_float, C.c_float, C.c_uint32]
        lib.hlqo_quantize_one.restype = C.c_int8
        lib.hlqo_quantize_rows.argtypes = [f32p, C.c_long, C.c_long, C.c_uint64, C.c_uint32, i8p, f32p]
        lib.hlqo_quantize_rows_q.argtypes = [f32p, C.c_long, C.c_long, C.c_uint64, C.c_uint32,
                                             C.POINTER(C.c_long), C.c_int, i8p, f32p]
        lib.hlqo_quantize_one_q.argtypes = [C.c_float, C.c_float, C.c_uint32, C.c_int]
        lib.hlqo_quantize_one_q.restype = C.c_int8
        lib.hlqo_int_gemm_nt.argtypes = [i8p, i8p, C.c_long, C.c_long, C.c_long, i32p]
        lib.hlqo_dequant.argtypes = [i32p, f32p, f32p, C.c_long, C.c_long, C.c_int, f64p]
        lib.hlqo_hla_f32.argtypes = [f32p, C.c_long, C.c_long, C.c_int, C.c_int, f32p]
        lib.hlqo_hla_f64.argtypes = [f32p, C.c_long, C.c_long, C.c_int, C.c_int, f64p]
        lib.hlqo_hla_basis_f32.argtypes = [f32p, C.c_long, C.c_long, C.c_int, C.c_int, C.c_int, f32p]
        lib.hlqo_hla_basis_f64.argtypes = [f32p, C.c_long, C.c_long, C.c_int, C.c_int, C.c_int, f64p]
        lib.hlqo_basis_rows.argtypes = [C.c_int, C.c_int, C.POINTER(C.c_int)]
        lib.hlqo_quantize_one_mantissa.argtypes = [C.c_float, C.c_float, C.c_int]
        lib.hlqo_quantize_one_mantissa.restype = C.c_int8
        lib.hlqo_quantize_rows_mantissa.argtypes = [f32p, C.c_long, C.c_long, C.c_int, i8p, f32p]
        lib.hlqo_round_bf16.argtypes = [C.c_float]
        lib.hlqo_round_bf16.restype = C.c_float
        lib.hlqo_round_bf16_array.argtypes = [f32p, C.c_long, f32p]
        lib.hlqo_round_bf16_array.restype = None
        lib.hlqo_gemm_nt_f64.argtypes = [f32p, f32p, C.c_long, C.c_long, C.c_long, C.c_double, f64p]
        lib.hlqo_linear_backward.argtypes = [f32p, f32p, f32p, C.c_long, C.c_long, C.c_long, C.c_int,
                                             C.c_int, C.c_uint64, f64p, f64p, i8p, f32p, i8p, f32p,
                                             i32p, f32p, f32p]
        _lib = lib
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct)) if a is not None else None


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i8(a):
    return np.ascontiguousarray(a, dtype=np.int8)


def _check(rc, what):
    if rc != 0:
        raise ValueError("%s: oracle rejected the arguments (rc=%d)" % (what, rc))


def num_threads() -> int:
    return int(_L().hlqo_num_threads())


def hadamard(B: int) -> np.ndarray:
    """+-1 Sylvester matrix of order B (Eq. 2 without the per-level 1/sqrt 2)."""
    H = np.zeros((B, B), dtype=np.int8)
    _check(_L().hlqo_hadamard(B, _p(H, C.c_int8)), "hadamard")
    return H


def coeff_f32(v, B: int, nout: int | None = None) -> np.ndarray:
    v = _f32(v)
    nout = B if nout is None else nout
    c = np.zeros(nout, dtype=np.float32)
    _check(_L().hlqo_coeff_f32(B, _p(v, C.c_float), 1, nout, _p(c, C.c_float)), "coeff_f32")
    return c


def coeff_f64(v, B: int, nout: int | None = None) -> np.ndarray:
    v = _f32(v)
    nout = B if nout is None else nout
    c = np.zeros(nout, dtype=np.float64)
    _check(_L().hlqo_coeff_f64(B, _p(v, C.c_float), 1, nout, _p(c, C.c_double)), "coeff_f64")
    return c


def transform_rows(G, B: int) -> np.ndarray:
    """G . H_O : block-diagonal transform along the contiguous (out-feature) axis."""
    G = _f32(G)
    N, O = G.shape
    out = np.empty_like(G)
    _check(_L().hlqo_transform_rows(_p(G, C.c_float), N, O, B, _p(out, C.c_float)), "transform_rows")
    return out


def transform_cols(W, B: int) -> np.ndarray:
    """(H_O^T . W)^T : transform along W's row (out-feature) axis, returned as [d_in, d_out]."""
    W = _f32(W)
    O, I = W.shape
    out = np.empty((I, O), dtype=np.float32)
    _check(_L().hlqo_transform_cols(_p(W, C.c_float), O, I, B, _p(out, C.c_float)), "transform_cols")
    return out


def stream_key(seed: int, tensor: int) -> int:
    return int(_L().hlqo_stream_key(seed, tensor))


def rand_word(key: int, counter: int) -> int:
    return int(_L().hlqo_rand_word(key, counter))


def rand_byte(key: int, row: int, pos: int, K: int) -> int:
    return int(_L().hlqo_rand_byte(key, row, pos, K))


def quantize_one(x: float, inv: float, byte: int, qmax: int = 7) -> int:
    return int(_L().hlqo_quantize_one_q(float(np.float32(x)), float(np.float32(inv)), byte, qmax))


ROUND_COUNTER, ROUND_MANTISSA = 0, 1


def quantize_one_mantissa(x: float, inv: float, qmax: int = 7) -> int:
    return int(_L().hlqo_quantize_one_mantissa(float(np.float32(x)), float(np.float32(inv)), qmax))


def quantize_rows(Cm, seed: int, tensor: int, row_ids=None, qmax: int = 7, rounding: int = 0):
    """Stochastic absmax quantiser, one scale per row -> (codes int8, scales fp32).

    rounding = ROUND_MANTISSA: the paper's pseudo-stochastic rounding from the low 11 mantissa bits
    of each value (seed, tensor and row_ids then play no part).

    qmax = 7: the 4-bit codes of the g_x path; qmax = 127: int8 codes (g_w path, 8-bit warm-up).
    tensor selects the random stream: 0 G, 1 W (g_x product); 2 projected X, 3 projected G (g_w).
    row_ids: indices of the given rows inside the full operand (they address the random bytes);
    default 0..rows-1."""
    Cm = _f32(Cm)
    rows, K = Cm.shape
    q = np.empty((rows, K), dtype=np.int8)
    s = np.empty(rows, dtype=np.float32)
    if rounding == ROUND_MANTISSA:
        _check(_L().hlqo_quantize_rows_mantissa(_p(Cm, C.c_float), rows, K, qmax, _p(q, C.c_int8), _p(s, C.c_float)),
               "quantize_rows_mantissa")
        return q, s
    ids = None
    if row_ids is not None:
        ids = np.ascontiguousarray(row_ids, dtype=np.int64)
        assert ids.shape == (rows,) and C.sizeof(C.c_long) == 8
    _check(_L().hlqo_quantize_rows_q(_p(Cm, C.c_float), rows, K, seed, tensor,
                                     ids.ctypes.data_as(C.POINTER(C.c_long)) if ids is not None else None,
                                     qmax, _p(q, C.c_int8), _p(s, C.c_float)), "quantize_rows")
    return q, s


def int_gemm_nt(A, Bm) -> np.ndarray:
    A, Bm = _i8(A), _i8(Bm)
    M, K = A.shape
    Nn, K2 = Bm.shape
    assert K == K2
    acc = np.empty((M, Nn), dtype=np.int32)
    _check(_L().hlqo_int_gemm_nt(_p(A, C.c_int8), _p(Bm, C.c_int8), M, Nn, K, _p(acc, C.c_int32)),
           "int_gemm_nt")
    return acc


def dequant(acc, sA, sB, B: int) -> np.ndarray:
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    sA, sB = _f32(sA), _f32(sB)
    M, Nn = acc.shape
    out = np.empty((M, Nn), dtype=np.float64)
    _check(_L().hlqo_dequant(_p(acc, C.c_int32), _p(sA, C.c_float), _p(sB, C.c_float), M, Nn, B,
                             _p(out, C.c_double)), "dequant")
    return out


BASIS_NATURAL, BASIS_SEQUENCY = 0, 1


def basis_rows(B: int, basis: int) -> np.ndarray:
    """Row of H kept as coefficient k: k itself (natural order), or the row with k sign changes."""
    rows = np.empty(B, dtype=np.int32)
    _check(_L().hlqo_basis_rows(B, basis, _p(rows, C.c_int)), "basis_rows")
    return rows


def hla_f32(T, B: int, r: int, basis: int = 0) -> np.ndarray:
    """First r Hadamard coefficients (in the order of `basis`) of every block of B tokens -> [D, N/B*r] fp32."""
    T = _f32(T)
    N, D = T.shape
    out = np.empty((D, N // B * r), dtype=np.float32)
    _check(_L().hlqo_hla_basis_f32(_p(T, C.c_float), N, D, B, r, basis, _p(out, C.c_float)), "hla_f32")
    return out


def hla_f64(T, B: int, r: int, basis: int = 0) -> np.ndarray:
    T = _f32(T)
    N, D = T.shape
    out = np.empty((D, N // B * r), dtype=np.float64)
    _check(_L().hlqo_hla_basis_f64(_p(T, C.c_float), N, D, B, r, basis, _p(out, C.c_double)), "hla_f64")
    return out


def round_bf16(x) -> np.ndarray:
    """Round fp32 values to the nearest bfloat16 (ties to even), returned widened to fp32."""
    x = _f32(x)
    y = np.empty_like(x)
    _L().hlqo_round_bf16_array(_p(x, C.c_float), x.size, _p(y, C.c_float))
    return y


def gemm_nt_f64(A, Bm, alpha: float = 1.0) -> np.ndarray:
    A, Bm = _f32(A), _f32(Bm)
    M, K = A.shape
    Nn, K2 = Bm.shape
    assert K == K2
    out = np.empty((M, Nn), dtype=np.float64)
    _check(_L().hlqo_gemm_nt_f64(_p(A, C.c_float), _p(Bm, C.c_float), M, Nn, K, alpha,
                                 _p(out, C.c_double)), "gemm_nt_f64")
    return out


def linear_backward(G, X, W, B: int, r: int, seed: int, want_dX: bool = True, want_dW: bool = True,
                    intermediates: bool = False):
    """The whole HLQ backward pass (Sec. 6.1, both six-stage lists) -> dict of fp64/int arrays."""
    G, X, W = _f32(G), _f32(X), _f32(W)
    N, O = G.shape
    N2, I = X.shape
    O2, I2 = W.shape
    assert N == N2 and O == O2 and I == I2
    Kc = N // B * r
    out = {}
    dX = np.empty((N, I), dtype=np.float64) if want_dX else None
    dW = np.empty((O, I), dtype=np.float64) if want_dW else None
    Gq = sG = Wq = sW = acc = gh = xh = None
    if intermediates and want_dX:
        Gq = np.empty((N, O), dtype=np.int8)
        sG = np.empty(N, dtype=np.float32)
        Wq = np.empty((I, O), dtype=np.int8)
        sW = np.empty(I, dtype=np.float32)
        acc = np.empty((N, I), dtype=np.int32)
    if intermediates and want_dW:
        gh = np.empty((O, Kc), dtype=np.float32)
        xh = np.empty((I, Kc), dtype=np.float32)
    rc = _L().hlqo_linear_backward(
        _p(G, C.c_float), _p(X, C.c_float), _p(W, C.c_float), N, I, O, B, r, seed,
        _p(dX, C.c_double), _p(dW, C.c_double), _p(Gq, C.c_int8), _p(sG, C.c_float),
        _p(Wq, C.c_int8), _p(sW, C.c_float), _p(acc, C.c_int32), _p(gh, C.c_float),
        _p(xh, C.c_float))
    _check(rc, "linear_backward")
    out.update(dX=dX, dW=dW, Gq=Gq, sG=sG, Wq=Wq, sW=sW, acc=acc, GhatT=gh, XhatT=xh)
    return out


def pack_nibbles(q) -> np.ndarray:
    """4-bit codes [rows, K] in [-7, 7] (K even) -> [rows, K/2] bytes, two codes to a byte: code 2b in
    the low nibble of byte b, code 2b+1 in the high nibble, each as a 4-bit two's-complement number --
    the storage format of the paper's int4 operands and of its int4 activation store (Sec. 6.1)."""
    q = np.asarray(q).astype(np.int16)
    assert q.ndim == 2 and q.shape[1] % 2 == 0 and np.max(np.abs(q), initial=0) <= 7
    lo = q[:, 0::2] & 0xF
    hi = q[:, 1::2] & 0xF
    return (lo | (hi << 4)).astype(np.uint8)


def linear_backward_mode(G, X, W, B: int, r: int, seed: int, gx_bits: int = 4, gw_int8: bool = False,
                         basis: int = 0, rounding: int = 0, xhat_bits: int = 8):
    """Both stage lists of Sec. 6.1 composed stage by stage, with the two options of the method:

    gx_bits = 8   the g_x codes use [-127, 127] (the int8 warm-up phase of Sec. 7) instead of 4 bits;
    gw_int8       the g_w list in full: the HLA-projected X and G are quantised to int8 (stages 2, 4),
                  multiplied in integers (stage 5) and dequantised (stage 6), instead of being kept
                  in bf16;
    basis         which r rows of H the g_w list keeps: 0 the first r in natural order, 1 the r of
                  lowest sequency;
    rounding      ROUND_COUNTER (seeded stream) or ROUND_MANTISSA (the paper's low-11-bit scheme), for
                  every quantiser of both lists.
    xhat_bits     with gw_int8: 8, or 4 -- the projected x is quantised to [-7, 7] instead of [-127, 127]
                  (same stream, same per-feature absmax scale), the form in which Sec. 6.1's activation
                  compression keeps it between the passes ("int4"); the projected g_o stays int8 and
                  the product is the same integer product.
    Returns a dict with dX, dW (fp64) and every intermediate."""
    G, X, W = _f32(G), _f32(X), _f32(W)
    qx = 7 if gx_bits == 4 else 127
    assert gx_bits in (4, 8)
    out = {}
    # g_x: 1. FWH(g_o) on O  2. Q  3. FWH(w) on O  4. Q  5. integer product  6. dequantise
    Gq, sG = quantize_rows(transform_rows(G, B), seed, TENSOR_G, qmax=qx, rounding=rounding)
    Wq, sW = quantize_rows(transform_cols(W, B), seed, TENSOR_W, qmax=qx, rounding=rounding)
    acc = int_gemm_nt(Gq, Wq)
    out.update(Gq=Gq, sG=sG, Wq=Wq, sW=sW, acc=acc, dX=dequant(acc, sG, sW, B))
    # g_w: 1. HLA(x) on L  2. Q8  3. HLA(g_o^T) on L  4. Q8  5. integer product  6. dequantise
    xh = hla_f32(X, B, r, basis)
    gh = hla_f32(G, B, r, basis)
    assert xhat_bits in (4, 8) and (gw_int8 or xhat_bits == 8)
    if gw_int8:
        Xq, sX = quantize_rows(xh, seed, TENSOR_XHAT, qmax=127 if xhat_bits == 8 else 7, rounding=rounding)
        Gq2, sG2 = quantize_rows(gh, seed, TENSOR_GHAT, qmax=127, rounding=rounding)
        accw = int_gemm_nt(Gq2, Xq)
        out.update(XqT=Xq, sX=sX, GqT=Gq2, sGhat=sG2, accw=accw, dW=dequant(accw, sG2, sX, B))
    else:
        xh, gh = round_bf16(xh), round_bf16(gh)
        out.update(XhatT=xh, GhatT=gh, dW=gemm_nt_f64(gh, xh, 1.0 / B))
    return out


# ---- convolution layers: the same products with the spatial positions as the sequence (Sec. 3.1) ----
# Tensors are channels-last: x [Nb, H, W, C], g [Nb, Ho, Wo, O], w [O, kh, kw, C].  Row t = (n, ho, wo)
# of the column matrix holds the receptive field of output position (ho, wo) of sample n, its
# columns ordered (ky, kx, c), which is the order of w's trailing axes; taps outside the image are 0.

def conv_out_size(size: int, k: int, stride: int, pad: int, dil: int) -> int:
    """Number of output positions along one spatial axis."""
    return (size + 2 * pad - dil * (k - 1) - 1) // stride + 1


def im2col(x, kh: int, kw: int, stride=(1, 1), pad=(0, 0), dil=(1, 1)) -> np.ndarray:
    """x [Nb, H, W, C] -> column matrix [Nb*Ho*Wo, kh*kw*C] (same dtype), by the definition."""
    x = np.asarray(x)
    Nb, H, W, Cc = x.shape
    Ho = conv_out_size(H, kh, stride[0], pad[0], dil[0])
    Wo = conv_out_size(W, kw, stride[1], pad[1], dil[1])
    cols = np.zeros((Nb, Ho, Wo, kh, kw, Cc), dtype=x.dtype)
    for ky in range(kh):
        for kx in range(kw):
            for ho in range(Ho):
                hi = ho * stride[0] - pad[0] + ky * dil[0]
                if hi < 0 or hi >= H:
                    continue
                for wo in range(Wo):
                    wi = wo * stride[1] - pad[1] + kx * dil[1]
                    if 0 <= wi < W:
                        cols[:, ho, wo, ky, kx, :] = x[:, hi, wi, :]
    return cols.reshape(Nb * Ho * Wo, kh * kw * Cc)


def col2im(cols, x_shape, kh: int, kw: int, stride=(1, 1), pad=(0, 0), dil=(1, 1)) -> np.ndarray:
    """Adjoint of im2col: every entry of the column matrix is added to the pixel it was copied from
    (fp64 sums) -> [Nb, H, W, C]."""
    Nb, H, W, Cc = x_shape
    Ho = conv_out_size(H, kh, stride[0], pad[0], dil[0])
    Wo = conv_out_size(W, kw, stride[1], pad[1], dil[1])
    cols = np.asarray(cols, dtype=np.float64).reshape(Nb, Ho, Wo, kh, kw, Cc)
    dx = np.zeros((Nb, H, W, Cc), dtype=np.float64)
    for ky in range(kh):
        for kx in range(kw):
            for ho in range(Ho):
                hi = ho * stride[0] - pad[0] + ky * dil[0]
                if hi < 0 or hi >= H:
                    continue
                for wo in range(Wo):
                    wi = wo * stride[1] - pad[1] + kx * dil[1]
                    if 0 <= wi < W:
                        dx[:, hi, wi, :] += cols[:, ho, wo, ky, kx, :]
    return dx


def conv2d_backward(G4, X4, W4, B: int, r: int, seed: int, stride=(1, 1), pad=(0, 0), dil=(1, 1), **mode):
    """HLQ backward pass of a convolution: column matrix of x, both stage lists of Sec. 6.1 on
    (g [N, O], columns [N, kh*kw*C], w [O, kh*kw*C]) with N = Nb*Ho*Wo, then the column gradient
    folded back onto the image.  Returns linear_backward_mode's dict plus dX_img, dW_k."""
    G4, X4, W4 = _f32(G4), _f32(X4), _f32(W4)
    O, kh, kw, Cc = W4.shape
    out = linear_backward_mode(G4.reshape(-1, O), im2col(X4, kh, kw, stride, pad, dil), W4.reshape(O, -1),
                               B, r, seed, **mode)
    out["dX_img"] = col2im(out["dX"], X4.shape, kh, kw, stride, pad, dil)
    out["dW_k"] = out["dW"].reshape(O, kh, kw, Cc)
    return out
