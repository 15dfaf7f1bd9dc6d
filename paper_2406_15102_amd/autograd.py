"""torch.autograd glue for the HLQ backward pass (arXiv 2406.15102, Sec. 6.1): vanilla forward,
activation compression at forward time (ACBP), both gradients from the C-ABI library.

This module only routes tensors: the forward product is torch's, everything of the backward pass
runs in the HIP kernels behind ``binding``.  Nothing here is needed by the library itself.
"""
from __future__ import annotations

import itertools

import torch

from . import binding as hlq

_layer_ids = itertools.count(1)


def _layer_seed(seed: int) -> int:
    """A rounding stream of its own for every layer object: the caller's seed plus the layer's
    number times an odd 64-bit constant (layers built in the same order get the same streams)."""
    return (int(seed) + next(_layer_ids) * 0x9E3779B97F4A7C15) & 0x7FFFFFFFFFFFFFFF


def _backward_workspace(N, d_in, d_out, B, r, flags, device):
    """Scratch of one backward pass as a torch tensor: the caching allocator orders its reuse on the
    stream, and the library call then allocates, frees and synchronises nothing."""
    need = hlq.hlq_workspace_bytes_mode(N, d_in, d_out, B, r, True, flags)
    if need == 0:
        raise ValueError("shape (N=%d, d_in=%d, d_out=%d, B=%d, r=%d, flags=%d) is outside the library's rules"
                         % (N, d_in, d_out, B, r, flags))
    return torch.empty(need, dtype=torch.uint8, device=device)


def _as_grad_dtype(w, dtype):
    """The weight in the element type of the incoming gradient (autocast hands a bf16 gradient to an
    fp32 parameter); the library reads every tensor of a call in one element type."""
    if dtype not in (torch.bfloat16, torch.float32):
        raise TypeError("gradient dtype must be bfloat16 or float32, got %s" % dtype)
    return w if w.dtype == dtype else w.to(dtype)


class HlqLinearFunction(torch.autograd.Function):
    """y = x @ w.T with the HLQ backward pass.

    x [..., d_in] and w [d_out, d_in] in bf16 or fp32 on the GPU.  Forward stores the compressed
    activation (the first r of every B token-axis Hadamard coefficients, bf16, or int8 codes with
    ``flags & HLQ_FLAG_GW_INT8``, or 4-bit codes with ``HLQ_FLAG_GW_INT8 | HLQ_FLAG_XC_INT4``: natural
    basis only) instead of x.  Backward returns dX = Q(G H) Q(H^T W) / B and
    dW = HLA(G)^T HLA(X) / B.  The number of tokens must be a multiple of B.
    """

    @staticmethod
    def forward(ctx, x, w, B=16, r=8, seed=0, flags=0):
        x2 = x.reshape(-1, x.shape[-1]).contiguous()
        N, d_in = x2.shape
        Kc = N // B * r
        basis = hlq.HLQ_BASIS_SEQUENCY if flags & hlq.HLQ_FLAG_GW_SEQUENCY else hlq.HLQ_BASIS_NATURAL
        if flags & hlq.HLQ_FLAG_XC_INT4:        # the paper's int4 store: 4-bit codes, two to a byte
            xc = torch.empty((d_in, Kc // 2), dtype=torch.uint8, device=x.device)
            sxc = torch.empty(d_in, dtype=torch.float32, device=x.device)
            ws = torch.empty(hlq.hlq_hla_quantize_workspace_bytes(d_in), dtype=torch.uint8, device=x.device)
            hlq.hlq_compress_act_int4(x2, B, r, seed, xc, sxc, ws)
        elif flags & hlq.HLQ_FLAG_GW_INT8:
            xc = torch.empty((d_in, Kc), dtype=torch.int8, device=x.device)
            sxc = torch.empty(d_in, dtype=torch.float32, device=x.device)
            ws = torch.empty(hlq.hlq_hla_quantize_workspace_bytes(d_in), dtype=torch.uint8, device=x.device)
            hlq.hlq_hla_quantize_basis(x2, B, r, basis, seed, 2, xc, sxc, ws)
        else:
            xc = torch.empty((d_in, Kc), dtype=torch.bfloat16, device=x.device)
            sxc = None
            hlq.hlq_hla_project_basis(x2, B, r, basis, xc)
        ctx.save_for_backward(xc, sxc, w)
        ctx.meta = (x.shape, N, d_in, w.shape[0], B, r, seed, flags)
        return torch.matmul(x, w.t())

    @staticmethod
    def backward(ctx, gy):
        xc, sxc, w = ctx.saved_tensors
        xshape, N, d_in, d_out, B, r, seed, flags = ctx.meta
        g2 = gy.reshape(N, d_out).contiguous()
        need_dx, need_dw = ctx.needs_input_grad[0], ctx.needs_input_grad[1]
        dX = torch.empty((N, d_in), dtype=g2.dtype, device=g2.device) if need_dx else None
        dW = torch.empty((d_out, d_in), dtype=g2.dtype, device=g2.device) if need_dw else None
        if need_dx or need_dw:
            ws = _backward_workspace(N, d_in, d_out, B, r, flags, g2.device)
            hlq.hlq_linear_backward_mode(g2, None, xc, sxc, _as_grad_dtype(w, g2.dtype).contiguous(), N, d_in, d_out,
                                         B, r, seed, flags, dX, dW, ws)
        if need_dw and dW.dtype != w.dtype:
            dW = dW.to(w.dtype)
        return (dX.reshape(xshape) if need_dx else None), dW, None, None, None, None


class HlqLinear(torch.nn.Module):
    """Bias-free linear layer trained with the HLQ backward pass; a fresh seed per call."""

    def __init__(self, d_in, d_out, B=16, r=8, flags=0, dtype=torch.bfloat16, device="cuda", seed=0):
        super().__init__()
        self.weight = torch.nn.Parameter(torch.randn((d_out, d_in), dtype=torch.float32, device=device).mul_(0.02).to(dtype))
        self.B, self.r, self.flags, self.seed, self.calls = B, r, flags, _layer_seed(seed), 0

    def forward(self, x):
        self.calls += 1
        return HlqLinearFunction.apply(x, self.weight, self.B, self.r, self.seed + self.calls, self.flags)


class HlqConv2dFunction(torch.autograd.Function):
    """y = conv2d(x, w) with the HLQ backward pass (Sec. 3.1: the spatial positions are the sequence).

    x [Nb, C, H, W] and w [O, C, kh, kw] in torch's channels_last memory format (other formats are
    converted), bf16 or fp32 on the GPU, groups = 1, no bias.  Forward keeps the compressed column
    matrix of x (as HlqLinearFunction keeps the compressed x), projected straight from the image when
    the channel count allows, else through a temporary column matrix; backward runs the
    two stage lists on (g, compressed columns, w) and folds the column gradient onto the image.
    Nb*Ho*Wo must be a multiple of B and kh*kw*C of 8.
    """

    @staticmethod
    def forward(ctx, x, w, stride=(1, 1), padding=(0, 0), dilation=(1, 1), B=16, r=8, seed=0, flags=0):
        Nb, Cc, H, W = x.shape
        O, _, kh, kw = w.shape
        x_l = x.permute(0, 2, 3, 1).contiguous()         # a view when x is channels_last
        geom = hlq.hlq_conv_geom(Nb=Nb, H=H, W=W, C=Cc, O=O, kh=kh, kw=kw, stride_h=stride[0], stride_w=stride[1],
                                 pad_h=padding[0], pad_w=padding[1], dil_h=dilation[0], dil_w=dilation[1])
        Ho, Wo, N, I = hlq.hlq_conv_sizes(geom)
        Kc = N // B * r
        pointwise = (kh, kw, tuple(stride), tuple(padding)) == (1, 1, (1, 1), (0, 0))
        from_image = not pointwise and Cc % (128 // B) == 0        # no column matrix is stored at all
        basis = hlq.HLQ_BASIS_SEQUENCY if flags & hlq.HLQ_FLAG_GW_SEQUENCY else hlq.HLQ_BASIS_NATURAL
        if not from_image:
            cols = x_l.reshape(N, I) if pointwise else torch.empty((N, I), dtype=x.dtype, device=x.device)
            if not pointwise:
                hlq.hlq_im2col(x_l, geom, cols)
        if flags & hlq.HLQ_FLAG_GW_INT8:
            xc = torch.empty((I, Kc), dtype=torch.int8, device=x.device)
            sxc = torch.empty(I, dtype=torch.float32, device=x.device)
            ws = torch.empty(hlq.hlq_hla_quantize_workspace_bytes(I), dtype=torch.uint8, device=x.device)
            if from_image:
                hlq.hlq_conv_compress_act_int8(x_l, geom, B, r, basis, seed, xc, sxc, ws)
            else:
                hlq.hlq_hla_quantize_basis(cols, B, r, basis, seed, 2, xc, sxc, ws)
        else:
            xc = torch.empty((I, Kc), dtype=torch.bfloat16, device=x.device)
            sxc = None
            if from_image:
                hlq.hlq_conv_compress_act(x_l, geom, B, r, basis, xc)
            else:
                hlq.hlq_hla_project_basis(cols, B, r, basis, xc)
        ctx.save_for_backward(xc, sxc, w)
        ctx.meta = (geom, (Nb, H, W, Cc), N, I, O, B, r, seed, flags, pointwise)
        return torch.nn.functional.conv2d(x, w, None, stride, padding, dilation)

    @staticmethod
    def backward(ctx, gy):
        xc, sxc, w = ctx.saved_tensors
        geom, xshape, N, I, O, B, r, seed, flags, pointwise = ctx.meta
        g2 = gy.permute(0, 2, 3, 1).contiguous().reshape(N, O)
        w_l = _as_grad_dtype(w, g2.dtype).permute(0, 2, 3, 1).contiguous().reshape(O, I)
        need_dx, need_dw = ctx.needs_input_grad[0], ctx.needs_input_grad[1]
        dcols = torch.empty((N, I), dtype=g2.dtype, device=g2.device) if need_dx else None
        dW = torch.empty((O, I), dtype=g2.dtype, device=g2.device) if need_dw else None
        dX = None
        if need_dx or need_dw:
            ws = _backward_workspace(N, I, O, B, r, flags, g2.device)
            hlq.hlq_linear_backward_mode(g2, None, xc, sxc, w_l, N, I, O, B, r, seed, flags, dcols, dW, ws)
        if need_dx:
            if pointwise:
                dX = dcols.reshape(xshape)
            else:
                dX = torch.empty(xshape, dtype=g2.dtype, device=g2.device)
                hlq.hlq_col2im(dcols, geom, dX)
            dX = dX.permute(0, 3, 1, 2)                  # [Nb, C, H, W], channels_last strides
        if need_dw:
            dW = dW.reshape(O, geom.kh, geom.kw, geom.C).permute(0, 3, 1, 2)
            if dW.dtype != w.dtype:
                dW = dW.to(w.dtype)
        return dX, dW, None, None, None, None, None, None, None


class HlqConv2d(torch.nn.Module):
    """Bias-free 2-D convolution trained with the HLQ backward pass; a fresh seed per call."""

    def __init__(self, c_in, c_out, kernel_size, stride=1, padding=0, dilation=1, B=16, r=8, flags=0,
                 dtype=torch.bfloat16, device="cuda", seed=0):
        super().__init__()
        pair = lambda v: (v, v) if isinstance(v, int) else tuple(v)   # noqa: E731
        kh, kw = pair(kernel_size)
        std = (2.0 / (c_in * kh * kw)) ** 0.5
        w = torch.randn((c_out, c_in, kh, kw), dtype=torch.float32, device=device).mul_(std).to(dtype)
        self.weight = torch.nn.Parameter(w.contiguous(memory_format=torch.channels_last))
        self.stride, self.padding, self.dilation = pair(stride), pair(padding), pair(dilation)
        self.B, self.r, self.flags, self.seed, self.calls = B, r, flags, _layer_seed(seed), 0

    def forward(self, x):
        self.calls += 1
        return HlqConv2dFunction.apply(x, self.weight, self.stride, self.padding, self.dilation, self.B, self.r,
                                       self.seed + self.calls, self.flags)
