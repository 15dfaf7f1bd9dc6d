"""torch.autograd glue for the HLQ backward pass (arXiv 2406.15102, Sec. 6.1): vanilla forward,
activation compression at forward time (ACBP), both gradients from the C-ABI library.

This module only routes tensors: the forward product is torch's, everything of the backward pass
runs in the HIP kernels behind ``binding``.  Nothing here is needed by the library itself.
"""
from __future__ import annotations

import torch

from . import binding as hlq


class HlqLinearFunction(torch.autograd.Function):
    """y = x @ w.T with the HLQ backward pass.

    x [..., d_in] and w [d_out, d_in] in bf16 or fp32 on the GPU.  Forward stores the compressed
    activation (the first r of every B token-axis Hadamard coefficients, bf16, or int8 codes with
    ``flags & HLQ_FLAG_GW_INT8``) instead of x.  Backward returns dX = Q(G H) Q(H^T W) / B and
    dW = HLA(G)^T HLA(X) / B.  The number of tokens must be a multiple of B.
    """

    @staticmethod
    def forward(ctx, x, w, B=16, r=8, seed=0, flags=0):
        x2 = x.reshape(-1, x.shape[-1]).contiguous()
        N, d_in = x2.shape
        Kc = N // B * r
        basis = hlq.HLQ_BASIS_SEQUENCY if flags & hlq.HLQ_FLAG_GW_SEQUENCY else hlq.HLQ_BASIS_NATURAL
        if flags & hlq.HLQ_FLAG_GW_INT8:
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
            hlq.hlq_linear_backward_mode(g2, None, xc, sxc, w.contiguous(), N, d_in, d_out, B, r, seed, flags, dX, dW)
        return (dX.reshape(xshape) if need_dx else None), dW, None, None, None, None


class HlqLinear(torch.nn.Module):
    """Bias-free linear layer trained with the HLQ backward pass; a fresh seed per call."""

    def __init__(self, d_in, d_out, B=16, r=8, flags=0, dtype=torch.bfloat16, device="cuda", seed=0):
        super().__init__()
        self.weight = torch.nn.Parameter(torch.randn((d_out, d_in), dtype=torch.float32, device=device).mul_(0.02).to(dtype))
        self.B, self.r, self.flags, self.seed, self.calls = B, r, flags, seed, 0

    def forward(self, x):
        self.calls += 1
        return HlqLinearFunction.apply(x, self.weight, self.B, self.r, self.seed + self.calls, self.flags)
