"""The autograd wrapper hands the same tensors to the same entry point: its gradients must equal a
direct call bit for bit, and it must keep the compressed activation, not x."""
import pytest
import torch

import paper_2406_15102_amd as hlq
from paper_2406_15102_amd import workloads as wl
from paper_2406_15102_amd.autograd import HlqLinear, HlqLinearFunction

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("flags", [0, hlq.HLQ_FLAG_GW_INT8, hlq.HLQ_FLAG_GW_SEQUENCY])
def test_function_matches_direct_call(flags):
    w_ = wl.scaled(wl.WORKLOADS["c2"], N=1024, d_in=264, d_out=512)
    t = wl.generate(w_)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    N, I, O, B, r = w_.N, w_.d_in, w_.d_out, w_.B, w_.r
    x = X.reshape(4, N // 4, I).clone().requires_grad_(True)
    w = W.clone().requires_grad_(True)
    y = HlqLinearFunction.apply(x, w, B, r, 7, flags)
    assert torch.equal(y, torch.matmul(x.detach(), w.detach().t()))
    y.backward(G.reshape(4, N // 4, O))
    dX = torch.empty((N, I), dtype=G.dtype, device=DEV)
    dW = torch.empty((O, I), dtype=G.dtype, device=DEV)
    hlq.hlq_linear_backward_mode(G, X, None, None, W, N, I, O, B, r, 7, flags, dX, dW)
    torch.cuda.synchronize()
    assert torch.equal(x.grad.reshape(N, I), dX) and torch.equal(w.grad, dW)


def test_module_saves_the_compressed_activation():
    lin = HlqLinear(256, 512, B=16, r=8, device=DEV)
    x = torch.randn((512, 256), dtype=torch.bfloat16, device=DEV, requires_grad=True)
    saved = []
    with torch.autograd.graph.saved_tensors_hooks(lambda t: (saved.append(tuple(t.shape)), t)[1], lambda t: t):
        y = lin(x)
    assert (256, 512 // 16 * 8) in saved and (512, 256) not in saved[:1]      # XhatT [d_in, N/B*r], not x
    y.float().square().mean().backward()
    assert lin.weight.grad is not None and torch.isfinite(lin.weight.grad.float()).all()
    assert x.grad is not None and torch.isfinite(x.grad.float()).all()


@pytest.mark.parametrize("flags,stride,ksize,pad", [(0, (1, 1), 3, (1, 1)), (hlq.HLQ_FLAG_GW_INT8, (2, 2), 3, (1, 1)),
                                                    (0, (1, 1), 1, (0, 0))])
def test_convolution_function_matches_direct_call(flags, stride, ksize, pad):
    from paper_2406_15102_amd.autograd import HlqConv2dFunction
    Nb, H, W, C, O = 8, 16, 16, 32, 64
    geom = hlq.hlq_conv_geom(Nb=Nb, H=H, W=W, C=C, O=O, kh=ksize, kw=ksize, stride_h=stride[0], stride_w=stride[1],
                             pad_h=pad[0], pad_w=pad[1], dil_h=1, dil_w=1)
    Ho, Wo, N, I = hlq.hlq_conv_sizes(geom)
    t = wl.generate_conv(Nb, H, W, C, O, ksize, ksize, Ho, Wo, "bf16")
    G, X, Wt = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    x = X.permute(0, 3, 1, 2).detach().requires_grad_(True)          # NCHW shape over channels-last memory
    w = Wt.permute(0, 3, 1, 2).detach().requires_grad_(True)
    y = HlqConv2dFunction.apply(x, w, stride, pad, (1, 1), 16, 8, 3, flags)
    assert y.shape == (Nb, O, Ho, Wo)
    y.backward(G.permute(0, 3, 1, 2))
    dX, dW = torch.empty_like(X), torch.empty_like(Wt)
    hlq.hlq_conv2d_backward(G, X, Wt, geom, 16, 8, 3, flags, dX, dW)
    torch.cuda.synchronize()
    assert x.grad.shape == x.shape and w.grad.shape == w.shape
    assert torch.equal(x.grad.permute(0, 2, 3, 1), dX) and torch.equal(w.grad.permute(0, 2, 3, 1), dW)


def test_convolution_module_trains_a_step():
    from paper_2406_15102_amd.autograd import HlqConv2d
    conv = HlqConv2d(16, 32, 3, padding=1, device=DEV)
    x = torch.randn((4, 16, 8, 8), dtype=torch.bfloat16, device=DEV).contiguous(memory_format=torch.channels_last)
    x.requires_grad_(True)
    y = conv(x)
    ref = torch.nn.functional.conv2d(x.detach(), conv.weight.detach(), padding=1)
    assert torch.equal(y, ref)
    y.float().square().mean().backward()
    gw = torch.autograd.grad(torch.nn.functional.conv2d(x.detach(), conv.weight, padding=1).float().square().mean(),
                             conv.weight)[0]
    # half of the token-axis coefficients are kept: the gradient correlates with the exact one
    a, b = conv.weight.grad.float().flatten(), gw.float().flatten()
    assert torch.isfinite(a).all() and float(torch.dot(a, b) / (a.norm() * b.norm())) > 0.3
    assert x.grad is not None and x.grad.shape == x.shape and torch.isfinite(x.grad.float()).all()


def test_fp32_weight_with_bf16_gradient_is_cast_not_misread():
    """Under autocast the gradient arrives in bf16 while the parameter is fp32: the wrapper hands the
    library a bf16 copy of the weight (it reads every tensor of a call in one element type) and
    returns the weight gradient in the parameter's type."""
    w_ = wl.scaled(wl.WORKLOADS["c2"], N=512, d_in=264, d_out=256)
    t = wl.generate(w_)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    N, I, O, B, r = w_.N, w_.d_in, w_.d_out, w_.B, w_.r
    w32 = W.float().clone()                               # exactly the bf16 values, held in fp32

    xc = torch.empty((I, N // B * r), dtype=torch.bfloat16, device=DEV)
    hlq.hlq_compress_act(X, B, r, xc)
    ctx = type("Ctx", (), {})()
    ctx.saved_tensors = (xc, None, w32)
    ctx.meta = (X.shape, N, I, O, B, r, 11, 0)
    ctx.needs_input_grad = (True, True, False, False, False, False)
    dx, dw = HlqLinearFunction.backward(ctx, G)[:2]
    dX = torch.empty((N, I), dtype=torch.bfloat16, device=DEV)
    dW = torch.empty((O, I), dtype=torch.bfloat16, device=DEV)
    hlq.hlq_linear_backward_mode(G, X, None, None, W, N, I, O, B, r, 11, 0, dX, dW)
    torch.cuda.synchronize()
    assert dw.dtype == torch.float32 and torch.equal(dw, dW.float())
    assert torch.equal(dx, dX)
    with pytest.raises(TypeError):
        hlq.hlq_linear_backward_mode(G, X, None, None, W.float(), N, I, O, B, r, 11, 0, dX, dW)


def test_layers_draw_different_rounding_streams():
    a = HlqLinear(64, 64, device=DEV)
    b = HlqLinear(64, 64, device=DEV)
    assert a.seed != b.seed
