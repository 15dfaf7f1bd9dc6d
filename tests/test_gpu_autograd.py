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
