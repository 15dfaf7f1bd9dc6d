"""The library's measurement switches (hlq_set_option) change how the work is laid out on the chip,
never what is computed: with either setting the whole path must give the same bits.  (That the
persistent form of the products is right against the oracle is checked by the full-size 70B-shaped
workloads, which take it by default.)"""
import pytest
import torch

import paper_2406_15102_amd as hlq
from paper_2406_15102_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run(w, G, X, W, seed=3, flags=0):
    N, I, O, B, r = w.N, w.d_in, w.d_out, w.B, w.r
    dX = torch.zeros((N, I), dtype=torch.bfloat16, device=DEV)
    dW = torch.zeros((O, I), dtype=torch.bfloat16, device=DEV)
    ws = torch.zeros(hlq.hlq_workspace_bytes_mode(N, I, O, B, r, False, flags), dtype=torch.uint8, device=DEV)
    hlq.hlq_linear_backward_mode(G, X, None, None, W, N, I, O, B, r, seed, flags, dX, dW, ws)
    torch.cuda.synchronize()
    return dX, dW


@pytest.mark.parametrize("B,r,flags", [(16, 8, 0), (32, 8, 0), (64, 32, 0), (16, 8, hlq.HLQ_FLAG_GW_INT8)])
def test_persistent_products_same_bits(B, r, flags):
    # 1024 + 128 tiles of 256 x 256 on 256 compute units: enough for the persistent form to be chosen
    w = wl.scaled(wl.WORKLOADS["c5_r8"], N=8192, d_in=8192, d_out=1024, B=B, r=r)
    t = wl.generate(w)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    try:
        hlq.hlq_set_option(hlq.HLQ_OPT_PERSISTENT_PRODUCTS, 0)
        dX0, dW0 = _run(w, G, X, W, flags=flags)
        hlq.hlq_set_option(hlq.HLQ_OPT_PERSISTENT_PRODUCTS, 1)
        dX1, dW1 = _run(w, G, X, W, flags=flags)
    finally:
        hlq.hlq_set_option(hlq.HLQ_OPT_PERSISTENT_PRODUCTS, 1)
    assert torch.equal(dX0, dX1) and torch.equal(dW0, dW1)
    assert float(dX1.float().abs().max()) > 0 and float(dW1.float().abs().max()) > 0


def test_persistent_products_ragged_edges_same_bits():
    # tiles that hang over both edges of either product (sizes that are no multiples of 256)
    w = wl.scaled(wl.WORKLOADS["c5_r8"], N=8192 - 64, d_in=8192 - 104, d_out=1024 + 64, B=32, r=16)
    t = wl.generate(w)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    try:
        hlq.hlq_set_option(hlq.HLQ_OPT_PERSISTENT_PRODUCTS, 0)
        dX0, dW0 = _run(w, G, X, W)
        hlq.hlq_set_option(hlq.HLQ_OPT_PERSISTENT_PRODUCTS, 1)
        dX1, dW1 = _run(w, G, X, W)
    finally:
        hlq.hlq_set_option(hlq.HLQ_OPT_PERSISTENT_PRODUCTS, 1)
    assert torch.equal(dX0, dX1) and torch.equal(dW0, dW1)


@pytest.mark.parametrize("B,r,N", [(16, 8, 2048), (32, 8, 2048 + 32), (64, 64, 2048), (16, 2, 2048 + 128)])
def test_shared_read_of_g_same_bits(B, r, N):
    # a G of 32 MB or more (the shared read is only taken for large tensors), token counts that are
    # and are not multiples of the 64-row groups
    w = wl.scaled(wl.WORKLOADS["c4"], N=N, d_in=1032, d_out=8192, B=B, r=r)   # a weight too large for the one-launch front
    t = wl.generate(w)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    try:
        hlq.hlq_set_option(hlq.HLQ_OPT_SHARED_G_READ, 0)
        dX0, dW0 = _run(w, G, X, W)
        hlq.hlq_set_option(hlq.HLQ_OPT_SHARED_G_READ, 1)
        dX1, dW1 = _run(w, G, X, W)
    finally:
        hlq.hlq_set_option(hlq.HLQ_OPT_SHARED_G_READ, 0)
    assert torch.equal(dX0, dX1) and torch.equal(dW0, dW1)


def test_unknown_option_is_refused():
    with pytest.raises(hlq.HlqError) as ei:
        hlq.hlq_set_option(99, 1)
    assert ei.value.status == 2
