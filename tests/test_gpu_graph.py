"""The whole backward pass under HIP graph capture: with a caller-owned workspace the entry point
allocates nothing, synchronises nothing and records no memset, so a caller may capture it once and
replay it.  Every replay is checked against the eager result, with eager work in between."""
import pytest
import torch

import paper_2406_15102_amd as hlq
from paper_2406_15102_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_backward_replays_from_a_captured_graph():
    w = wl.scaled(wl.WORKLOADS["c4"], N=512, d_in=520, d_out=1376)
    t = wl.generate(w)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    N, I, O, B, r = w.N, w.d_in, w.d_out, w.B, w.r
    ws = torch.empty(hlq.hlq_workspace_bytes(N, I, O, B, r), dtype=torch.uint8, device=DEV)
    dX_e = torch.empty((N, I), dtype=torch.bfloat16, device=DEV)
    dW_e = torch.empty((O, I), dtype=torch.bfloat16, device=DEV)
    hlq.hlq_linear_backward_ex(G, X, None, W, N, I, O, B, r, 3, dX_e, dW_e, ws)   # eager reference (also warms up)
    torch.cuda.synchronize()

    dX_g = torch.zeros_like(dX_e)
    dW_g = torch.zeros_like(dW_e)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        with torch.cuda.graph(graph, stream=s):
            hlq.hlq_linear_backward_ex(G, X, None, W, N, I, O, B, r, 3, dX_g, dW_g, ws)
    torch.cuda.current_stream().wait_stream(s)
    for rep in range(4):
        dX_g.zero_()
        dW_g.zero_()
        ws.random_(0, 255)                       # eager work that scribbles over the scratch memory
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(dX_g, dX_e) and torch.equal(dW_g, dW_e), "replay %d differs from the eager result" % rep


def test_plain_call_on_a_registered_workspace_is_capturable():
    """hlq_set_workspace, then the plain 12-argument call straight under stream capture -- no eager
    call of that size first: it may not allocate, free or synchronise, or the capture fails."""
    w = wl.scaled(wl.WORKLOADS["c4"], N=384, d_in=264, d_out=1120)
    t = wl.generate(w)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    N, I, O, B, r = w.N, w.d_in, w.d_out, w.B, w.r
    need = hlq.hlq_workspace_bytes(N, I, O, B, r)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    dX_e = torch.empty((N, I), dtype=torch.bfloat16, device=DEV)
    dW_e = torch.empty((O, I), dtype=torch.bfloat16, device=DEV)
    hlq.hlq_linear_backward_ex(G, X, None, W, N, I, O, B, r, 5, dX_e, dW_e, ws)   # reference, caller workspace
    torch.cuda.synchronize()
    reg = torch.empty(need, dtype=torch.uint8, device=DEV)
    dX_g, dW_g = torch.zeros_like(dX_e), torch.zeros_like(dW_e)
    try:
        small = torch.empty(4096, dtype=torch.uint8, device=DEV)
        hlq.hlq_set_workspace(small)
        with pytest.raises(hlq.HlqError) as ei:
            hlq.hlq_linear_backward(G, X, W, B, r, 5, dX_g, dW_g)
        assert ei.value.status == 6                      # too small: refused, nothing allocated behind the caller's back
        hlq.hlq_set_workspace(reg)
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(s):
            with torch.cuda.graph(graph, stream=s):
                hlq.hlq_linear_backward(G, X, W, B, r, 5, dX_g, dW_g)
        torch.cuda.current_stream().wait_stream(s)
        for rep in range(3):
            dX_g.zero_()
            dW_g.zero_()
            reg.random_(0, 255)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(dX_g, dX_e) and torch.equal(dW_g, dW_e), "replay %d differs from the eager result" % rep
    finally:
        hlq.hlq_set_workspace(None)
