"""GPU parity at the full sizes of the named workloads, in the launch configuration bench.py times
(whole path through hlq_linear_backward_ex with a caller workspace; stages through their entry
points).  The oracle cannot run the full matrix products in seconds, so:
  * the quantised operands (cheap for the oracle) are compared IN FULL, bit for bit;
  * dX is compared on sampled token rows and dW on sampled out-feature rows, each row computed by
    the oracle from scratch (transform, quantise with the row's own random bytes, integer product,
    dequantise / project, round, multiply);
  * properties that hold at any size are checked on everything: |code| <= 7, finite outputs.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2406_15102_amd as hlq
from paper_2406_15102_amd import workloads as wl
from test_gpu_parity import TOL_OUT, row_rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _sample(n, count, edges, seed):
    rng = np.random.default_rng(seed)
    e = [x for x in edges if 0 <= x < n]
    return np.unique(np.concatenate([e, rng.integers(0, n, count)])).astype(np.int64)


FULL = ["c2", "c3", "c4", "c4_b32", "c4_b64", "c5_r4", "c5_r8", "c5_r16"]


@pytest.mark.parametrize("name", FULL)
def test_full_size_workload_sampled(name):
    w = wl.WORKLOADS[name]
    N, I, O, B, r = w.N, w.d_in, w.d_out, w.B, w.r
    Kc = N // B * r
    t = wl.generate(w)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    dX = torch.empty((N, I), dtype=torch.bfloat16, device=DEV)
    dW = torch.empty((O, I), dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(hlq.hlq_workspace_bytes(N, I, O, B, r), dtype=torch.uint8, device=DEV)
    hlq.hlq_linear_backward_ex(G, X, None, W, N, I, O, B, r, w.seed, dX, dW, ws)
    torch.cuda.synchronize()
    assert torch.isfinite(dX.float()).all() and torch.isfinite(dW.float()).all()
    del ws

    Gn, Wn = wl.as_f32_numpy(t["G"]), wl.as_f32_numpy(t["W"])

    # ---- W operand in full: codes and scales bit-exact ----
    WqT = torch.empty((I, O), dtype=torch.int8, device=DEV)
    sW = torch.empty(I, dtype=torch.float32, device=DEV)
    wws = torch.empty(hlq.hlq_quantize_w_workspace_bytes(O, I), dtype=torch.uint8, device=DEV)
    hlq.hlq_quantize_w(W, B, w.seed, WqT, sW, wws)
    ref_Wq, ref_sW = oracle.quantize_rows(oracle.transform_cols(Wn, B), w.seed, 1)
    got_Wq = WqT.cpu().numpy()
    assert np.max(np.abs(got_Wq)) <= 7
    assert np.array_equal(sW.cpu().numpy().view(np.uint32), ref_sW.view(np.uint32))
    assert int(np.count_nonzero(got_Wq != ref_Wq)) == 0
    del WqT, got_Wq

    # ---- G operand in full ----
    Gq = torch.empty((N, O), dtype=torch.int8, device=DEV)
    sG = torch.empty(N, dtype=torch.float32, device=DEV)
    hlq.hlq_quantize_g(G, B, w.seed, Gq, sG)
    ref_Gq, ref_sG = oracle.quantize_rows(oracle.transform_rows(Gn, B), w.seed, 0)
    got_Gq = Gq.cpu().numpy()
    assert np.max(np.abs(got_Gq)) <= 7
    assert np.array_equal(sG.cpu().numpy().view(np.uint32), ref_sG.view(np.uint32))
    assert int(np.count_nonzero(got_Gq != ref_Gq)) == 0
    del Gq, got_Gq

    # ---- dX on sampled token rows (tile edges of the 256- and 128-row tiles, plus random rows) ----
    rows = _sample(N, 12, [0, 1, 127, 128, 255, 256, N - 257, N - 1], seed=1)
    gq_s, sg_s = oracle.quantize_rows(oracle.transform_rows(Gn[rows], B), w.seed, 0, row_ids=rows)
    assert np.array_equal(gq_s, ref_Gq[rows])
    acc = oracle.int_gemm_nt(gq_s, ref_Wq)
    assert np.max(np.abs(acc)) <= 49 * O
    ref_dX = oracle.dequant(acc, sg_s, ref_sW, B)
    ex = row_rel_err(dX[torch.from_numpy(rows).to(DEV)].float().cpu().numpy(), ref_dX, True, label=name + " dX")
    del ref_Gq, ref_Wq

    # ---- dW on sampled out-feature rows ----
    Xn = wl.as_f32_numpy(t["X"])
    xh = oracle.round_bf16(oracle.hla_f32(Xn, B, r))
    XhT = torch.empty((I, Kc), dtype=torch.bfloat16, device=DEV)
    hlq.hlq_compress_act(X, B, r, XhT)
    assert np.array_equal(XhT.float().cpu().numpy().view(np.uint32), xh.view(np.uint32))   # ACBP store, in full
    # the backward pass that consumes the store (how the 70B-shaped workload is meant to run): same bits
    ws = torch.empty(hlq.hlq_workspace_bytes(N, I, O, B, r, True), dtype=torch.uint8, device=DEV)
    dX2, dW2 = torch.empty_like(dX), torch.empty_like(dW)
    hlq.hlq_linear_backward_ex(G, None, XhT, W, N, I, O, B, r, w.seed, dX2, dW2, ws)
    torch.cuda.synchronize()
    assert torch.equal(dX2, dX) and torch.equal(dW2, dW)
    del ws, dX2, dW2
    orows = _sample(O, 12, [0, 1, 127, 128, 255, 256, O - 257, O - 1], seed=2)
    gh = oracle.round_bf16(oracle.hla_f32(np.ascontiguousarray(Gn[:, orows]), B, r))
    ref_dW = oracle.gemm_nt_f64(gh, xh, 1.0 / B)
    ew = row_rel_err(dW[torch.from_numpy(orows).to(DEV)].float().cpu().numpy(), ref_dW, True, label=name + " dW")
    print("%s: dX err %.3e (%d rows)  dW err %.3e (%d rows)" % (name, ex, len(rows), ew, len(orows)))
    assert ex < TOL_OUT and ew < TOL_OUT


PAPER_LAYERS = ["p%02d" % k for k in range(1, 13)]


@pytest.mark.parametrize("name", PAPER_LAYERS)
def test_paper_latency_table_layers_in_full(name):
    """The twelve layer shapes of the paper's latency table at batch 64: small enough for the oracle
    to compute the whole backward pass, odd enough (d_out = 64 ... 896, d_in = 64 ... 2304, up to
    65536 tokens) to visit tile and split plans the large workloads do not."""
    w = wl.WORKLOADS[name]
    N, I, O, B, r = w.N, w.d_in, w.d_out, w.B, w.r
    t = wl.generate(w)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    dX = torch.empty((N, I), dtype=torch.bfloat16, device=DEV)
    dW = torch.empty((O, I), dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(hlq.hlq_workspace_bytes(N, I, O, B, r), dtype=torch.uint8, device=DEV)
    hlq.hlq_linear_backward_ex(G, X, None, W, N, I, O, B, r, w.seed, dX, dW, ws)
    torch.cuda.synchronize()
    ref = oracle.linear_backward_mode(wl.as_f32_numpy(t["G"]), wl.as_f32_numpy(t["X"]), wl.as_f32_numpy(t["W"]), B, r, w.seed)
    ex = row_rel_err(dX.float().cpu().numpy(), ref["dX"], True)
    ew = row_rel_err(dW.float().cpu().numpy(), ref["dW"], True)
    print("%s: dX err %.3e  dW err %.3e" % (name, ex, ew))
    assert ex < TOL_OUT and ew < TOL_OUT


@pytest.mark.parametrize("name", sorted(wl.CONV_GEOMS))
def test_convolution_layers_in_full(name):
    """The ResNet-shaped workloads as real convolutions (channels-last image in, image gradient out),
    in the configuration bench.py times them, against the oracle's whole pass."""
    w = wl.WORKLOADS[name]
    Nb, H, Wd, C, kh, kw, st, pd = wl.CONV_GEOMS[name]
    O, B, r = w.d_out, w.B, w.r
    geom = hlq.hlq_conv_geom(Nb=Nb, H=H, W=Wd, C=C, O=O, kh=kh, kw=kw, stride_h=st, stride_w=st, pad_h=pd, pad_w=pd,
                             dil_h=1, dil_w=1)
    Ho, Wo, N, I = hlq.hlq_conv_sizes(geom)
    assert (N, I) == (w.N, w.d_in)
    t = wl.generate_conv(Nb, H, Wd, C, O, kh, kw, Ho, Wo, w.dtype)
    G, X, Wt = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    dX, dW = torch.empty_like(X), torch.empty_like(Wt)
    ws = torch.empty(hlq.hlq_conv_workspace_bytes(geom, B, r, hlq.HLQ_BF16, 0), dtype=torch.uint8, device=DEV)
    hlq.hlq_conv2d_backward(G, X, Wt, geom, B, r, w.seed, 0, dX, dW, ws)
    torch.cuda.synchronize()
    ref = oracle.conv2d_backward(wl.as_f32_numpy(t["G"]), wl.as_f32_numpy(t["X"]), wl.as_f32_numpy(t["W"]), B, r, w.seed,
                                 stride=(st, st), pad=(pd, pd))
    ex = row_rel_err(dX.float().cpu().numpy().reshape(-1, C), ref["dX_img"].reshape(-1, C), True)
    ew = row_rel_err(dW.float().cpu().numpy().reshape(O, I), ref["dW_k"].reshape(O, I), True)
    print("%s as a convolution: dX err %.3e  dW err %.3e" % (name, ex, ew))
    assert ex < TOL_OUT and ew < TOL_OUT
