"""GPU parity for the paper's pseudo-stochastic rounding (low 11 mantissa bits of each value decide,
Sec. 6.1): codes and scales bit-exact against the oracle for every quantiser, whole path within the
usual bar."""
import numpy as np
import pytest
import torch

import oracle
import paper_2406_15102_amd as hlq
from paper_2406_15102_amd import workloads as wl
from test_gpu_packed import unpack_nibbles
from test_gpu_parity import TOL_OUT, dev, rand_tensor, row_rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
MANT = hlq.HLQ_BITS_ROUND_MANTISSA
RM = oracle.ROUND_MANTISSA


@pytest.mark.parametrize("N,O,B,dtype,bits", [(37, 256, 16, torch.float32, 4), (9, 11008, 32, torch.bfloat16, 0x104),
                                              (5, 8192, 64, torch.float32, 8), (300, 96, 16, torch.float32, 0x104)])
def test_quantize_g_mantissa_rounding(N, O, B, dtype, bits):
    G = rand_tensor((N, O), dtype, seed=N + O, scale=1e-3, spread=1.0)
    G[N // 2] = 0
    packed = bits == 0x104
    Gq = torch.empty((N, O // 2 if packed else O), dtype=torch.uint8 if packed else torch.int8, device=DEV)
    sG = torch.empty(N, dtype=torch.float32, device=DEV)
    hlq.hlq_quantize_g(dev(G), B, 21, Gq, sG, None, bits=bits | MANT)
    ref_q, ref_s = oracle.quantize_rows(oracle.transform_rows(wl.as_f32_numpy(G), B), 0, 0, qmax=127 if bits == 8 else 7,
                                        rounding=RM)
    got = unpack_nibbles(Gq.cpu().numpy()) if packed else Gq.cpu().numpy()
    assert np.array_equal(sG.cpu().numpy().view(np.uint32), ref_s.view(np.uint32))
    assert int(np.count_nonzero(got != ref_q)) == 0


@pytest.mark.parametrize("O,I,B,dtype,bits", [(1024, 776, 16, torch.float32, 0x104), (2112, 264, 64, torch.bfloat16, 4)])
def test_quantize_w_mantissa_rounding(O, I, B, dtype, bits):
    W = rand_tensor((O, I), dtype, seed=O + I, scale=0.02)
    packed = bits == 0x104
    WqT = torch.empty((I, O // 2 if packed else O), dtype=torch.uint8 if packed else torch.int8, device=DEV)
    sW = torch.empty(I, dtype=torch.float32, device=DEV)
    ws = torch.empty(hlq.hlq_quantize_w_workspace_bytes(O, I), dtype=torch.uint8, device=DEV)
    hlq.hlq_quantize_w(dev(W), B, 22, WqT, sW, ws, None, bits=bits | MANT)
    ref_q, ref_s = oracle.quantize_rows(oracle.transform_cols(wl.as_f32_numpy(W), B), 0, 1, rounding=RM)
    got = unpack_nibbles(WqT.cpu().numpy()) if packed else WqT.cpu().numpy()
    assert np.array_equal(sW.cpu().numpy().view(np.uint32), ref_s.view(np.uint32))
    assert int(np.count_nonzero(got != ref_q)) == 0


@pytest.mark.parametrize("N,D,B,r,dtype,basis", [(256, 256, 16, 8, torch.float32, 0), (416, 776, 16, 8, torch.bfloat16, 1)])
def test_hla_quantize_mantissa_rounding(N, D, B, r, dtype, basis):
    T = rand_tensor((N, D), dtype, seed=N + D + r, scale=1.0, spread=0.5)
    Kc = N // B * r
    TqT = torch.empty((D, Kc), dtype=torch.int8, device=DEV)
    sT = torch.empty(D, dtype=torch.float32, device=DEV)
    ws = torch.empty(hlq.hlq_hla_quantize_workspace_bytes(D), dtype=torch.uint8, device=DEV)
    hlq.hlq_hla_quantize_basis(dev(T), B, r, basis | hlq.HLQ_BASIS_ROUND_MANTISSA, 31, 2, TqT, sT, ws)
    torch.cuda.synchronize()
    ref_q, ref_s = oracle.quantize_rows(oracle.hla_f32(wl.as_f32_numpy(T), B, r, basis), 0, 2, qmax=127, rounding=RM)
    assert np.array_equal(sT.cpu().numpy().view(np.uint32), ref_s.view(np.uint32))
    assert int(np.count_nonzero(TqT.cpu().numpy() != ref_q)) == 0


SMALL = [wl.WORKLOADS["c1"], wl.scaled(wl.WORKLOADS["c2"], N=3136, d_in=264, d_out=512, dtype="f32")]


@pytest.mark.parametrize("extra", [0, hlq.HLQ_FLAG_GW_INT8])
@pytest.mark.parametrize("w", SMALL, ids=lambda w: "%s_N%d" % (w.name, w.N))
def test_backward_mantissa_rounding_matches_oracle(w, extra):
    flags = hlq.HLQ_FLAG_ROUND_MANTISSA | extra
    t = wl.generate(w)
    G, X, W = dev(t["G"]), dev(t["X"]), dev(t["W"])
    N, I, O, B, r = w.N, w.d_in, w.d_out, w.B, w.r
    dX = torch.empty((N, I), dtype=G.dtype, device=DEV)
    dW = torch.empty((O, I), dtype=G.dtype, device=DEV)
    ws = torch.empty(hlq.hlq_workspace_bytes_mode(N, I, O, B, r, False, flags), dtype=torch.uint8, device=DEV)
    hlq.hlq_linear_backward_mode(G, X, None, None, W, N, I, O, B, r, 12345, flags, dX, dW, ws)
    dX2, dW2 = torch.empty_like(dX), torch.empty_like(dW)
    hlq.hlq_linear_backward_mode(G, X, None, None, W, N, I, O, B, r, 999, flags, dX2, dW2, ws)   # the seed plays no part
    torch.cuda.synchronize()
    assert torch.equal(dX, dX2) and torch.equal(dW, dW2)
    ref = oracle.linear_backward_mode(wl.as_f32_numpy(t["G"]), wl.as_f32_numpy(t["X"]), wl.as_f32_numpy(t["W"]), B, r, 0,
                                      gw_int8=bool(extra), rounding=RM)
    ex = row_rel_err(dX.float().cpu().numpy(), ref["dX"], False)
    ew = row_rel_err(dW.float().cpu().numpy(), ref["dW"], False)
    print("%s flags=%d: dX err %.3e  dW err %.3e" % (w.name, flags, ex, ew))
    assert ex < 1e-5 and ew < (1e-5 if extra else TOL_OUT)
