"""GPU parity for the sequency-ordered basis of the g_w list (the r rows of H with the fewest
sign changes): coefficients, bf16 store, int8 codes and the whole path against the oracle, which
finds those rows by counting sign changes."""
import numpy as np
import pytest
import torch

import oracle
import paper_2406_15102_amd as hlq
from paper_2406_15102_amd import workloads as wl
from test_gpu_parity import same_up_to_split_order, TOL_OUT, dev, rand_tensor, row_rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
SEQ = hlq.HLQ_BASIS_SEQUENCY

CASES = [
    (256, 256, 16, 8, torch.float32), (416, 776, 16, 8, torch.bfloat16), (512, 136, 32, 4, torch.bfloat16),
    (512, 136, 32, 16, torch.bfloat16), (256, 72, 32, 32, torch.bfloat16), (512, 264, 64, 32, torch.bfloat16),
    (256, 40, 64, 2, torch.float32), (128, 48, 16, 1, torch.float32), (4096, 40, 16, 8, torch.bfloat16),
]


@pytest.mark.parametrize("N,D,B,r,dtype", CASES)
def test_hla_project_sequency(N, D, B, r, dtype):
    if (N // B * r) % 8:
        pytest.skip("compressed axis not a multiple of 8")
    T = rand_tensor((N, D), dtype, seed=N + D + r, scale=1.0, spread=0.5)
    Kc = N // B * r
    out = torch.empty((D, Kc), dtype=torch.bfloat16, device=DEV)
    coeff = torch.empty((D, Kc), dtype=torch.float32, device=DEV)
    hlq.hlq_hla_project_basis(dev(T), B, r, SEQ, out, coeff)
    torch.cuda.synchronize()
    ref = oracle.hla_f32(wl.as_f32_numpy(T), B, r, oracle.BASIS_SEQUENCY)
    assert np.array_equal(coeff.cpu().numpy(), ref)
    assert np.array_equal(out.float().cpu().numpy().view(np.uint32), oracle.round_bf16(ref).view(np.uint32))
    if r < B:   # and it is not the natural-order selection
        nat = torch.empty_like(out)
        hlq.hlq_hla_project(dev(T), B, r, nat)
        assert not torch.equal(nat, out) or r == 1


@pytest.mark.parametrize("N,D,B,r,dtype,tensor", [(256, 256, 16, 8, torch.float32, 2), (416, 776, 16, 8, torch.bfloat16, 3),
                                                  (512, 136, 32, 4, torch.bfloat16, 2), (512, 264, 64, 32, torch.bfloat16, 3)])
def test_hla_quantize_sequency(N, D, B, r, dtype, tensor):
    T = rand_tensor((N, D), dtype, seed=N + D + r, scale=1.0, spread=0.5)
    Kc = N // B * r
    TqT = torch.empty((D, Kc), dtype=torch.int8, device=DEV)
    sT = torch.empty(D, dtype=torch.float32, device=DEV)
    ws = torch.empty(hlq.hlq_hla_quantize_workspace_bytes(D), dtype=torch.uint8, device=DEV)
    hlq.hlq_hla_quantize_basis(dev(T), B, r, SEQ, 31, tensor, TqT, sT, ws)
    torch.cuda.synchronize()
    ref_q, ref_s = oracle.quantize_rows(oracle.hla_f32(wl.as_f32_numpy(T), B, r, oracle.BASIS_SEQUENCY), 31, tensor, qmax=127)
    assert np.array_equal(sT.cpu().numpy().view(np.uint32), ref_s.view(np.uint32))
    assert int(np.count_nonzero(TqT.cpu().numpy() != ref_q)) == 0


SMALL = [
    wl.WORKLOADS["c1"],
    wl.scaled(wl.WORKLOADS["c2"], N=3136, d_in=264, d_out=512),
    wl.scaled(wl.WORKLOADS["c4_b32"], N=512, d_in=264, d_out=1376),
    wl.scaled(wl.WORKLOADS["c5_r4"], N=512, d_in=1032, d_out=512),
]


@pytest.mark.parametrize("extra", [0, hlq.HLQ_FLAG_GW_INT8])
@pytest.mark.parametrize("w", SMALL, ids=lambda w: "%s_N%d_B%d_r%d" % (w.name, w.N, w.B, w.r))
def test_backward_sequency_matches_oracle(w, extra):
    flags = hlq.HLQ_FLAG_GW_SEQUENCY | extra
    t = wl.generate(w)
    G, X, W = dev(t["G"]), dev(t["X"]), dev(t["W"])
    N, I, O, B, r = w.N, w.d_in, w.d_out, w.B, w.r
    dX = torch.empty((N, I), dtype=G.dtype, device=DEV)
    dW = torch.empty((O, I), dtype=G.dtype, device=DEV)
    ws = torch.empty(hlq.hlq_workspace_bytes_mode(N, I, O, B, r, False, flags), dtype=torch.uint8, device=DEV)
    hlq.hlq_linear_backward_mode(G, X, None, None, W, N, I, O, B, r, w.seed, flags, dX, dW, ws)
    torch.cuda.synchronize()
    ref = oracle.linear_backward_mode(wl.as_f32_numpy(t["G"]), wl.as_f32_numpy(t["X"]), wl.as_f32_numpy(t["W"]), B, r,
                                      w.seed, gw_int8=bool(extra), basis=oracle.BASIS_SEQUENCY)
    bf = w.dtype == "bf16"
    ex = row_rel_err(dX.float().cpu().numpy(), ref["dX"], bf)
    ew = row_rel_err(dW.float().cpu().numpy(), ref["dW"], bf)
    print("%s flags=%d: dX err %.3e  dW err %.3e" % (w.name, flags, ex, ew))
    assert ex < TOL_OUT and ew < TOL_OUT
    # a forward-time store made with the same basis gives the same bits
    if not extra:
        XhT = torch.empty((I, N // B * r), dtype=torch.bfloat16, device=DEV)
        hlq.hlq_hla_project_basis(X, B, r, SEQ, XhT)
        dX2, dW2 = torch.empty_like(dX), torch.empty_like(dW)
        hlq.hlq_linear_backward_mode(G, None, XhT, None, W, N, I, O, B, r, w.seed, flags, dX2, dW2, ws)
        torch.cuda.synchronize()
        assert torch.equal(dW, dW2) and torch.equal(dX, dX2)
        hlq.hlq_linear_backward_mode(G, None, XhT, None, W, N, I, O, B, r, w.seed, flags, None, dW2, ws)
        torch.cuda.synchronize()
        assert same_up_to_split_order(dW2, dW)     # dW alone may split its reduction differently
