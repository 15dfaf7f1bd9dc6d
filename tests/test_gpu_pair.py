"""The two matrix products in one launch against one launch each: dX must not change by a bit (same
tiles, same reduction order), dW only by the order in which its k splits are summed; both against
the oracle.  Shapes visit both tile sizes of either product, ragged k steps and split reductions."""
import numpy as np
import pytest
import torch

import oracle
import paper_2406_15102_amd as hlq
from paper_2406_15102_amd import workloads as wl
from test_gpu_parity import TOL_OUT, row_rel_err, same_up_to_split_order

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

CASES = [
    # N, d_in, d_out, B, r, dtype
    (1024, 264, 512, 16, 8, "bf16"),
    (4096, 768, 3072, 16, 8, "bf16"),      # both products under-fill the chip alone
    (12544, 576, 64, 16, 8, "bf16"),       # ragged k step of the g_x product, long split reduction of g_w
    (2048, 1152, 128, 16, 8, "bf16"),
    (512, 96, 224, 32, 16, "bf16"),        # d_out % 32 == 0 but ragged everywhere
    (256, 256, 256, 16, 8, "f32"),
    (1536, 200, 320, 64, 16, "f32"),
    (8192, 2048, 1024, 32, 4, "bf16"),
]


MODES = [0, hlq.HLQ_FLAG_GW_INT8, hlq.HLQ_FLAG_GX_8BIT, hlq.HLQ_FLAG_GX_UNPACKED | hlq.HLQ_FLAG_GW_INT8]


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("N,d_in,d_out,B,r,dtype", CASES)
def test_paired_products_equal_separate_ones(N, d_in, d_out, B, r, dtype, mode):
    w = wl.scaled(wl.WORKLOADS["c2"], N=N, d_in=d_in, d_out=d_out, B=B, r=r, dtype=dtype)
    t = wl.generate(w)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    if mode & hlq.HLQ_FLAG_GW_INT8 and (N // B * r) % 16:
        pytest.skip("the integer g_w list needs whole 16-byte rows of codes")
    ws = torch.empty(hlq.hlq_workspace_bytes_mode(N, d_in, d_out, B, r, False, mode), dtype=torch.uint8, device=DEV)
    SEP = mode | hlq.HLQ_FLAG_SEPARATE_PRODUCTS
    out = {}
    for flags in (mode, SEP):
        dX = torch.full((N, d_in), 7.0, dtype=G.dtype, device=DEV)
        dW = torch.full((d_out, d_in), 7.0, dtype=G.dtype, device=DEV)
        print("pair case", N, d_in, d_out, B, r, dtype, "flags", flags, flush=True)
        hlq.hlq_linear_backward_mode(G, X, None, None, W, N, d_in, d_out, B, r, 3, flags, dX, dW, ws)
        torch.cuda.synchronize()
        out[flags] = (dX, dW)
    assert torch.equal(out[mode][0], out[SEP][0])
    if mode & hlq.HLQ_FLAG_GW_INT8:
        assert torch.equal(out[mode][1], out[SEP][1])      # integer partial sums: exact in any order
    else:
        a, b = out[mode][1].float(), out[SEP][1].float()
        scale = float(b.abs().max())
        assert float((a - b).abs().max()) <= (2.0 ** -7 if dtype == "bf16" else 1e-5) * scale
    ref = oracle.linear_backward_mode(wl.as_f32_numpy(t["G"]), wl.as_f32_numpy(t["X"]), wl.as_f32_numpy(t["W"]), B, r, 3,
                                      gx_bits=8 if mode & hlq.HLQ_FLAG_GX_8BIT else 4,
                                      gw_int8=bool(mode & hlq.HLQ_FLAG_GW_INT8))
    bf = dtype == "bf16"
    for dX, dW in out.values():
        assert row_rel_err(dX.float().cpu().numpy(), ref["dX"], bf) < TOL_OUT
        assert row_rel_err(dW.float().cpu().numpy(), ref["dW"], bf) < TOL_OUT


def test_one_output_alone_takes_the_single_launches():
    N, d_in, d_out, B, r = 1024, 264, 512, 16, 8
    w = wl.scaled(wl.WORKLOADS["c2"], N=N, d_in=d_in, d_out=d_out, B=B, r=r)
    t = wl.generate(w)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    dX, dW = (torch.empty((N, d_in), dtype=G.dtype, device=DEV), torch.empty((d_out, d_in), dtype=G.dtype, device=DEV))
    hlq.hlq_linear_backward_mode(G, X, None, None, W, N, d_in, d_out, B, r, 3, 0, dX, dW)
    dX1, dW1 = torch.empty_like(dX), torch.empty_like(dW)
    hlq.hlq_linear_backward_mode(G, X, None, None, W, N, d_in, d_out, B, r, 3, 0, dX1, None)
    hlq.hlq_linear_backward_mode(G, X, None, None, W, N, d_in, d_out, B, r, 3, 0, None, dW1)
    torch.cuda.synchronize()
    assert torch.equal(dX, dX1)
    assert float((dW.float() - dW1.float()).abs().max()) <= 2.0 ** -7 * float(dW1.float().abs().max())


@pytest.mark.parametrize("gw_int8", [False, True])
@pytest.mark.parametrize("N,d_in,d_out,B,r,dtype", [CASES[0], CASES[1], CASES[5]])
def test_products_entry_point_equals_the_whole_path(N, d_in, d_out, B, r, dtype, gw_int8):
    """Stage entry points up to the stored codes and projections, then both products through
    hlq_backward_products: what the whole path computes."""
    w = wl.scaled(wl.WORKLOADS["c2"], N=N, d_in=d_in, d_out=d_out, B=B, r=r, dtype=dtype)
    t = wl.generate(w)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    Kc, seed = N // B * r, 3
    flags = hlq.HLQ_FLAG_GW_INT8 if gw_int8 else 0
    dX0 = torch.empty((N, d_in), dtype=G.dtype, device=DEV)
    dW0 = torch.empty((d_out, d_in), dtype=G.dtype, device=DEV)
    hlq.hlq_linear_backward_mode(G, X, None, None, W, N, d_in, d_out, B, r, seed, flags, dX0, dW0)
    bits = hlq.hlq_weight_code_bits(d_out, flags)
    cb = d_out // 2 if bits == hlq.HLQ_BITS_4_PACKED else d_out
    Gq = torch.empty((N, cb), dtype=torch.uint8, device=DEV)
    WqT = torch.empty((d_in, cb), dtype=torch.uint8, device=DEV)
    sG, sW = torch.empty(N, dtype=torch.float32, device=DEV), torch.empty(d_in, dtype=torch.float32, device=DEV)
    wws = torch.empty(hlq.hlq_quantize_w_workspace_bytes(d_out, d_in), dtype=torch.uint8, device=DEV)
    hlq.hlq_quantize_g(G, B, seed, Gq, sG, None, bits)
    hlq.hlq_quantize_w(W, B, seed, WqT, sW, wws, None, bits)
    if gw_int8:
        Gh, Xh = (torch.empty((d, Kc), dtype=torch.int8, device=DEV) for d in (d_out, d_in))
        sGh, sXh = (torch.empty(d, dtype=torch.float32, device=DEV) for d in (d_out, d_in))
        hws = torch.empty(hlq.hlq_hla_quantize_workspace_bytes(max(d_in, d_out)), dtype=torch.uint8, device=DEV)
        hlq.hlq_hla_quantize(G, B, r, seed, 3, Gh, sGh, hws)
        hlq.hlq_hla_quantize(X, B, r, seed, 2, Xh, sXh, hws)
    else:
        Gh, Xh = (torch.empty((d, Kc), dtype=torch.bfloat16, device=DEV) for d in (d_out, d_in))
        sGh = sXh = None
        hlq.hlq_hla_project(G, B, r, Gh)
        hlq.hlq_hla_project(X, B, r, Xh)
    pws = torch.empty(max(16, hlq.hlq_backward_products_workspace_bytes(N, d_in, d_out, Kc, bits, gw_int8)),
                      dtype=torch.uint8, device=DEV)
    dX1, dW1 = torch.full_like(dX0, 7.0), torch.full_like(dW0, 7.0)
    hlq.hlq_backward_products(Gq, sG, WqT, sW, bits, Gh, sGh, Xh, sXh, B, dX1, dW1, pws)
    torch.cuda.synchronize()
    assert torch.equal(dX0, dX1)
    assert torch.equal(dW0, dW1) if gw_int8 else same_up_to_split_order(dW1, dW0)
