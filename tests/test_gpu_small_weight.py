"""Weights of few rows are quantised inside the first launch of the path, both passes by one
workgroup per strip of columns.  The codes must be those of the stand-alone stage (two passes, many
workgroups), which the bit-exact parity tests pin to the oracle: the path given those codes returns
the same bits as the path that makes its own.  Shapes cover the three strip widths (up to 16, 32, 64
row blocks a round), several rounds, ragged last strips and rounds, every block order, both dtypes,
both code storages, and weights just past either limit, which take the other route."""
import numpy as np
import pytest
import torch

import oracle
import paper_2406_15102_amd as hlq
from paper_2406_15102_amd import workloads as wl
from test_gpu_parity import TOL_OUT, row_rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

#        N    d_in  d_out  B   r  dtype
CASES = [
    (256, 72, 64, 16, 8, "bf16"),       # 4 row blocks, one ragged strip of 128 columns
    (256, 264, 256, 16, 8, "bf16"),     # 16 row blocks: the widest strips, full
    (256, 264, 272, 16, 4, "f32"),      # 17: strips of 8 lanes
    (512, 200, 512, 16, 8, "bf16"),     # 32
    (256, 136, 528, 16, 8, "bf16"),     # 33: strips of 4 lanes
    (256, 104, 1024, 16, 8, "f32"),     # 64: one full round
    (256, 104, 1040, 16, 8, "bf16"),    # 65: a second round of one
    (256, 40, 2080, 16, 8, "bf16"),     # 130: three rounds
    (128, 72, 4096, 16, 8, "f32"),      # 256: the limit
    (128, 72, 4112, 16, 8, "bf16"),     # 257: past it
    (256, 520, 1024, 32, 8, "bf16"),    # B = 32, 32 row blocks
    (256, 40, 2048, 32, 16, "f32"),     # B = 32, 64 row blocks
    (256, 264, 1024, 64, 32, "bf16"),   # B = 64, 16 row blocks
    (128, 72, 4096, 64, 8, "bf16"),     # B = 64, 64 row blocks
    (128, 8200, 512, 16, 8, "bf16"),    # 8.4 MB: past the size limit
]


@pytest.mark.parametrize("flags", [0, hlq.HLQ_FLAG_GX_UNPACKED, hlq.HLQ_FLAG_GX_8BIT])
@pytest.mark.parametrize("N,I,O,B,r,dtype", CASES)
def test_codes_made_in_the_path_equal_the_stage_codes(N, I, O, B, r, dtype, flags):
    w = wl.scaled(wl.WORKLOADS["c2"], N=N, d_in=I, d_out=O, B=B, r=r, dtype=dtype)
    t = wl.generate(w)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    seed = 77
    ws = torch.empty(hlq.hlq_workspace_bytes_mode(N, I, O, B, r, False, flags), dtype=torch.uint8, device=DEV)
    dX0 = torch.empty((N, I), dtype=G.dtype, device=DEV)
    dW0 = torch.empty((O, I), dtype=G.dtype, device=DEV)
    hlq.hlq_linear_backward_mode(G, X, None, None, W, N, I, O, B, r, seed, flags, dX0, dW0, ws)
    bits = hlq.hlq_weight_code_bits(O, flags)
    WqT = torch.empty((I, O // 2 if bits == hlq.HLQ_BITS_4_PACKED else O), dtype=torch.uint8, device=DEV)
    sW = torch.empty(I, dtype=torch.float32, device=DEV)
    wws = torch.empty(hlq.hlq_quantize_w_workspace_bytes(O, I), dtype=torch.uint8, device=DEV)
    hlq.hlq_quantize_w(W, B, seed, WqT, sW, wws, None, bits)
    ws.fill_(0x5A)
    dX1, dW1 = torch.empty_like(dX0), torch.empty_like(dW0)
    hlq.hlq_linear_backward_cached(G, X, None, None, WqT, sW, N, I, O, B, r, seed, flags, dX1, dW1, ws)
    torch.cuda.synchronize()
    assert torch.equal(dX0, dX1) and torch.equal(dW0, dW1)
    if flags == 0:
        ref = oracle.linear_backward_mode(wl.as_f32_numpy(t["G"]), wl.as_f32_numpy(t["X"]), wl.as_f32_numpy(t["W"]), B, r, seed)
        assert row_rel_err(dX0.float().cpu().numpy(), ref["dX"], dtype == "bf16") < TOL_OUT


def test_zero_weight_columns_give_zero_scales_and_codes():
    """A column of zeros has maximum 0: scale 0 and codes 0, so those columns of dX are exactly 0."""
    N, I, O, B, r = 256, 136, 256, 16, 8
    w = wl.scaled(wl.WORKLOADS["c2"], N=N, d_in=I, d_out=O, B=B, r=r)
    t = wl.generate(w)
    W = t["W"].clone()
    W[:, 5] = 0
    W[:, 128:136] = 0
    G, X, W = t["G"].to(DEV).contiguous(), t["X"].to(DEV).contiguous(), W.to(DEV).contiguous()
    dX = torch.full((N, I), 7.0, dtype=G.dtype, device=DEV)
    dW = torch.empty((O, I), dtype=G.dtype, device=DEV)
    ws = torch.empty(hlq.hlq_workspace_bytes_mode(N, I, O, B, r, False, 0), dtype=torch.uint8, device=DEV)
    hlq.hlq_linear_backward_mode(G, X, None, None, W, N, I, O, B, r, 3, 0, dX, dW, ws)
    torch.cuda.synchronize()
    out = dX.float().cpu().numpy()
    assert np.all(out[:, 5] == 0) and np.all(out[:, 128:136] == 0) and np.any(out[:, :5] != 0)
