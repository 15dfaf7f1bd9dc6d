"""Seeded sweep of odd shapes and option combinations through the whole path against the oracle:
ragged tiles in every dimension, reductions that are not whole k steps, every block order, ranks
from 1 to B, both dtypes, every option flag.  Sizes are small enough for the oracle to compute each
case in full."""
import numpy as np
import pytest
import torch

import oracle
import paper_2406_15102_amd as hlq
from paper_2406_15102_amd import workloads as wl
from test_gpu_parity import TOL_OUT, row_rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        B = int(rng.choice([16, 32, 64]))
        r = int(2 ** rng.integers(0, int(np.log2(B)) + 1))
        nblk = int(rng.integers(1, 40))
        N = nblk * B
        if (N // B * r) % 8:
            continue
        d_out = B * int(rng.integers(1, 24))
        d_in = 8 * int(rng.integers(1, 60))
        dtype = "bf16" if rng.random() < 0.6 else "f32"
        flags = 0
        if rng.random() < 0.3:
            flags |= hlq.HLQ_FLAG_GX_8BIT
        if rng.random() < 0.3 and r % 4 == 0 and (N // B * r) % 16 == 0:
            flags |= hlq.HLQ_FLAG_GW_INT8
        if rng.random() < 0.3:
            flags |= hlq.HLQ_FLAG_GW_SEQUENCY
        if rng.random() < 0.2:
            flags |= hlq.HLQ_FLAG_GX_UNPACKED
        if rng.random() < 0.2:
            flags |= hlq.HLQ_FLAG_ROUND_MANTISSA
        out.append((N, d_in, d_out, B, r, dtype, flags, int(rng.integers(0, 2 ** 31))))
    return out


@pytest.mark.parametrize("N,d_in,d_out,B,r,dtype,flags,seed", _cases(40, 2024))
def test_random_shape_matches_oracle(N, d_in, d_out, B, r, dtype, flags, seed):
    w = wl.scaled(wl.WORKLOADS["c2"], N=N, d_in=d_in, d_out=d_out, B=B, r=r, dtype=dtype)
    t = wl.generate(w)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    dX = torch.empty((N, d_in), dtype=G.dtype, device=DEV)
    dW = torch.empty((d_out, d_in), dtype=G.dtype, device=DEV)
    ws = torch.empty(hlq.hlq_workspace_bytes_mode(N, d_in, d_out, B, r, False, flags), dtype=torch.uint8, device=DEV)
    assert ws.numel() > 0
    print("case N=%d d_in=%d d_out=%d B=%d r=%d %s flags=%d" % (N, d_in, d_out, B, r, dtype, flags), flush=True)
    hlq.hlq_linear_backward_mode(G, X, None, None, W, N, d_in, d_out, B, r, seed, flags, dX, dW, ws)
    torch.cuda.synchronize()
    ref = oracle.linear_backward_mode(
        wl.as_f32_numpy(t["G"]), wl.as_f32_numpy(t["X"]), wl.as_f32_numpy(t["W"]), B, r, seed,
        gx_bits=8 if flags & hlq.HLQ_FLAG_GX_8BIT else 4, gw_int8=bool(flags & hlq.HLQ_FLAG_GW_INT8),
        basis=1 if flags & hlq.HLQ_FLAG_GW_SEQUENCY else 0, rounding=1 if flags & hlq.HLQ_FLAG_ROUND_MANTISSA else 0)
    bf = dtype == "bf16"
    ex = row_rel_err(dX.float().cpu().numpy(), ref["dX"], bf)
    ew = row_rel_err(dW.float().cpu().numpy(), ref["dW"], bf)
    assert ex < TOL_OUT and ew < TOL_OUT
    if not bf:
        assert ex < 1e-5        # exact integer product: only the epilogue rounding differs
