"""A gradient tensor of more than 2^32 bytes and 2^32 elements' worth of offsets: every kernel of the
path must index in 64 bits.  G [262144, 16384] bf16 (8.6 GB) is drawn on the GPU from a seeded
generator; the oracle recomputes sampled token rows of dX and sampled out-feature rows of dW from
scratch, the first and last rows and those around the 2^31-element boundary included."""
import numpy as np
import pytest
import torch

import oracle
import paper_2406_15102_amd as hlq
from paper_2406_15102_amd import workloads as wl
from test_gpu_parity import TOL_OUT, row_rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_whole_path_beyond_32_bit_offsets():
    N, I, O, B, r, seed = 262144, 256, 16384, 16, 8, 17
    Kc = N // B * r
    assert N * O >= 2 ** 32 and Kc == 131072
    free, _ = torch.cuda.mem_get_info()
    if free < 40 * 2 ** 30:
        pytest.skip("needs 40 GB of free device memory")
    gen = torch.Generator(device=DEV)
    gen.manual_seed(1234)
    G = torch.empty((N, O), dtype=torch.bfloat16, device=DEV)
    for a in range(0, N, 16384):           # in slabs: no fp32 copy of the whole tensor
        G[a:a + 16384] = (torch.randn((16384, O), device=DEV, generator=gen) * 1e-3).to(torch.bfloat16)
    X = torch.randn((N, I), device=DEV, generator=gen).to(torch.bfloat16)
    W = (torch.randn((O, I), device=DEV, generator=gen) * 0.02).to(torch.bfloat16)
    dX = torch.empty((N, I), dtype=torch.bfloat16, device=DEV)
    dW = torch.empty((O, I), dtype=torch.bfloat16, device=DEV)
    need = hlq.hlq_workspace_bytes(N, I, O, B, r)
    assert need > 2 ** 32
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    print("large-index case N=%d d_in=%d d_out=%d workspace %.1f GB" % (N, I, O, need / 2 ** 30), flush=True)
    hlq.hlq_linear_backward_ex(G, X, None, W, N, I, O, B, r, seed, dX, dW, ws)
    torch.cuda.synchronize()
    assert torch.isfinite(dX.float()).all() and torch.isfinite(dW.float()).all()
    del ws

    Wn, Xn = wl.as_f32_numpy(W), wl.as_f32_numpy(X)
    # ---- dX on sampled token rows (rows whose element offsets straddle 2^31 among them; the last row ends at 2^32) ----
    rows = np.unique(np.array([0, 1, 15, 16, 2 ** 31 // O - 1, 2 ** 31 // O, N // 2 + 7, N - 17, N - 1]
                              + list(np.random.default_rng(3).integers(0, N, 12)), dtype=np.int64))
    assert rows.max() < N
    ridx = torch.from_numpy(rows).to(DEV)
    # plain slices, row by row (bounds-checked on the host, unlike an index kernel)
    Gs = wl.as_f32_numpy(torch.cat([G[int(i):int(i) + 1] for i in rows], dim=0))
    gq, sg = oracle.quantize_rows(oracle.transform_rows(Gs, B), seed, oracle.TENSOR_G, row_ids=rows)
    wq, sw = oracle.quantize_rows(oracle.transform_cols(Wn, B), seed, oracle.TENSOR_W)
    ref_dX = oracle.dequant(oracle.int_gemm_nt(gq, wq), sg, sw, B)
    ex = row_rel_err(dX[ridx].float().cpu().numpy(), ref_dX, True)
    # ---- dW on sampled out-feature rows: the whole token axis of those columns of G ----
    orows = np.unique(np.array([0, 1, 255, 256, O // 2, O - 257, O - 1] + list(np.random.default_rng(4).integers(0, O, 5)),
                               dtype=np.int64))
    oidx = torch.from_numpy(orows).to(DEV)
    # the sampled columns as plain strided slices, slab by slab (each slab well inside 32-bit offsets)
    Gcols = wl.as_f32_numpy(torch.cat(
        [torch.cat([G[a:a + 16384, int(j):int(j) + 1].float() for j in orows], dim=1) for a in range(0, N, 16384)], dim=0))
    gh = oracle.round_bf16(oracle.hla_f32(Gcols, B, r))
    xh = oracle.round_bf16(oracle.hla_f32(Xn, B, r))
    ref_dW = oracle.gemm_nt_f64(gh, xh, 1.0 / B)
    ew = row_rel_err(dW[oidx].float().cpu().numpy(), ref_dW, True)
    print("large-index case: dX err %.3e (%d rows)  dW err %.3e (%d rows)" % (ex, len(rows), ew, len(orows)))
    assert ex < TOL_OUT and ew < TOL_OUT
