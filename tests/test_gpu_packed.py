"""GPU parity for the packed storage of the 4-bit g_x codes (two codes to a byte, the paper's int4
operands of Sec. 6.1): the packed quantisers must produce the oracle's codes bit for bit, the
product on packed operands the oracle's integer accumulators, and the whole path the same dX as
with one int8 per code."""
import numpy as np
import pytest
import torch

import oracle
import paper_2406_15102_amd as hlq
from paper_2406_15102_amd import workloads as wl
from test_gpu_parity import same_up_to_split_order, dev, rand_tensor

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
P4 = hlq.HLQ_BITS_4_PACKED


def unpack_nibbles(b):
    """[rows, K/2] uint8 -> [rows, K] int8: code 2b = low nibble of byte b, code 2b+1 = high nibble."""
    b = b.astype(np.int16)
    lo = ((b & 15) ^ 8) - 8
    hi = (((b >> 4) & 15) ^ 8) - 8
    return np.stack([lo, hi], axis=-1).reshape(b.shape[0], -1).astype(np.int8)


def pack_nibbles(c):
    c = c.astype(np.int16) & 15
    return (c[:, 0::2] | (c[:, 1::2] << 4)).astype(np.uint8)


def test_pack_helpers_round_trip():
    c = np.arange(-8, 8, dtype=np.int8).reshape(1, 16).repeat(3, 0)
    assert np.array_equal(unpack_nibbles(pack_nibbles(c)), c)


@pytest.mark.parametrize("N,O,B,dtype", [(37, 256, 16, torch.bfloat16), (9, 11008, 32, torch.bfloat16),
                                         (5, 8192, 64, torch.float32), (300, 96, 16, torch.float32),
                                         (3, 40000 // 64 * 64, 64, torch.bfloat16)])
def test_quantize_g_packed_bit_exact(N, O, B, dtype):
    G = rand_tensor((N, O), dtype, seed=N + O, scale=1e-3, spread=1.0)
    G[N // 2] = 0
    Gq = torch.empty((N, O // 2), dtype=torch.uint8, device=DEV)
    sG = torch.empty(N, dtype=torch.float32, device=DEV)
    hlq.hlq_quantize_g(dev(G), B, 21, Gq, sG, None, bits=P4)
    ref_q, ref_s = oracle.quantize_rows(oracle.transform_rows(wl.as_f32_numpy(G), B), 21, 0)
    assert np.array_equal(sG.cpu().numpy().view(np.uint32), ref_s.view(np.uint32))
    assert int(np.count_nonzero(unpack_nibbles(Gq.cpu().numpy()) != ref_q)) == 0


@pytest.mark.parametrize("O,I,B,dtype", [(1024, 776, 16, torch.bfloat16), (2112, 264, 64, torch.bfloat16),
                                         (96, 520, 32, torch.float32)])
def test_quantize_w_packed_bit_exact(O, I, B, dtype):
    W = rand_tensor((O, I), dtype, seed=O + I, scale=0.02)
    WqT = torch.empty((I, O // 2), dtype=torch.uint8, device=DEV)
    sW = torch.empty(I, dtype=torch.float32, device=DEV)
    ws = torch.empty(hlq.hlq_quantize_w_workspace_bytes(O, I), dtype=torch.uint8, device=DEV)
    hlq.hlq_quantize_w(dev(W), B, 22, WqT, sW, ws, None, bits=P4)
    ref_q, ref_s = oracle.quantize_rows(oracle.transform_cols(wl.as_f32_numpy(W), B), 22, 1)
    assert np.array_equal(sW.cpu().numpy().view(np.uint32), ref_s.view(np.uint32))
    assert int(np.count_nonzero(unpack_nibbles(WqT.cpu().numpy()) != ref_q)) == 0


def test_packed_rows_need_32_codes():
    G = torch.zeros((16, 48), dtype=torch.float32, device=DEV)
    Gq = torch.empty((16, 24), dtype=torch.uint8, device=DEV)
    sG = torch.empty(16, dtype=torch.float32, device=DEV)
    with pytest.raises(hlq.HlqError):
        hlq.hlq_quantize_g(G, 16, 1, Gq, sG, None, bits=P4)


GEMM_CASES = [
    (256, 256, 128, False), (300, 260, 256, False), (100, 36, 352, False), (260, 132, 96, False),
    (700, 520, 640, False), (384, 3072, 6272, True), (130, 516, 11008, True),
    (72, 68, 131072, False), (72, 68, 131072, True),      # longest supported reduction: 256 * 49 * K still fits int32
    (300, 260, 64, False), (515, 200, 160, False), (260, 388, 256, False), (4096, 4096, 96, False),   # one k step
]


@pytest.mark.parametrize("M,Nn,K,split", GEMM_CASES)
def test_int4_gemm_exact(M, Nn, K, split):
    rng = np.random.default_rng(M + Nn + K)
    A = rng.integers(-7, 8, (M, K)).astype(np.int8)
    Bm = rng.integers(-7, 8, (Nn, K)).astype(np.int8)
    A[0], Bm[0] = 7, 7                                  # the extreme dot product 49 K
    sA = (rng.random(M) + 0.5).astype(np.float32)
    sB = (rng.random(Nn) + 0.5).astype(np.float32)
    ref = oracle.int_gemm_nt(A, Bm)
    assert ref[0, 0] == 49 * K
    A4, B4 = torch.from_numpy(pack_nibbles(A)).to(DEV), torch.from_numpy(pack_nibbles(Bm)).to(DEV)
    A8, B8 = torch.from_numpy(A).to(DEV), torch.from_numpy(Bm).to(DEV)
    sAd, sBd = torch.from_numpy(sA).to(DEV), torch.from_numpy(sB).to(DEV)
    ws = None
    if split:
        need = max(hlq.hlq_gemm_workspace_bytes(2, M, Nn, K), hlq.hlq_gemm_workspace_bytes(0, M, Nn, K))
        assert need > 0
        ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    acc = torch.empty((M, Nn), dtype=torch.int32, device=DEV)
    for out_dt in (torch.bfloat16, torch.float32):
        C4 = torch.empty((M, Nn), dtype=out_dt, device=DEV)
        C8 = torch.empty_like(C4)
        hlq.hlq_int4_gemm_nt(A4, B4, sAd, sBd, 1.0 / 16, C4, acc, ws)
        hlq.hlq_int8_gemm_nt(A8, B8, sAd, sBd, 1.0 / 16, C8, None, ws)
        torch.cuda.synchronize()
        assert int(np.count_nonzero(acc.cpu().numpy() != ref)) == 0
        assert torch.equal(C4, C8)                       # same integers, same epilogue: same bits
    want = oracle.dequant(ref, sA, sB, 16)
    assert np.max(np.abs(C4.cpu().numpy() - want) / np.abs(want).max()) < 1e-6


SMALL = [
    wl.WORKLOADS["c1"],
    wl.scaled(wl.WORKLOADS["c2"], N=3136, d_in=264, d_out=512),
    wl.scaled(wl.WORKLOADS["c4_b32"], N=512, d_in=264, d_out=1376),
    wl.scaled(wl.WORKLOADS["c5_r4"], N=512, d_in=1032, d_out=512),
]


@pytest.mark.parametrize("w", SMALL, ids=lambda w: "%s_N%d_O%d" % (w.name, w.N, w.d_out))
def test_backward_packed_equals_unpacked(w):
    t = wl.generate(w)
    G, X, W = dev(t["G"]), dev(t["X"]), dev(t["W"])
    N, I, O, B, r = w.N, w.d_in, w.d_out, w.B, w.r
    assert O % 32 == 0                                   # so the default path does pack
    ws = torch.empty(hlq.hlq_workspace_bytes_mode(N, I, O, B, r, False, 0), dtype=torch.uint8, device=DEV)
    out = []
    SEP = hlq.HLQ_FLAG_SEPARATE_PRODUCTS
    for flags in (0, hlq.HLQ_FLAG_GX_UNPACKED, SEP, SEP | hlq.HLQ_FLAG_GX_UNPACKED):
        dX = torch.empty((N, I), dtype=G.dtype, device=DEV)
        dW = torch.empty((O, I), dtype=G.dtype, device=DEV)
        hlq.hlq_linear_backward_mode(G, X, None, None, W, N, I, O, B, r, w.seed, flags, dX, dW, ws)
        torch.cuda.synchronize()
        out.append((dX, dW))
    # dX: the same bits however the codes are stored and however the products are launched
    assert all(torch.equal(out[0][0], o[0]) for o in out[1:])
    # dW does not depend on the code storage: with one launch per product it is the same launch; sharing
    # a launch with a differently stored g_x product may only change how its reduction is split
    assert torch.equal(out[2][1], out[3][1])
    assert same_up_to_split_order(out[0][1], out[2][1]) and same_up_to_split_order(out[1][1], out[2][1])


@pytest.mark.parametrize("flags", [0, hlq.HLQ_FLAG_GX_UNPACKED, hlq.HLQ_FLAG_GX_8BIT, hlq.HLQ_FLAG_GW_INT8])
@pytest.mark.parametrize("w", SMALL[:3], ids=lambda w: "%s_N%d_O%d" % (w.name, w.N, w.d_out))
def test_backward_with_cached_weight_codes(w, flags):
    """Weight quantised once by its stage entry point, then handed to the path: same bits as the
    path that quantises it itself (same seed, same codes)."""
    t = wl.generate(w)
    G, X, W = dev(t["G"]), dev(t["X"]), dev(t["W"])
    N, I, O, B, r = w.N, w.d_in, w.d_out, w.B, w.r
    ws = torch.empty(hlq.hlq_workspace_bytes_mode(N, I, O, B, r, False, flags), dtype=torch.uint8, device=DEV)
    dX0 = torch.empty((N, I), dtype=G.dtype, device=DEV)
    dW0 = torch.empty((O, I), dtype=G.dtype, device=DEV)
    hlq.hlq_linear_backward_mode(G, X, None, None, W, N, I, O, B, r, w.seed, flags, dX0, dW0, ws)
    bits = hlq.hlq_weight_code_bits(O, flags)
    assert bits == (8 if flags & hlq.HLQ_FLAG_GX_8BIT else (4 if flags & hlq.HLQ_FLAG_GX_UNPACKED else P4))
    WqT = torch.empty((I, O // 2 if bits == P4 else O), dtype=torch.uint8, device=DEV)
    sW = torch.empty(I, dtype=torch.float32, device=DEV)
    wws = torch.empty(hlq.hlq_quantize_w_workspace_bytes(O, I), dtype=torch.uint8, device=DEV)
    hlq.hlq_quantize_w(W, B, w.seed, WqT, sW, wws, None, bits)
    ws.fill_(0x5A)                                       # nothing of the first call may be reused
    dX1, dW1 = torch.empty_like(dX0), torch.empty_like(dW0)
    hlq.hlq_linear_backward_cached(G, X, None, None, WqT, sW, N, I, O, B, r, w.seed, flags, dX1, dW1, ws)
    torch.cuda.synchronize()
    assert torch.equal(dX0, dX1) and torch.equal(dW0, dW1)
    # dW alone needs no weight at all
    dW2 = torch.empty_like(dW0)
    hlq.hlq_linear_backward_cached(G, X, None, None, None, None, N, I, O, B, r, w.seed, flags, None, dW2, ws)
    torch.cuda.synchronize()
    assert same_up_to_split_order(dW2, dW0)             # the product alone may split its reduction differently
