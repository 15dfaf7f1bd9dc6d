"""GPU parity: every stage of the HIP path against the CPU oracle, element by element, through
the C ABI (python binding = argument marshalling only).

Bars: bit-exact for coefficients on the g_x path, scales, 4-bit codes and int32 accumulators;
<= 1e-5 (relative to the block norm) for fp32 HLA coefficients; <= 2e-2 for the final dX / dW,
as max_n |delta[n,:]|_inf / (|ref[n,:]|_2 / sqrt(cols)) (see row_rel_err for the bf16 output step).
"""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2406_15102_amd as hlq
from paper_2406_15102_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL_OUT = 2e-2


def same_up_to_split_order(a, b):
    """dW of one configuration against dW of another whose product split its reduction differently
    (the two products in one launch, or one launch each): the partial sums are the same fp32
    numbers added in another order, so the results agree to a few fp32 roundings of the largest
    term -- far inside one bf16 step of the largest entry."""
    a, b = a.float(), b.float()
    return float((a - b).abs().max()) <= 2.0 ** -7 * float(b.abs().max())


def row_rel_err(got, ref, bf16_out=False, label=None):
    """max over rows n of |delta[n,:]|_inf / (|ref[n,:]|_2 / sqrt(cols)).

    For a bf16 output each element is first allowed the round-to-nearest-even bound of its own final
    rounding: half a unit in the last place of the binade the exact value lies in,
    2^(floor(log2 |ref|) - 8), between 2^-9 |ref| and 2^-8 |ref| (times 1 + 2^-10 for the fp32
    arithmetic in front of the rounding, which can flip its direction).  A row whose entries span a
    wide range (outlier channels) otherwise exceeds any fixed fraction of the row rms by the output
    rounding alone, whoever computes it.  Rows whose reference is zero must be exactly zero.  The
    plain row-wise L2 ratio is checked against the same bar as well, with no allowance.
    With HLQ_PARITY_LOG=<file> every labelled call appends its two figures to that file."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    norm = np.linalg.norm(ref, axis=1)
    rms = norm / np.sqrt(ref.shape[1])
    d = np.abs(got - ref)
    if bf16_out:
        mag = np.abs(ref)
        half_ulp = np.where(mag > 0, 2.0 ** (np.floor(np.log2(np.where(mag > 0, mag, 1.0))) - 8), 0.0)
        d_allow = np.maximum(d - half_ulp * (1.0 + 2.0 ** -10), 0.0)
    else:
        d_allow = d
    dmax = np.max(d_allow, axis=1)
    if np.any(rms == 0):
        assert np.all(np.max(d, axis=1)[rms == 0] == 0)
    ok = rms > 0
    if not ok.any():
        return 0.0
    l2 = float(np.max(np.linalg.norm(got - ref, axis=1)[ok] / norm[ok]))
    linf = float(np.max(dmax[ok] / rms[ok]))
    log = os.environ.get("HLQ_PARITY_LOG")
    if log and label:
        with open(log, "a") as f:
            f.write("%s: max row |d|_inf/rms beyond the output rounding = %.3e, max row L2 ratio = %.3e, "
                    "max |d|_inf/rms with no allowance = %.3e\n"
                    % (label, linf, l2, float(np.max(np.max(d, axis=1)[ok] / rms[ok]))))
    return max(linf, l2)


def rand_tensor(shape, dtype, seed, scale=1.0, spread=0.0):
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(shape).astype(np.float32) * np.float32(scale)
    if spread:
        a *= np.exp(spread * rng.standard_normal((shape[0], 1))).astype(np.float32)
    return torch.from_numpy(a).to(dtype)


def dev(t):
    return t.to(DEV).contiguous()


# --------------------------------------------------------------------------------------------
# K1: rows of G -> coefficients, scales, codes
# --------------------------------------------------------------------------------------------
QG_CASES = [
    # N, d_out, B, dtype                     what the shape exercises
    (256, 256, 16, torch.float32),         # config 1; 8 lanes per row, 32 rows per workgroup
    (37, 256, 16, torch.bfloat16),         # ragged last workgroup
    (19, 3072, 16, torch.bfloat16),        # one wavefront per row, 6 chunks per lane
    (9, 11008, 16, torch.bfloat16),        # one workgroup per row, ragged chunk count (5.375 per lane)
    (9, 11008, 32, torch.bfloat16),
    (9, 11008, 64, torch.bfloat16),
    (5, 8192, 32, torch.float32),
    (33, 64, 64, torch.bfloat16),          # a single Hadamard block per row
    (3, 16384, 64, torch.bfloat16),        # largest row the 256-thread variant takes
    (3, 65536, 16, torch.bfloat16),        # largest supported row (1024-thread variant)
    (2, 20480, 32, torch.float32),
]


@pytest.mark.parametrize("N,O,B,dtype", QG_CASES)
def test_quantize_g_bit_exact(N, O, B, dtype):
    G = rand_tensor((N, O), dtype, seed=N * 7 + O, scale=1e-3, spread=1.0)
    G[N // 2] = 0                                   # a zero row: scale 0, codes 0
    if N > 2:
        G[1, :] = 0
        G[1, O // 3] = 1.0                          # a single non-zero
    seed = 12345
    Gq = torch.empty((N, O), dtype=torch.int8, device=DEV)
    sG = torch.empty(N, dtype=torch.float32, device=DEV)
    coeff = torch.empty((N, O), dtype=torch.float32, device=DEV)
    hlq.hlq_quantize_g(dev(G), B, seed, Gq, sG, coeff)
    torch.cuda.synchronize()
    ref_c = oracle.transform_rows(wl.as_f32_numpy(G), B)
    ref_q, ref_s = oracle.quantize_rows(ref_c, seed, 0)
    # exact equality of values (the sign of a zero coefficient is not part of the contract: it has
    # no effect on a code)
    assert np.array_equal(coeff.cpu().numpy(), ref_c), "coefficients differ"
    assert np.array_equal(sG.cpu().numpy().view(np.uint32), ref_s.view(np.uint32)), "scales differ"
    mism = int(np.count_nonzero(Gq.cpu().numpy() != ref_q))
    assert mism == 0, "%d code mismatches" % mism
    # and without the debug export the codes are the same
    Gq2 = torch.empty_like(Gq)
    hlq.hlq_quantize_g(dev(G), B, seed, Gq2, sG, None)
    assert torch.equal(Gq, Gq2)


# --------------------------------------------------------------------------------------------
# K1T: W -> transposed coefficients, per-in-feature scales, codes
# --------------------------------------------------------------------------------------------
QW_CASES = [
    (256, 256, 16, torch.float32),         # config 1
    (1024, 776, 16, torch.bfloat16),       # d_in not a multiple of the 512-column tile
    (11008, 136, 16, torch.bfloat16),      # 43 row tiles, ragged
    (2112, 264, 32, torch.bfloat16),       # ragged row tile (2112 = 8*256 + 64)
    (2112, 264, 64, torch.bfloat16),
    (320, 72, 64, torch.float32),
    (64, 8, 64, torch.bfloat16),           # smallest legal problem
]


@pytest.mark.parametrize("O,I,B,dtype", QW_CASES)
def test_quantize_w_bit_exact(O, I, B, dtype):
    W = rand_tensor((O, I), dtype, seed=O + 3 * I, scale=0.02)
    W[:, I // 2] = 0                                # a zero in-feature
    W[O // 3, 0] *= 40                              # an outlier
    seed = 777
    WqT = torch.empty((I, O), dtype=torch.int8, device=DEV)
    sW = torch.empty(I, dtype=torch.float32, device=DEV)
    coeffT = torch.empty((I, O), dtype=torch.float32, device=DEV)
    ws = torch.empty(hlq.hlq_quantize_w_workspace_bytes(O, I), dtype=torch.uint8, device=DEV)
    hlq.hlq_quantize_w(dev(W), B, seed, WqT, sW, ws, coeffT)
    torch.cuda.synchronize()
    ref_c = oracle.transform_cols(wl.as_f32_numpy(W), B)
    ref_q, ref_s = oracle.quantize_rows(ref_c, seed, 1)
    assert np.array_equal(coeffT.cpu().numpy().view(np.uint32), ref_c.view(np.uint32)), "coefficients differ"
    assert np.array_equal(sW.cpu().numpy().view(np.uint32), ref_s.view(np.uint32)), "scales differ"
    mism = int(np.count_nonzero(WqT.cpu().numpy() != ref_q))
    assert mism == 0, "%d code mismatches" % mism


# --------------------------------------------------------------------------------------------
# K2: int8 MFMA product, exact int32 accumulators, dequantising epilogue
# --------------------------------------------------------------------------------------------
def _codes(shape, seed):
    rng = np.random.default_rng(seed)
    return torch.from_numpy(rng.integers(-7, 8, size=shape).astype(np.int8))


GEMM_I8_CASES = [
    (768, 520, 3072),       # few tiles, long reduction: split over k when scratch is given
    (256, 256, 256),        # config 1
    (300, 260, 320),        # ragged M and Nn (128-tiles), K a multiple of 64
    (130, 132, 592),        # K = 9*64 + 16: ragged last k step
    (64, 8, 16),            # tiny
    (515, 1028, 11008),     # the LLaMA reduction length, 5 x 9 tiles
    (300, 260, 32), (515, 200, 48), (256, 384, 96), (1000, 136, 128),   # one k step: whole, ragged, every sub-step count
    (4096, 4096, 64),       # one k step on 256-tiles
]


@pytest.mark.parametrize("M,Nn,K", GEMM_I8_CASES)
def test_int8_gemm_accumulators_bit_exact(M, Nn, K):
    A, Bm = _codes((M, K), M + K), _codes((Nn, K), Nn + K + 1)
    rng = np.random.default_rng(5)
    sA = torch.from_numpy(rng.random(M).astype(np.float32) + 0.5)
    sB = torch.from_numpy(rng.random(Nn).astype(np.float32) + 0.5)
    acc = torch.empty((M, Nn), dtype=torch.int32, device=DEV)
    out = torch.empty((M, Nn), dtype=torch.float32, device=DEV)
    hlq.hlq_int8_gemm_nt(dev(A), dev(Bm), dev(sA), dev(sB), 1.0 / 16, out, acc)
    torch.cuda.synchronize()
    ref = oracle.int_gemm_nt(A.numpy(), Bm.numpy())
    assert np.array_equal(acc.cpu().numpy(), ref), "int32 accumulators differ"
    want = oracle.dequant(ref, sA.numpy(), sB.numpy(), 16)
    assert np.allclose(out.cpu().numpy(), want, rtol=3e-7, atol=0)
    outb = torch.empty((M, Nn), dtype=torch.bfloat16, device=DEV)
    hlq.hlq_int8_gemm_nt(dev(A), dev(Bm), dev(sA), dev(sB), 1.0 / 16, outb, None)
    assert row_rel_err(outb.float().cpu().numpy(), want, True) < TOL_OUT
    # with scratch the reduction may be split over several workgroups per tile: integer partial
    # sums are exact, so the result has to be the same bits
    need = hlq.hlq_gemm_workspace_bytes(0, M, Nn, K)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=DEV)
    out2 = torch.empty_like(out)
    hlq.hlq_int8_gemm_nt(dev(A), dev(Bm), dev(sA), dev(sB), 1.0 / 16, out2, None, ws)
    assert torch.equal(out, out2)
    outb2 = torch.empty_like(outb)
    hlq.hlq_int8_gemm_nt(dev(A), dev(Bm), dev(sA), dev(sB), 1.0 / 16, outb2, None, ws)
    assert torch.equal(outb, outb2)


def test_int8_gemm_large_tile_variant_sampled():
    # 4096 x 4096 output selects the 256 x 256 tile kernel; the oracle checks sampled rows of A
    # (first, last and random rows, so every row position within a tile edge is covered somewhere)
    M = Nn = 4096
    K = 592
    A, Bm = _codes((M, K), 1), _codes((Nn, K), 2)
    acc = torch.empty((M, Nn), dtype=torch.int32, device=DEV)
    hlq.hlq_int8_gemm_nt(dev(A), dev(Bm), None, None, 1.0, None, acc)
    torch.cuda.synchronize()
    rng = np.random.default_rng(3)
    rows = np.unique(np.concatenate([[0, 1, 31, 32, 127, 128, 255, 256, 4095], rng.integers(0, M, 40)]))
    ref = oracle.int_gemm_nt(A.numpy()[rows], Bm.numpy())
    assert np.array_equal(acc.cpu().numpy()[rows], ref)
    # all codes at the extreme: the largest accumulator magnitude, 49 K
    ones = torch.full((M, K), 7, dtype=torch.int8)
    hlq.hlq_int8_gemm_nt(dev(ones), dev(-ones), None, None, 1.0, None, acc)
    assert torch.all(acc == -49 * K)


# --------------------------------------------------------------------------------------------
# K3: token-axis HLA projection
# --------------------------------------------------------------------------------------------
HLA_CASES = [
    (256, 256, 16, 8, torch.float32),      # config 1
    (208, 776, 16, 8, torch.bfloat16),     # ragged feature tile and ragged token-block group
    (256, 136, 32, 4, torch.bfloat16),
    (256, 136, 32, 16, torch.bfloat16),
    (256, 72, 32, 32, torch.bfloat16),     # r = B: nothing dropped
    (512, 264, 64, 32, torch.bfloat16),
    (512, 264, 64, 2, torch.float32),
    (512, 8, 64, 1, torch.bfloat16),
    (4096, 40, 16, 8, torch.bfloat16),     # many token blocks
]


@pytest.mark.parametrize("N,D,B,r,dtype", HLA_CASES)
def test_hla_project(N, D, B, r, dtype):
    T = rand_tensor((N, D), dtype, seed=N + D + r, scale=1.0, spread=0.5)
    Kc = N // B * r
    ThatT = torch.empty((D, Kc), dtype=torch.bfloat16, device=DEV)
    coeffT = torch.empty((D, Kc), dtype=torch.float32, device=DEV)
    hlq.hlq_hla_project(dev(T), B, r, ThatT, coeffT)
    torch.cuda.synchronize()
    Tn = wl.as_f32_numpy(T)
    ref32 = oracle.hla_f32(Tn, B, r)
    ref64 = oracle.hla_f64(Tn, B, r)
    got = coeffT.cpu().numpy()
    # bar: 1e-5 relative to the block norm; the ascending-stride butterflies in fact reproduce the
    # oracle's pairwise sums bit for bit
    blocknorm = np.sqrt((Tn.astype(np.float64) ** 2).reshape(N // B, B, D).sum(axis=1)).T   # [D, N/B]
    bound = 1e-5 * np.repeat(blocknorm, r, axis=1) * np.sqrt(B)
    assert np.all(np.abs(got - ref64) <= bound + 1e-30)
    assert np.array_equal(got.view(np.uint32), ref32.view(np.uint32))
    assert np.array_equal(ThatT.float().cpu().numpy().view(np.uint32), oracle.round_bf16(ref32).view(np.uint32))
    # hlq_compress_act is the same projection
    X2 = torch.empty_like(ThatT)
    hlq.hlq_compress_act(dev(T), B, r, X2)
    assert torch.equal(X2, ThatT)


# --------------------------------------------------------------------------------------------
# K4: bf16 MFMA product
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("M,Nn,K", [(256, 256, 128), (300, 260, 104), (1030, 520, 6304), (64, 8, 8), (768, 264, 6272),
                                    (300, 260, 16), (515, 200, 40), (260, 384, 64),      # one k step, whole and ragged
                                    (136, 264, 2048)])                                  # split until one step is left
def test_bf16_gemm(M, Nn, K):
    A = rand_tensor((M, K), torch.bfloat16, seed=M + K)
    Bm = rand_tensor((Nn, K), torch.bfloat16, seed=Nn + K + 1)
    ref = oracle.gemm_nt_f64(wl.as_f32_numpy(A), wl.as_f32_numpy(Bm), 0.0625)
    out32 = torch.empty((M, Nn), dtype=torch.float32, device=DEV)
    hlq.hlq_bf16_gemm_nt(dev(A), dev(Bm), 0.0625, out32)
    # fp32 accumulation of exact bf16 products: error ~ sqrt(K) ulps of the row scale
    assert row_rel_err(out32.cpu().numpy(), ref) < 1e-5
    out16 = torch.empty((M, Nn), dtype=torch.bfloat16, device=DEV)
    hlq.hlq_bf16_gemm_nt(dev(A), dev(Bm), 0.0625, out16)
    assert row_rel_err(out16.float().cpu().numpy(), ref, True) < TOL_OUT
    # split over k when scratch is given (fp32 partial sums added in a fixed order)
    ws = torch.empty(max(hlq.hlq_gemm_workspace_bytes(1, M, Nn, K), 16), dtype=torch.uint8, device=DEV)
    out32s = torch.empty_like(out32)
    hlq.hlq_bf16_gemm_nt(dev(A), dev(Bm), 0.0625, out32s, ws)
    assert row_rel_err(out32s.cpu().numpy(), ref) < 1e-5
    out32t = torch.empty_like(out32)
    hlq.hlq_bf16_gemm_nt(dev(A), dev(Bm), 0.0625, out32t, ws)
    assert torch.equal(out32s, out32t)          # deterministic


def test_bf16_gemm_large_tile_variant_sampled():
    M, Nn, K = 4096, 4096, 264
    A = rand_tensor((M, K), torch.bfloat16, seed=11)
    Bm = rand_tensor((Nn, K), torch.bfloat16, seed=12)
    out = torch.empty((M, Nn), dtype=torch.float32, device=DEV)
    hlq.hlq_bf16_gemm_nt(dev(A), dev(Bm), 1.0, out)
    rng = np.random.default_rng(3)
    rows = np.unique(np.concatenate([[0, 1, 31, 32, 127, 128, 255, 256, 4095], rng.integers(0, M, 40)]))
    ref = oracle.gemm_nt_f64(wl.as_f32_numpy(A)[rows], wl.as_f32_numpy(Bm), 1.0)
    assert row_rel_err(out.cpu().numpy()[rows], ref) < 1e-5


# --------------------------------------------------------------------------------------------
# the whole backward pass
# --------------------------------------------------------------------------------------------
def _backward_gpu(t, w, use_ex=False, workspace=False):
    G, X, W = dev(t["G"]), dev(t["X"]), dev(t["W"])
    dX = torch.empty((w.N, w.d_in), dtype=G.dtype, device=DEV)
    dW = torch.empty((w.d_out, w.d_in), dtype=G.dtype, device=DEV)
    if use_ex or G.dtype != torch.bfloat16:
        ws = None
        if workspace:
            ws = torch.empty(hlq.hlq_workspace_bytes(w.N, w.d_in, w.d_out, w.B, w.r), dtype=torch.uint8, device=DEV)
        hlq.hlq_linear_backward_ex(G, X, None, W, w.N, w.d_in, w.d_out, w.B, w.r, w.seed, dX, dW, ws)
    else:
        hlq.hlq_linear_backward(G, X, W, w.B, w.r, w.seed, dX, dW)
    torch.cuda.synchronize()
    return dX, dW


SMALL = [
    wl.WORKLOADS["c1"],
    wl.scaled(wl.WORKLOADS["c2"], N=4 * 197 * 4, d_in=264, d_out=512),     # ragged everywhere
    wl.scaled(wl.WORKLOADS["c3"], N=784, d_in=576, d_out=256),
    wl.scaled(wl.WORKLOADS["c4"], N=512, d_in=520, d_out=1376),
    wl.scaled(wl.WORKLOADS["c4_b32"], N=512, d_in=264, d_out=1376),
    wl.scaled(wl.WORKLOADS["c4_b64"], N=512, d_in=264, d_out=1408),
    wl.scaled(wl.WORKLOADS["c5_r4"], N=512, d_in=1032, d_out=512),
    wl.scaled(wl.WORKLOADS["c5_r16"], N=512, d_in=1032, d_out=512),
]


@pytest.mark.parametrize("w", SMALL, ids=lambda w: "%s_N%d_I%d_O%d_B%d_r%d" % (w.name, w.N, w.d_in, w.d_out, w.B, w.r))
def test_linear_backward_matches_oracle(w):
    t = wl.generate(w)
    dX, dW = _backward_gpu(t, w, workspace=(w.name == "c1"))
    ref = oracle.linear_backward(wl.as_f32_numpy(t["G"]), wl.as_f32_numpy(t["X"]), wl.as_f32_numpy(t["W"]),
                                 w.B, w.r, w.seed)
    ex = row_rel_err(dX.float().cpu().numpy(), ref["dX"], w.dtype == "bf16")
    ew = row_rel_err(dW.float().cpu().numpy(), ref["dW"], w.dtype == "bf16")
    print("%s: dX err %.3e  dW err %.3e" % (w.name, ex, ew))
    assert ex < TOL_OUT and ew < TOL_OUT
    if w.dtype == "f32":
        # fp32 outputs: only the epilogue's rounding order separates the two
        assert ex < 1e-5 and ew < 1e-4


def test_linear_backward_is_deterministic_and_seeded():
    w = SMALL[3]
    t = wl.generate(w)
    a = _backward_gpu(t, w)
    b = _backward_gpu(t, w, use_ex=True, workspace=True)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    w2 = wl.scaled(w, seed=1)
    c = _backward_gpu(t, w2)
    assert not torch.equal(a[0], c[0])          # another rounding stream
    assert torch.equal(a[1], c[1])              # dW does not use random bits


def test_backward_from_compressed_activation():
    # ACBP: X is compressed at forward time, the backward pass consumes XhatT and never sees X
    w = SMALL[6]
    t = wl.generate(w)
    G, X, W = dev(t["G"]), dev(t["X"]), dev(t["W"])
    Kc = w.N // w.B * w.r
    XhatT = torch.empty((w.d_in, Kc), dtype=torch.bfloat16, device=DEV)
    hlq.hlq_compress_act(X, w.B, w.r, XhatT)
    dX1, dW1 = _backward_gpu(t, w)
    dX2 = torch.empty_like(dX1)
    dW2 = torch.empty_like(dW1)
    hlq.hlq_linear_backward_ex(G, None, XhatT, W, w.N, w.d_in, w.d_out, w.B, w.r, w.seed, dX2, dW2, None)
    torch.cuda.synchronize()
    assert torch.equal(dX1, dX2) and torch.equal(dW1, dW2)
    # halves on their own
    dX3 = torch.empty_like(dX1)
    hlq.hlq_linear_backward_ex(G, None, None, W, w.N, w.d_in, w.d_out, w.B, w.r, w.seed, dX3, None, None)
    dW3 = torch.empty_like(dW1)
    hlq.hlq_linear_backward_ex(G, X, None, None, w.N, w.d_in, w.d_out, w.B, w.r, w.seed, None, dW3, None)
    torch.cuda.synchronize()
    assert torch.equal(dX1, dX3) and torch.equal(dW1, dW3)


def test_zero_gradient_gives_zero_outputs():
    w = wl.scaled(wl.WORKLOADS["c2"], N=256, d_in=256, d_out=256)
    t = wl.generate(w)
    t["G"] = torch.zeros_like(t["G"])
    dX, dW = _backward_gpu(t, w)
    assert not dX.any() and not dW.any()
