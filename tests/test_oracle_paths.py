"""Pins for the oracle's GEMMs, HLA projection and the composed backward pass (CPU only)."""
import numpy as np
import pytest
import scipy.linalg
import torch

import oracle


def test_int_gemm_brute_force_and_bounds():
    rng = np.random.default_rng(0)
    M, Nn, K = 5, 6, 12
    A = rng.integers(-7, 8, size=(M, K)).astype(np.int8)
    Bm = rng.integers(-7, 8, size=(Nn, K)).astype(np.int8)
    acc = oracle.int_gemm_nt(A, Bm)
    for m in range(M):
        for n in range(Nn):
            assert acc[m, n] == sum(int(A[m, k]) * int(Bm[n, k]) for k in range(K))
    # larger case against numpy's int64 product; A and Bm have different shapes so a transposed
    # operand or swapped index would not even fit
    A = rng.integers(-7, 8, size=(33, 128)).astype(np.int8)
    Bm = rng.integers(-7, 8, size=(17, 128)).astype(np.int8)
    assert np.array_equal(oracle.int_gemm_nt(A, Bm), A.astype(np.int64) @ Bm.astype(np.int64).T)
    # all codes at 7: every accumulator is exactly 49 K (the largest possible magnitude)
    K = 11008
    acc = oracle.int_gemm_nt(np.full((2, K), 7, np.int8), np.full((3, K), -7, np.int8))
    assert np.all(acc == -49 * K)


def test_dequant_closed_form():
    rng = np.random.default_rng(1)
    acc = rng.integers(-1000, 1000, size=(4, 5)).astype(np.int32)
    sA = rng.random(4).astype(np.float32)
    sB = rng.random(5).astype(np.float32)
    out = oracle.dequant(acc, sA, sB, 16)
    want = acc * sA.astype(np.float64)[:, None] * sB.astype(np.float64)[None, :] / 16
    assert np.allclose(out, want, rtol=1e-15, atol=0)


def test_round_bf16_matches_torch_and_ties_to_even():
    rng = np.random.default_rng(2)
    x = (rng.standard_normal(20000) * np.exp(rng.standard_normal(20000) * 8)).astype(np.float32)
    # ties and near-ties around the bf16 rounding boundary
    base = np.array([1.0, 1.0078125, -2.5, 3.0e-39, 65280.0], dtype=np.float32).view(np.uint32)
    ties = np.concatenate([base | 0x8000, (base | 0x8000) + 1, (base | 0x8000) - 1,
                           base | 0x18000]).astype(np.uint32).view(np.float32)
    x = np.concatenate([x, ties, np.array([0.0, -0.0, np.inf, -np.inf], dtype=np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(oracle.round_bf16(x).view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("B,r", [(16, 8), (32, 4), (64, 32), (16, 16)])
def test_hla_layout_and_basis(B, r):
    # one-hot probe: T[n0, j0] = 1 -> ChatT[j0, (n0//B)*r + k] = H[k, n0 % B] for k < r: pins the
    # natural-order first-r basis choice and the [column, block*r + k] layout
    H = scipy.linalg.hadamard(B).astype(np.float32)
    N, D = 3 * B, 5
    n0, j0 = B + 5, 3
    T = np.zeros((N, D), dtype=np.float32)
    T[n0, j0] = 1.0
    Ch = oracle.hla_f32(T, B, r)
    assert Ch.shape == (D, N // B * r)
    blk = n0 // B
    assert np.array_equal(Ch[j0, blk * r:(blk + 1) * r], H[:r, n0 % B])
    Ch[j0, blk * r:(blk + 1) * r] = 0
    assert not Ch.any()
    # integer data: exact against scipy's matrix
    rng = np.random.default_rng(3)
    T = rng.integers(-500, 500, size=(N, D)).astype(np.float32)
    want = np.einsum("kn,bnd->dbk", H[:r].astype(np.float64),
                     T.astype(np.float64).reshape(N // B, B, D)).reshape(D, -1)
    assert np.array_equal(oracle.hla_f32(T, B, r).astype(np.float64), want)
    assert np.array_equal(oracle.hla_f64(T, B, r), want)


@pytest.mark.parametrize("B", [16, 32])
def test_hla_full_rank_reproduces_dense_dw(B):
    # Sec. 5.1: with all B bases kept, (G^T H^T)(H X)/B = G^T X  (H^T H = B I)
    rng = np.random.default_rng(4)
    N, O, I = 4 * B, 24, 10
    G = rng.standard_normal((N, O)).astype(np.float32)
    X = rng.standard_normal((N, I)).astype(np.float32)
    Gh = oracle.hla_f64(G, B, B)
    Xh = oracle.hla_f64(X, B, B)
    ref = G.astype(np.float64).T @ X.astype(np.float64)
    assert np.allclose(Gh @ Xh.T / B, ref, rtol=1e-12, atol=1e-12)
    dW = oracle.gemm_nt_f64(oracle.hla_f32(G, B, B), oracle.hla_f32(X, B, B), 1.0 / B)
    assert np.max(np.abs(dW - ref)) <= 2e-6 * np.max(np.abs(ref)) * np.sqrt(N)


@pytest.mark.parametrize("B,r", [(32, 4), (32, 8), (32, 16), (16, 8), (64, 32)])
def test_hla_low_rank_closed_form(B, r):
    # keeping rows 0..r-1 of the natural-order matrix projects every block onto vectors that are
    # periodic with period r: P = H_r^T H_r / B has P[j, j'] = r/B when j = j' (mod r), else 0.
    # Hence dW_HLA = (r/B) sum_blocks sum_{c<r} F_G[c]^T F_X[c], F_T[c] = sum of the block's
    # tokens congruent to c mod r.  Computed here with numpy only.
    rng = np.random.default_rng(5)
    N, O, I = 3 * B, 12, 7
    G = rng.standard_normal((N, O)).astype(np.float32)
    X = rng.standard_normal((N, I)).astype(np.float32)
    FG = G.astype(np.float64).reshape(N // B, B // r, r, O).sum(axis=1)
    FX = X.astype(np.float64).reshape(N // B, B // r, r, I).sum(axis=1)
    want = (r / B) * np.einsum("bco,bci->oi", FG, FX)
    got = oracle.gemm_nt_f64(oracle.hla_f32(G, B, r), oracle.hla_f32(X, B, r), 1.0 / B)
    assert np.max(np.abs(got - want)) <= 1e-5 * np.max(np.abs(want))


def test_gemm_nt_f64_against_numpy():
    rng = np.random.default_rng(6)
    A = rng.standard_normal((9, 40)).astype(np.float32)
    Bm = rng.standard_normal((4, 40)).astype(np.float32)
    want = 0.25 * A.astype(np.float64) @ Bm.astype(np.float64).T
    assert np.allclose(oracle.gemm_nt_f64(A, Bm, 0.25), want, rtol=1e-13, atol=1e-13)


def _small_problem(seed=7, N=64, I=24, O=48):
    rng = np.random.default_rng(seed)
    G = (rng.standard_normal((N, O)) * 1e-3).astype(np.float32)
    X = rng.standard_normal((N, I)).astype(np.float32)
    W = (rng.standard_normal((O, I)) * 0.02).astype(np.float32)
    return G, X, W


def test_linear_backward_is_the_composition_of_its_stages():
    G, X, W = _small_problem()
    B, r, seed = 16, 8, 5
    out = oracle.linear_backward(G, X, W, B, r, seed, intermediates=True)
    Gq, sG = oracle.quantize_rows(oracle.transform_rows(G, B), seed, 0)
    Wq, sW = oracle.quantize_rows(oracle.transform_cols(W, B), seed, 1)
    assert np.array_equal(out["Gq"], Gq) and np.array_equal(out["sG"], sG)
    assert np.array_equal(out["Wq"], Wq) and np.array_equal(out["sW"], sW)
    acc = Gq.astype(np.int64) @ Wq.astype(np.int64).T
    assert np.array_equal(out["acc"], acc)
    assert np.allclose(out["dX"], acc * sG.astype(np.float64)[:, None] * sW.astype(np.float64)[None, :] / B,
                       rtol=1e-14, atol=0)
    gh = oracle.round_bf16(oracle.hla_f32(G, B, r))
    xh = oracle.round_bf16(oracle.hla_f32(X, B, r))
    assert np.array_equal(out["GhatT"], gh) and np.array_equal(out["XhatT"], xh)
    assert np.allclose(out["dW"], gh.astype(np.float64) @ xh.astype(np.float64).T / B, rtol=1e-13, atol=1e-18)


def test_dx_is_an_unbiased_estimate_of_g_times_w():
    # E[dX] = G.W (Sec. 5/6.1: unbiased quantiser on both operands, independent streams);
    # the error of the seed-average falls like 1/sqrt(S)
    G, X, W = _small_problem(seed=8, N=32, I=16, O=64)
    ref = G.astype(np.float64) @ W.astype(np.float64)
    scale = np.sqrt(np.mean(ref ** 2))
    errs = []
    for S in (1, 16, 256):
        acc = np.zeros_like(ref)
        for seed in range(S):
            acc += oracle.linear_backward(G, X, W, 16, 8, seed, want_dW=False)["dX"]
        errs.append(np.sqrt(np.mean((acc / S - ref) ** 2)) / scale)
    assert errs[0] < 0.5
    assert errs[1] < errs[0] / 2.5 and errs[2] < errs[1] / 2.5
    assert errs[2] < 0.03


def test_hadamard_quantisation_beats_plain_quantisation_on_outliers():
    # Sec. 5 / Table 1: Q(aH)Q(H^T b) has lower error than Q(a)Q(b) when the operands carry
    # outliers (sanity check of the point of the method, not a parity pin)
    rng = np.random.default_rng(9)
    N, O, I, B = 64, 128, 32, 16
    G = (rng.standard_normal((N, O)) * 1e-3).astype(np.float32)
    G[rng.random((N, O)) < 0.01] *= 30.0
    W = (rng.standard_normal((O, I)) * 0.02).astype(np.float32)
    W[rng.random((O, I)) < 0.01] *= 30.0
    X = np.zeros((N, I), dtype=np.float32)
    ref = G.astype(np.float64) @ W.astype(np.float64)
    e_h = e_p = 0.0
    for seed in range(8):
        dX = oracle.linear_backward(G, X, W, B, 8, seed, want_dW=False)["dX"]
        e_h += np.mean((dX - ref) ** 2)
        Gq, sG = oracle.quantize_rows(G, seed, 0)
        Wq, sW = oracle.quantize_rows(np.ascontiguousarray(W.T), seed, 1)
        plain = oracle.dequant(oracle.int_gemm_nt(Gq, Wq), sG, sW, 1)
        e_p += np.mean((plain - ref) ** 2)
    assert e_h < 0.6 * e_p


def test_linear_backward_rejects_bad_shapes():
    G, X, W = _small_problem()
    with pytest.raises(ValueError):
        oracle.linear_backward(G[:60], X[:60], W, 16, 8, 0)      # N not a multiple of B
    with pytest.raises(ValueError):
        oracle.linear_backward(G, X, W, 16, 32, 0)               # r > B
    with pytest.raises(ValueError):
        oracle.linear_backward(G[:, :40], X, W[:40], 16, 8, 0)   # d_out not a multiple of B
