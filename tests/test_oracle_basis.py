"""Pins of the oracle's choice of kept Hadamard rows on the g_w list (Sec. 4, Sec. 6.1): natural
order (rows 0..r-1 of Eq. 2's matrix) and sequency order (the r rows with the fewest sign changes).
Each check comes from a definition or a closed form that the oracle does not compute itself."""
import numpy as np
import pytest
import scipy.linalg

import oracle


def _bitrev(x, bits):
    return int(format(x, "0%db" % bits)[::-1], 2)


@pytest.mark.parametrize("B", [2, 4, 16, 32, 64])
def test_sequency_rows_are_bit_reversed_gray_codes(B):
    bits = B.bit_length() - 1
    rows = oracle.basis_rows(B, oracle.BASIS_SEQUENCY)
    assert sorted(rows.tolist()) == list(range(B))
    # textbook relation between the natural (Hadamard) and the sequency (Walsh) orderings
    assert rows.tolist() == [_bitrev(k ^ (k >> 1), bits) for k in range(B)]
    H = scipy.linalg.hadamard(B)
    for k, n in enumerate(rows):
        assert int(np.count_nonzero(np.diff(H[n]) != 0)) == k          # row n changes sign k times
    assert oracle.basis_rows(B, oracle.BASIS_NATURAL).tolist() == list(range(B))


@pytest.mark.parametrize("B,r", [(16, 8), (16, 4), (32, 8), (64, 32), (32, 32), (16, 1)])
def test_lowest_sequencies_are_the_natural_rows_that_are_multiples_of_B_over_r(B, r):
    rows = oracle.basis_rows(B, oracle.BASIS_SEQUENCY)[:r]
    assert sorted(rows.tolist()) == list(range(0, B, B // r))


@pytest.mark.parametrize("B,r", [(16, 8), (32, 4), (64, 16), (16, 16)])
def test_sequency_projection_is_block_averaging(B, r):
    """The r lowest-sequency Walsh functions span the step functions on B/r-long segments, so the
    projector (1/B) H_r^T H_r averages within segments: dW = (r/B) sum_segments (sum G)^T (sum X)."""
    rng = np.random.default_rng(B + r)
    N, O, I = 4 * B, 24, 40
    G = rng.standard_normal((N, O)).astype(np.float32)
    X = rng.standard_normal((N, I)).astype(np.float32)
    gh = oracle.hla_f64(G, B, r, oracle.BASIS_SEQUENCY)
    xh = oracle.hla_f64(X, B, r, oracle.BASIS_SEQUENCY)
    dW = gh @ xh.T / B
    seg = B // r
    Gs = G.astype(np.float64).reshape(N // seg, seg, O).sum(axis=1)
    Xs = X.astype(np.float64).reshape(N // seg, seg, I).sum(axis=1)
    want = (r / B) * (Gs.T @ Xs)                                # averaging: 1/seg = r/B within a segment
    assert np.allclose(dW, want, rtol=1e-12, atol=1e-12)
    if r == B:
        assert np.allclose(dW, G.astype(np.float64).T @ X.astype(np.float64), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("B,r", [(16, 8), (32, 16)])
def test_sequency_coefficients_are_the_natural_ones_reordered(B, r):
    rng = np.random.default_rng(3)
    T = (rng.standard_normal((2 * B, 7)) * np.exp(rng.standard_normal((2 * B, 1)))).astype(np.float32)
    full = oracle.hla_f32(T, B, B, oracle.BASIS_NATURAL).reshape(7, 2, B)
    rows = oracle.basis_rows(B, oracle.BASIS_SEQUENCY)[:r]
    got = oracle.hla_f32(T, B, r, oracle.BASIS_SEQUENCY).reshape(7, 2, r)
    assert np.array_equal(got.view(np.uint32), full[:, :, rows].view(np.uint32))
    # and the default is what it always was
    assert np.array_equal(oracle.hla_f32(T, B, r), oracle.hla_f32(T, B, r, oracle.BASIS_NATURAL))


def test_mode_composition_takes_the_basis():
    rng = np.random.default_rng(9)
    N, I, O, B, r = 64, 24, 32, 16, 8
    G = (rng.standard_normal((N, O)) * 1e-3).astype(np.float32)
    X = rng.standard_normal((N, I)).astype(np.float32)
    W = (rng.standard_normal((O, I)) * 0.02).astype(np.float32)
    a = oracle.linear_backward_mode(G, X, W, B, r, 5, basis=oracle.BASIS_NATURAL)
    b = oracle.linear_backward_mode(G, X, W, B, r, 5, basis=oracle.BASIS_SEQUENCY)
    assert np.array_equal(a["dX"], b["dX"])                          # the g_x list does not use it
    assert not np.allclose(a["dW"], b["dW"])
    want = oracle.gemm_nt_f64(oracle.round_bf16(oracle.hla_f32(G, B, r, 1)), oracle.round_bf16(oracle.hla_f32(X, B, r, 1)), 1.0 / B)
    assert np.array_equal(b["dW"], want)
    c = oracle.linear_backward_mode(G, X, W, B, r, 5, gw_int8=True, basis=oracle.BASIS_SEQUENCY)
    full = oracle.hla_f64(G, B, r, 1) @ oracle.hla_f64(X, B, r, 1).T / B
    assert np.abs(c["dW"] - full).max() < 0.05 * np.abs(full).max()  # int8 codes: a percent-level perturbation
