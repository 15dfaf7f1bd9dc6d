"""Pins for the oracle's Hadamard matrix, coefficients and block transforms (CPU only).

Each test checks the oracle against something it does not compute itself: scipy's
Sylvester construction, the popcount closed form, exact integer arithmetic, Parseval's
identity, one-hot probes of the index layout, or a brute-force summation tree.
"""
import numpy as np
import pytest
import scipy.linalg

import oracle

BLOCKS = [2, 4, 8, 16, 32, 64]


@pytest.mark.parametrize("B", BLOCKS)
def test_matrix_is_sylvester(B):
    H = oracle.hadamard(B).astype(np.int64)
    # Eq. 2 (Sec. 3.2) up to the 1/sqrt(2) per level: scipy builds the same Kronecker recursion
    assert np.array_equal(H, scipy.linalg.hadamard(B).astype(np.int64))
    # closed form of the natural-order Walsh-Hadamard matrix
    i, j = np.meshgrid(np.arange(B), np.arange(B), indexing="ij")
    pop = np.vectorize(lambda x: bin(int(x)).count("1"))(i & j)
    assert np.array_equal(H, (-1) ** pop)
    # orthogonality (Sec. 3.2): unnormalised, so H.H^T = B.I, and H is symmetric
    assert np.array_equal(H @ H.T, B * np.eye(B, dtype=np.int64))
    assert np.array_equal(H, H.T)


def test_matrix_rejects_bad_order():
    for B in (0, 3, 12, 128):
        with pytest.raises(ValueError):
            oracle.hadamard(B)


@pytest.mark.parametrize("B", [16, 32, 64])
def test_coefficients_exact_on_integers(B):
    # integer-valued inputs below 2^17 make every partial sum exact in fp32, whatever the order,
    # so the result must equal int64 arithmetic with scipy's matrix
    rng = np.random.default_rng(B)
    H = scipy.linalg.hadamard(B).astype(np.int64)
    for _ in range(20):
        v = rng.integers(-(1 << 17), 1 << 17, size=B)
        c = oracle.coeff_f32(v.astype(np.float32), B)
        assert np.array_equal(c.astype(np.int64), H @ v)
        c64 = oracle.coeff_f64(v.astype(np.float32), B)
        assert np.array_equal(c64.astype(np.int64), H @ v)


@pytest.mark.parametrize("B", [16, 32, 64])
def test_coefficients_parseval_and_fp64(B):
    rng = np.random.default_rng(100 + B)
    for _ in range(20):
        v = (rng.standard_normal(B) * np.exp(3 * rng.standard_normal(B))).astype(np.float32)
        c32 = oracle.coeff_f32(v, B).astype(np.float64)
        c64 = oracle.coeff_f64(v, B)
        nv = np.linalg.norm(v.astype(np.float64))
        # Parseval for an unnormalised Hadamard matrix: sum c^2 = B sum v^2
        assert abs(np.sum(c64 ** 2) - B * nv ** 2) <= 1e-12 * B * nv ** 2
        # the fp32 pairwise sums stay within a few ulps (relative to the block norm) of fp64
        assert np.max(np.abs(c32 - c64)) <= 1e-6 * nv * np.sqrt(B)


def _pairwise(vals):
    """Balanced pairwise fp32 sum, written independently of the C code (iterative halving)."""
    vals = [np.float32(x) for x in vals]
    while len(vals) > 1:
        vals = [np.float32(vals[2 * k] + vals[2 * k + 1]) for k in range(len(vals) // 2)]
    return vals[0]


@pytest.mark.parametrize("B", [16, 64])
def test_coefficients_use_the_balanced_pairwise_tree(B):
    # wide dynamic range makes the fp32 result depend on the summation order; adjacent-pair
    # halving is the same tree as the recursive midpoint split for power-of-two lengths
    rng = np.random.default_rng(7 + B)
    H = scipy.linalg.hadamard(B)
    differs_from_sequential = 0
    for _ in range(10):
        v = (rng.standard_normal(B) * np.exp(6 * rng.standard_normal(B))).astype(np.float32)
        c = oracle.coeff_f32(v, B)
        for i in range(B):
            want = _pairwise(H[i] * v)
            assert c[i] == want
            seq = np.float32(0)
            for j in range(B):
                seq = np.float32(seq + np.float32(H[i, j] * v[j]))
            differs_from_sequential += int(seq != want)
    assert differs_from_sequential > 0  # the probe really is order-sensitive


def _butterfly_ascending(v):
    """In-place radix-2 butterflies with strides 1, 2, 4, ... in fp32 (the GPU's evaluation order)."""
    v = [np.float32(x) for x in v]
    n, h = len(v), 1
    while h < n:
        for base in range(0, n, 2 * h):
            for k in range(base, base + h):
                a, b = v[k], v[k + h]
                v[k], v[k + h] = np.float32(a + b), np.float32(a - b)
        h *= 2
    return np.array(v, dtype=np.float32)


@pytest.mark.parametrize("B", [16, 32, 64])
def test_ascending_stride_butterfly_matches_bit_for_bit(B):
    # the definition (explicit mat-vec + pairwise sum) and an ascending-stride FWHT are the
    # same fp32 expression tree: this is what lets a fast transform be bit-exact
    rng = np.random.default_rng(11 + B)
    for _ in range(10):
        v = (rng.standard_normal(B) * np.exp(6 * rng.standard_normal(B))).astype(np.float32)
        assert np.array_equal(oracle.coeff_f32(v, B), _butterfly_ascending(v))


@pytest.mark.parametrize("B", [16, 32])
def test_transform_rows_layout(B):
    rng = np.random.default_rng(3)
    N, O = 5, 4 * B
    G = rng.integers(-1000, 1000, size=(N, O)).astype(np.float32)
    H = scipy.linalg.hadamard(B).astype(np.float64)
    want = (G.astype(np.float64).reshape(N, O // B, B) @ H.T).reshape(N, O)  # c_i = sum_j H[i,j] v_j
    assert np.array_equal(oracle.transform_rows(G, B).astype(np.float64), want)
    # one-hot probe: G[n0, o0] = 1 -> row n0, block o0//B holds column (o0 % B) of H
    G1 = np.zeros((N, O), dtype=np.float32)
    G1[2, B + 3] = 1.0
    T = oracle.transform_rows(G1, B)
    assert np.array_equal(T[2, B:2 * B], H[:, 3].astype(np.float32))
    T[2, B:2 * B] = 0
    assert not T.any()


@pytest.mark.parametrize("B", [16, 32])
def test_transform_cols_layout(B):
    rng = np.random.default_rng(4)
    O, I = 3 * B, 7
    W = rng.integers(-1000, 1000, size=(O, I)).astype(np.float32)
    H = scipy.linalg.hadamard(B).astype(np.float64)
    # (H_O^T W): blocks of B consecutive rows of W are mixed; result returned transposed [I, O]
    blocks = W.astype(np.float64).reshape(O // B, B, I)
    want = np.einsum("ij,bjc->bic", H, blocks).reshape(O, I).T
    assert np.array_equal(oracle.transform_cols(W, B).astype(np.float64), want)
    W1 = np.zeros((O, I), dtype=np.float32)
    W1[2 * B + 5, 4] = 1.0
    T = oracle.transform_cols(W1, B)
    assert T.shape == (I, O)
    assert np.array_equal(T[4, 2 * B:3 * B], H[:, 5].astype(np.float32))
    T[4, 2 * B:3 * B] = 0
    assert not T.any()


def test_transforms_cancel_in_the_product():
    # Sec. 5: (a H)(H^T b^T) = B . a b^T, so without quantisation the g_x path is exactly G.W
    rng = np.random.default_rng(5)
    B, N, O, I = 16, 12, 64, 9
    G = rng.integers(-50, 50, size=(N, O)).astype(np.float32)
    W = rng.integers(-50, 50, size=(O, I)).astype(np.float32)
    Gh = oracle.transform_rows(G, B).astype(np.float64)
    WhT = oracle.transform_cols(W, B).astype(np.float64)
    assert np.array_equal(Gh @ WhT.T / B, G.astype(np.float64) @ W.astype(np.float64))
    # and on real-valued data up to fp32 rounding of the coefficients
    G = rng.standard_normal((N, O)).astype(np.float32)
    W = rng.standard_normal((O, I)).astype(np.float32)
    Gh = oracle.transform_rows(G, B).astype(np.float64)
    WhT = oracle.transform_cols(W, B).astype(np.float64)
    ref = G.astype(np.float64) @ W.astype(np.float64)
    assert np.max(np.abs(Gh @ WhT.T / B - ref)) <= 1e-5 * np.max(np.abs(ref))


def test_transform_flattens_outliers():
    # Sec. 5.1 / Fig. 2: after the transform a row with a few huge entries has a much smaller
    # max/rms ratio, which is why the quantiser loses less (sanity check, not a parity pin)
    rng = np.random.default_rng(6)
    G = rng.standard_normal((64, 256)).astype(np.float32)
    G[:, ::37] *= 40.0
    T = oracle.transform_rows(G, 16)
    crest = lambda a: np.mean(np.max(np.abs(a), axis=1) / np.sqrt(np.mean(a.astype(np.float64) ** 2, axis=1)))
    assert crest(T) < 0.6 * crest(G)
