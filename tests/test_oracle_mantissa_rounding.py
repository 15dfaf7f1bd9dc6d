"""Pins of the oracle's version of the paper's pseudo-stochastic rounding (Sec. 6.1: the low 11
bits of the floating-point value decide the rounding)."""
import numpy as np
import pytest

import oracle


def _bits(x):
    return np.float32(x).view(np.uint32)


def test_threshold_comes_from_the_low_11_bits():
    # y = 2.5 exactly with inv = 1: rounds up iff u >= 0.5, i.e. iff the low 11 bits are >= 1024
    base = _bits(2.5) & ~np.uint32(0x7FF)
    for m, want in [(0, 2), (1023, 2), (1024, 3), (2047, 3)]:
        x = np.uint32(base | m).view(np.float32)
        # the low bits also move x itself, by less than 2^-13 relative: recompute the exact decision
        u = (m + 0.5) / 2048.0
        assert oracle.quantize_one_mantissa(float(x), 1.0, 7) == int(np.floor(np.float64(x) + u))
        if m in (0, 2047):
            assert oracle.quantize_one_mantissa(float(x), 1.0, 7) == want


@pytest.mark.parametrize("qmax", [7, 127])
def test_invariants_hold_as_for_the_counter_stream(qmax):
    rng = np.random.default_rng(qmax)
    Cm = (rng.standard_normal((64, 256)) * np.exp(rng.standard_normal((64, 1)))).astype(np.float32)
    Cm[5] = 0
    q, s = oracle.quantize_rows(Cm, 1, 0, qmax=qmax, rounding=oracle.ROUND_MANTISSA)
    q2, _ = oracle.quantize_rows(Cm, 99, 3, qmax=qmax, rounding=oracle.ROUND_MANTISSA)
    assert np.array_equal(q, q2)                                      # no seed, no stream: a function of the data
    assert np.abs(q).max() <= qmax and np.all(q[5] == 0) and s[5] == 0
    nz = np.arange(64) != 5
    assert np.all(np.abs(q[nz]).max(axis=1) == qmax)                  # the absmax element lands on +-qmax
    assert np.all(np.abs(q[nz] * s[nz, None] - Cm[nz]) < s[nz, None] * (1 + 1e-6))
    k = rng.integers(-qmax, qmax + 1, (8, 32)).astype(np.float32)
    k[:, 0] = qmax
    qk, sk = oracle.quantize_rows(k * np.float32(0.375), 0, 0, qmax=qmax, rounding=oracle.ROUND_MANTISSA)
    assert np.array_equal(qk, k.astype(np.int8))                      # exact grid points stay put


def test_unbiased_on_full_precision_data_and_biased_on_bf16_data():
    rng = np.random.default_rng(11)
    Cm = rng.standard_normal((256, 4096)).astype(np.float32)            # 24 significant bits: low bits are noise
    q, s = oracle.quantize_rows(Cm, 0, 0, rounding=oracle.ROUND_MANTISSA)
    err = (q * s[:, None] - Cm) / s[:, None]
    # a uniform threshold gives zero mean error; the standard error over 1M elements is ~4e-4 steps
    assert abs(err.mean()) < 3e-3
    # the same values cut to 8 significant bits: the low 11 bits are all zero, u = 2^-12, the
    # quantiser rounds down and the mean error is minus half a step
    Cb = (Cm.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)
    qb, sb = oracle.quantize_rows(Cb, 0, 0, rounding=oracle.ROUND_MANTISSA)
    errb = (qb * sb[:, None] - Cb) / sb[:, None]
    assert -0.52 < errb.mean() < -0.45
    qf, sf = oracle.quantize_rows(Cb, 0, 0)                             # the seeded stream does not care
    assert abs(((qf * sf[:, None] - Cb) / sf[:, None]).mean()) < 3e-3


def test_mode_composition_takes_the_rounding():
    rng = np.random.default_rng(9)
    N, I, O, B, r = 64, 24, 32, 16, 8
    G = (rng.standard_normal((N, O)) * 1e-3).astype(np.float32)
    X = rng.standard_normal((N, I)).astype(np.float32)
    W = (rng.standard_normal((O, I)) * 0.02).astype(np.float32)
    a = oracle.linear_backward_mode(G, X, W, B, r, 5, rounding=oracle.ROUND_MANTISSA)
    b = oracle.linear_backward_mode(G, X, W, B, r, 77, rounding=oracle.ROUND_MANTISSA)
    assert np.array_equal(a["dX"], b["dX"]) and np.array_equal(a["Gq"], b["Gq"])
    dense = G.astype(np.float64) @ W.astype(np.float64)
    assert np.linalg.norm(a["dX"] - dense) < 0.25 * np.linalg.norm(dense)
    Gq, sG = oracle.quantize_rows(oracle.transform_rows(G, B), 0, 0, rounding=oracle.ROUND_MANTISSA)
    assert np.array_equal(a["Gq"], Gq) and np.array_equal(a["sG"], sG)
