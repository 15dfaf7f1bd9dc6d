"""Pins for the oracle's 8-bit quantiser and the integer g_w path (CPU only).

Sec. 6.1 lists six stages for g_w: project x, quantise to int8, project g_o^T, quantise to int8,
integer product, dequantise.  Sec. 7 runs every quantiser in int8 during a warm-up phase."""
import numpy as np
import pytest

import oracle


def test_quantize_one_qmax127_is_stochastic_rounding():
    for k in (-127, -64, -1, 0, 1, 77, 127):
        for byte in (0, 128, 255):
            assert oracle.quantize_one(float(k), 1.0, byte, qmax=127) == k
    for x in (0.25, 100.5, -126.875, 126.99):
        codes = [oracle.quantize_one(x, 1.0, b, qmax=127) for b in range(256)]
        lo = int(np.floor(x))
        assert all(codes[i] <= codes[i + 1] for i in range(255)) and set(codes) <= {lo, lo + 1}
        assert abs(sum(c == lo + 1 for c in codes) - 256 * (x - lo)) <= 1
    assert oracle.quantize_one(1000.0, 1.0, 0, qmax=127) == 127
    assert oracle.quantize_one(-1000.0, 1.0, 255, qmax=127) == -127
    assert oracle.quantize_one(10.0, 1.0, 0, qmax=7) == 7          # the 4-bit clamp is unchanged


@pytest.mark.parametrize("tensor", [2, 3])
def test_quantize_rows_qmax127_invariants(tensor):
    rng = np.random.default_rng(tensor)
    rows, K = 24, 64
    Cm = (rng.standard_normal((rows, K)) * np.exp(2 * rng.standard_normal((rows, 1)))).astype(np.float32)
    Cm[5] = 0
    q, s = oracle.quantize_rows(Cm, seed=4, tensor=tensor, qmax=127)
    a = np.max(np.abs(Cm), axis=1)
    assert np.array_equal(s, (a / np.float32(127.0)).astype(np.float32))
    assert np.max(np.abs(q.astype(np.int32))) == 127 and not q[5].any()
    nz = a > 0
    assert np.all(np.max(np.abs(q[nz].astype(np.int32)), axis=1) == 127)
    err = np.abs(q.astype(np.float64) * s[:, None] - Cm)
    assert np.all(err[nz] < s[nz, None] * (1 + 1e-6))
    # one code by hand, from the stream's byte
    key = oracle.stream_key(4, tensor)
    rw, k = 7, 33
    inv = np.float32(127.0) / a[rw]
    t = np.float32(np.float64(Cm[rw, k]) * np.float64(inv) + (oracle.rand_byte(key, rw, k, K) + 0.5) / 256.0)
    assert q[rw, k] == int(np.clip(np.floor(t), -127, 127))
    # 8-bit codes resolve 127/7 times finer than 4-bit ones
    q4, s4 = oracle.quantize_rows(Cm, seed=4, tensor=tensor, qmax=7)
    e8 = np.sqrt(np.mean((q.astype(np.float64) * s[:, None] - Cm)[nz] ** 2))
    e4 = np.sqrt(np.mean((q4.astype(np.float64) * s4[:, None] - Cm)[nz] ** 2))
    assert e8 < e4 / 10
    # the four operands draw from four different streams
    assert not np.array_equal(q, oracle.quantize_rows(Cm, seed=4, tensor=tensor ^ 1, qmax=127)[0])


def _problem(seed=3, N=64, I=24, O=48):
    rng = np.random.default_rng(seed)
    G = (rng.standard_normal((N, O)) * 1e-3).astype(np.float32)
    X = rng.standard_normal((N, I)).astype(np.float32)
    W = (rng.standard_normal((O, I)) * 0.02).astype(np.float32)
    return G, X, W


def test_mode_default_equals_linear_backward():
    G, X, W = _problem()
    a = oracle.linear_backward_mode(G, X, W, 16, 8, 5)
    b = oracle.linear_backward(G, X, W, 16, 8, 5, intermediates=True)
    assert np.array_equal(a["Gq"], b["Gq"]) and np.array_equal(a["acc"], b["acc"])
    assert np.array_equal(a["dX"], b["dX"]) and np.array_equal(a["dW"], b["dW"])


def test_integer_gw_path_layout_and_unbiasedness():
    G, X, W = _problem(N=64, I=16, O=32)
    B, r = 16, 8
    out = oracle.linear_backward_mode(G, X, W, B, r, 0, gw_int8=True)
    Kc = 64 // B * r
    assert out["XqT"].shape == (16, Kc) and out["GqT"].shape == (32, Kc) and out["dW"].shape == (32, 16)
    assert np.array_equal(out["accw"], out["GqT"].astype(np.int64) @ out["XqT"].astype(np.int64).T)
    # stages 2 and 4 quantise the fp32 projections (no bf16 rounding in between)
    Xq, sX = oracle.quantize_rows(oracle.hla_f32(X, B, r), 0, oracle.TENSOR_XHAT, qmax=127)
    assert np.array_equal(out["XqT"], Xq) and np.array_equal(out["sX"], sX)
    # the integer estimate of the projected product is unbiased: its seed-average converges to it
    exact = oracle.hla_f64(G, B, r) @ oracle.hla_f64(X, B, r).T / B
    scale = np.sqrt(np.mean(exact ** 2))
    errs = []
    for S in (1, 16, 256):
        m = np.zeros_like(exact)
        for seed in range(S):
            m += oracle.linear_backward_mode(G, X, W, B, r, seed, gw_int8=True)["dW"]
        errs.append(np.sqrt(np.mean((m / S - exact) ** 2)) / scale)
    assert errs[0] < 0.05                      # int8 operands: already close with one draw
    assert errs[1] < errs[0] / 2.5 and errs[2] < errs[1] / 2.5


def test_eight_bit_gx_is_closer_to_the_dense_product():
    G, X, W = _problem(seed=9, N=32, I=16, O=64)
    ref = G.astype(np.float64) @ W.astype(np.float64)
    e4 = e8 = 0.0
    for seed in range(8):
        e4 += np.mean((oracle.linear_backward_mode(G, X, W, 16, 8, seed, gx_bits=4)["dX"] - ref) ** 2)
        o8 = oracle.linear_backward_mode(G, X, W, 16, 8, seed, gx_bits=8)
        e8 += np.mean((o8["dX"] - ref) ** 2)
        assert np.max(np.abs(o8["acc"])) <= 127 * 127 * 64
    assert e8 < e4 / 50


def test_pack_nibbles_layout():
    """Two codes to a byte: code 2b low nibble, code 2b+1 high nibble, 4-bit two's complement --
    checked against arithmetic done by hand, and by unpacking with sign extension."""
    q = np.array([[1, -1, 7, -7, 0, 3, -4, 5]], dtype=np.int8)
    p = oracle.pack_nibbles(q)
    assert p.dtype == np.uint8 and p.shape == (1, 4)
    assert p.tolist() == [[0x01 | (0xF << 4), 0x07 | (0x9 << 4), 0x00 | (0x3 << 4), 0xC | (0x5 << 4)]]
    rng = np.random.default_rng(0)
    q = rng.integers(-7, 8, size=(5, 64)).astype(np.int8)
    p = oracle.pack_nibbles(q).astype(np.int16)
    lo = ((p & 0xF) ^ 8) - 8                      # sign-extend a nibble
    hi = (((p >> 4) & 0xF) ^ 8) - 8
    back = np.stack([lo, hi], axis=2).reshape(5, 64)
    assert np.array_equal(back, q)
    with pytest.raises(AssertionError):
        oracle.pack_nibbles(np.array([[8, 0]], dtype=np.int8))


def test_int4_activation_store_is_the_same_quantiser_at_qmax_7():
    """Sec. 6.1 keeps the compressed activation as 4-bit integers between the passes: the stage-2
    quantiser with codes in [-7, 7].  Same projection, same stream, same absmax per feature; only the
    grid is coarser, the product stays the integer product, and the estimate stays unbiased."""
    G, X, W = _problem(N=64, I=16, O=32)
    B, r = 16, 8
    o4 = oracle.linear_backward_mode(G, X, W, B, r, 2, gw_int8=True, xhat_bits=4)
    o8 = oracle.linear_backward_mode(G, X, W, B, r, 2, gw_int8=True, xhat_bits=8)
    xh = oracle.hla_f32(X, B, r)
    Xq, sX = oracle.quantize_rows(xh, 2, oracle.TENSOR_XHAT, qmax=7)
    assert np.array_equal(o4["XqT"], Xq) and np.array_equal(o4["sX"], sX)
    a = np.max(np.abs(xh), axis=1)
    assert np.array_equal(sX, (a / np.float32(7.0)).astype(np.float32))
    assert np.max(np.abs(Xq.astype(np.int32))) == 7 and np.all(np.max(np.abs(Xq.astype(np.int32)), axis=1) == 7)
    assert np.all(np.abs(Xq.astype(np.float64) * sX[:, None] - xh) < sX[:, None] * (1 + 1e-6))
    # the other operand and the whole g_x list do not change
    assert np.array_equal(o4["GqT"], o8["GqT"]) and np.array_equal(o4["dX"], o8["dX"])
    assert np.array_equal(o4["accw"], o4["GqT"].astype(np.int64) @ Xq.astype(np.int64).T)
    # dequantisation: acc * sGhat[o] * sX[i] / B, recomputed here in fp64 from the parts
    want = o4["accw"].astype(np.float64) * o4["sGhat"].astype(np.float64)[:, None] * sX.astype(np.float64)[None, :] / B
    assert np.allclose(o4["dW"], want, rtol=1e-6, atol=0)
    # unbiased: the seed average converges to the product of the exact projections, from further away
    # than with 8-bit codes
    exact = oracle.hla_f64(G, B, r) @ oracle.hla_f64(X, B, r).T / B
    scale = np.sqrt(np.mean(exact ** 2))
    errs = []
    for S in (1, 16, 256):
        m = np.zeros_like(exact)
        for seed in range(S):
            m += oracle.linear_backward_mode(G, X, W, B, r, seed, gw_int8=True, xhat_bits=4)["dW"]
        errs.append(np.sqrt(np.mean((m / S - exact) ** 2)) / scale)
    e8 = np.sqrt(np.mean((o8["dW"] - exact) ** 2)) / scale
    assert e8 < errs[0] < 0.6
    assert errs[1] < errs[0] / 2.5 and errs[2] < errs[1] / 2.5
    with pytest.raises(AssertionError):
        oracle.linear_backward_mode(G, X, W, B, r, 0, gw_int8=False, xhat_bits=4)
