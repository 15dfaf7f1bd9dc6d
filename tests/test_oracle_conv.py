"""Pins of the oracle's convolution glue (Sec. 3.1: a convolution is the layer's product with the
spatial positions as the sequence).  The column matrix and its adjoint are checked against torch's
own convolution and its autograd (a library routine that builds no column matrix in this layout),
against six nested loops on a tiny case, and against the adjoint identity."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import hlq_oracle as orc

GEOMS = [
    # Nb, H, W, C, O, kh, kw, stride, pad, dil
    (2, 6, 6, 4, 5, 3, 3, (1, 1), (1, 1), (1, 1)),
    (2, 7, 9, 3, 4, 3, 3, (2, 2), (1, 1), (1, 1)),
    (1, 8, 8, 2, 3, 1, 1, (1, 1), (0, 0), (1, 1)),
    (2, 9, 8, 2, 3, 3, 2, (2, 1), (0, 1), (1, 1)),
    (1, 11, 10, 3, 2, 3, 3, (1, 2), (2, 2), (2, 2)),
    (3, 5, 5, 2, 2, 5, 5, (1, 1), (2, 2), (1, 1)),
    (2, 8, 8, 4, 6, 2, 2, (2, 2), (0, 0), (1, 1)),
]


def _data(g, seed=0):
    Nb, H, W, Cc, O, kh, kw, st, pd, dl = g
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((Nb, H, W, Cc))
    w = rng.standard_normal((O, kh, kw, Cc))
    Ho = orc.conv_out_size(H, kh, st[0], pd[0], dl[0])
    Wo = orc.conv_out_size(W, kw, st[1], pd[1], dl[1])
    gy = rng.standard_normal((Nb, Ho, Wo, O))
    return x, w, gy


@pytest.mark.parametrize("g", GEOMS)
def test_column_matrix_product_is_the_library_convolution(g):
    Nb, H, W, Cc, O, kh, kw, st, pd, dl = g
    x, w, gy = _data(g)
    y = orc.im2col(x, kh, kw, st, pd, dl) @ w.reshape(O, -1).T
    ref = F.conv2d(torch.from_numpy(x).permute(0, 3, 1, 2), torch.from_numpy(w).permute(0, 3, 1, 2), stride=st,
                   padding=pd, dilation=dl).permute(0, 2, 3, 1).numpy()
    assert y.shape == (Nb * ref.shape[1] * ref.shape[2], O)
    np.testing.assert_allclose(y.reshape(ref.shape), ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("g", GEOMS)
def test_folded_gradients_are_autograds(g):
    Nb, H, W, Cc, O, kh, kw, st, pd, dl = g
    x, w, gy = _data(g, 1)
    xt = torch.from_numpy(x).permute(0, 3, 1, 2).requires_grad_(True)
    wt = torch.from_numpy(w).permute(0, 3, 1, 2).requires_grad_(True)
    F.conv2d(xt, wt, stride=st, padding=pd, dilation=dl).backward(torch.from_numpy(gy).permute(0, 3, 1, 2))
    g2 = gy.reshape(-1, O)
    dx = orc.col2im(g2 @ w.reshape(O, -1), x.shape, kh, kw, st, pd, dl)                 # g_x = g_y . w, folded
    dw = (g2.T @ orc.im2col(x, kh, kw, st, pd, dl)).reshape(O, kh, kw, Cc)              # g_w = g_y^T . x
    np.testing.assert_allclose(dx, xt.grad.permute(0, 2, 3, 1).numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dw, wt.grad.permute(0, 2, 3, 1).numpy(), rtol=1e-11, atol=1e-11)


@pytest.mark.parametrize("g", GEOMS)
def test_adjoint_identity(g):
    Nb, H, W, Cc, O, kh, kw, st, pd, dl = g
    rng = np.random.default_rng(2)
    x = rng.integers(-50, 50, (Nb, H, W, Cc)).astype(np.float64)
    cols = orc.im2col(x, kh, kw, st, pd, dl)
    y = rng.integers(-50, 50, cols.shape).astype(np.float64)
    assert np.sum(cols * y) == np.sum(x * orc.col2im(y, x.shape, kh, kw, st, pd, dl))    # integers: exact


def test_six_loops_on_a_tiny_case():
    Nb, H, W, Cc, kh, kw, st, pd, dl = 2, 4, 5, 2, 3, 2, (2, 1), (1, 0), (1, 2)
    Ho = (H + 2 * pd[0] - dl[0] * (kh - 1) - 1) // st[0] + 1
    Wo = (W + 2 * pd[1] - dl[1] * (kw - 1) - 1) // st[1] + 1
    x = np.arange(Nb * H * W * Cc, dtype=np.float64).reshape(Nb, H, W, Cc) + 1.0
    want = np.zeros((Nb * Ho * Wo, kh * kw * Cc))
    fold = np.zeros_like(x)
    y = np.arange(want.size, dtype=np.float64).reshape(want.shape) % 7 - 3
    for n in range(Nb):
        for ho in range(Ho):
            for wo in range(Wo):
                for ky in range(kh):
                    for kx in range(kw):
                        for c in range(Cc):
                            hi, wi = ho * st[0] - pd[0] + ky * dl[0], wo * st[1] - pd[1] + kx * dl[1]
                            row, col = (n * Ho + ho) * Wo + wo, (ky * kw + kx) * Cc + c
                            if 0 <= hi < H and 0 <= wi < W:
                                want[row, col] = x[n, hi, wi, c]
                                fold[n, hi, wi, c] += y[row, col]
    assert np.array_equal(orc.im2col(x, kh, kw, st, pd, dl), want)
    assert np.array_equal(orc.col2im(y, x.shape, kh, kw, st, pd, dl), fold)


def test_pointwise_kernel_is_the_identity():
    x = np.random.default_rng(3).standard_normal((2, 4, 4, 8))
    assert np.array_equal(orc.im2col(x, 1, 1), x.reshape(32, 8))
    assert np.array_equal(orc.col2im(x.reshape(32, 8), x.shape, 1, 1), x)


def test_full_rank_unquantised_limit_of_the_layer_pass():
    """With r = B the g_w list is exact: dW of the convolution pass equals autograd's up to the
    bf16 rounding of the transformed operands."""
    g = (2, 8, 8, 8, 16, 3, 3, (1, 1), (1, 1), (1, 1))
    Nb, H, W, Cc, O, kh, kw, st, pd, dl = g
    x, w, gy = _data(g, 4)
    x, w, gy = (orc.round_bf16(a.astype(np.float32)) for a in (x, w, gy))
    out = orc.conv2d_backward(gy, x, w, 16, 16, seed=5, stride=st, pad=pd, dil=dl)
    xt = torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(w.astype(np.float64)).permute(0, 3, 1, 2).requires_grad_(True)
    F.conv2d(xt, wt, stride=st, padding=pd, dilation=dl).backward(torch.from_numpy(gy.astype(np.float64)).permute(0, 3, 1, 2))
    ref = wt.grad.permute(0, 2, 3, 1).numpy()
    err = np.abs(out["dW_k"] - ref).max() / np.sqrt(np.mean(ref ** 2))
    assert err < 2e-2, err
    assert out["dX_img"].shape == x.shape
