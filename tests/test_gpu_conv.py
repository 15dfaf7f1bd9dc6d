"""Convolution layers on the GPU (Sec. 3.1) against the oracle: the column matrix bit for bit, its
adjoint exactly on small integers and to fp32 rounding otherwise, and the whole backward pass of a
convolution to the bar of the linear layer's."""
import numpy as np
import pytest
import torch

import oracle
import paper_2406_15102_amd as hlq
from paper_2406_15102_amd import workloads as wl
from test_gpu_parity import TOL_OUT, row_rel_err, same_up_to_split_order

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

# Nb, H, W, C, O, kh, kw, stride, pad, dil, dtype
GEOMS = [
    (4, 14, 14, 32, 64, 3, 3, (1, 1), (1, 1), (1, 1), "bf16"),     # ResNet-style 3x3
    (4, 16, 16, 16, 32, 3, 3, (2, 2), (1, 1), (1, 1), "bf16"),     # strided
    (2, 8, 8, 64, 32, 1, 1, (1, 1), (0, 0), (1, 1), "bf16"),       # pointwise: its own column matrix
    (4, 8, 8, 32, 32, 1, 1, (2, 2), (0, 0), (1, 1), "bf16"),       # 1x1 with a stride: pixels nobody reads
    (4, 12, 16, 8, 16, 3, 2, (1, 2), (2, 1), (2, 1), "bf16"),      # dilated, non-square, uneven strides and pads
    (4, 8, 8, 4, 16, 2, 2, (2, 2), (0, 0), (1, 1), "bf16"),        # 4 channels: element-wise lanes
    (4, 8, 8, 2, 16, 2, 2, (2, 2), (0, 0), (1, 1), "f32"),         # same in fp32
    (4, 8, 8, 4, 16, 2, 2, (2, 2), (0, 0), (1, 1), "f32"),
    (2, 32, 32, 8, 16, 7, 7, (2, 2), (3, 3), (1, 1), "bf16"),      # stem-like 7x7 / 2
    (16, 14, 14, 64, 64, 3, 3, (1, 1), (1, 1), (1, 1), "bf16"),    # several GEMM tiles
    (2, 10, 10, 16, 16, 3, 3, (1, 1), (0, 0), (1, 1), "f32"),      # no padding, 8x8 output
]


def _geom(g):
    Nb, H, W, C, O, kh, kw, st, pd, dl, dtype = g
    return hlq.hlq_conv_geom(Nb=Nb, H=H, W=W, C=C, O=O, kh=kh, kw=kw, stride_h=st[0], stride_w=st[1], pad_h=pd[0],
                             pad_w=pd[1], dil_h=dl[0], dil_w=dl[1])


def _tensors(g):
    Nb, H, W, C, O, kh, kw, st, pd, dl, dtype = g
    Ho, Wo, N, I = hlq.hlq_conv_sizes(_geom(g))
    assert (Ho, Wo) == (oracle.conv_out_size(H, kh, st[0], pd[0], dl[0]), oracle.conv_out_size(W, kw, st[1], pd[1], dl[1]))
    assert N == Nb * Ho * Wo and I == kh * kw * C
    return wl.generate_conv(Nb, H, W, C, O, kh, kw, Ho, Wo, dtype), N, I


@pytest.mark.parametrize("g", GEOMS)
def test_column_matrix_bit_exact(g):
    Nb, H, W, C, O, kh, kw, st, pd, dl, dtype = g
    t, N, I = _tensors(g)
    X = t["X"].to(DEV).contiguous()
    cols = torch.full((N, I), 7.0, dtype=X.dtype, device=DEV)
    hlq.hlq_im2col(X, _geom(g), cols)
    torch.cuda.synchronize()
    ref = oracle.im2col(wl.as_f32_numpy(t["X"]), kh, kw, st, pd, dl)
    assert np.array_equal(wl.as_f32_numpy(cols), ref)


@pytest.mark.parametrize("g", GEOMS)
def test_fold_matches_adjoint(g):
    Nb, H, W, C, O, kh, kw, st, pd, dl, dtype = g
    _, N, I = _tensors(g)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    rng = np.random.default_rng(11)
    small = rng.integers(-2, 3, (N, I)).astype(np.float32)          # sums of <= 49 of these are exact in bf16
    dX = torch.full((Nb, H, W, C), 7.0, dtype=tdt, device=DEV)
    hlq.hlq_col2im(torch.from_numpy(small).to(tdt).to(DEV), _geom(g), dX)
    torch.cuda.synchronize()
    assert np.array_equal(wl.as_f32_numpy(dX).astype(np.float64), oracle.col2im(small, (Nb, H, W, C), kh, kw, st, pd, dl))
    if dtype == "f32":
        y = rng.standard_normal((N, I)).astype(np.float32)
        hlq.hlq_col2im(torch.from_numpy(y).to(DEV), _geom(g), dX)
        torch.cuda.synchronize()
        ref = oracle.col2im(y, (Nb, H, W, C), kh, kw, st, pd, dl)
        assert np.max(np.abs(wl.as_f32_numpy(dX) - ref)) <= 1e-6 * kh * kw * np.max(np.abs(y))


def _oracle_pass(t, g, B, r, seed, flags):
    Nb, H, W, C, O, kh, kw, st, pd, dl, dtype = g
    return oracle.conv2d_backward(
        wl.as_f32_numpy(t["G"]), wl.as_f32_numpy(t["X"]), wl.as_f32_numpy(t["W"]), B, r, seed, stride=st, pad=pd, dil=dl,
        gx_bits=8 if flags & hlq.HLQ_FLAG_GX_8BIT else 4, gw_int8=bool(flags & hlq.HLQ_FLAG_GW_INT8),
        basis=1 if flags & hlq.HLQ_FLAG_GW_SEQUENCY else 0, rounding=1 if flags & hlq.HLQ_FLAG_ROUND_MANTISSA else 0)


@pytest.mark.parametrize("g,flags", [(g, 0) for g in GEOMS] + [
    (GEOMS[1], hlq.HLQ_FLAG_GW_INT8), (GEOMS[4], hlq.HLQ_FLAG_GX_8BIT | hlq.HLQ_FLAG_GW_SEQUENCY),
    (GEOMS[9], hlq.HLQ_FLAG_GW_INT8 | hlq.HLQ_FLAG_GX_UNPACKED), (GEOMS[10], hlq.HLQ_FLAG_ROUND_MANTISSA),
    (GEOMS[1], hlq.HLQ_FLAG_ROUND_MANTISSA | hlq.HLQ_FLAG_GW_INT8), (GEOMS[0], hlq.HLQ_FLAG_SEPARATE_PRODUCTS)])
def test_convolution_backward_matches_oracle(g, flags):
    Nb, H, W, C, O, kh, kw, st, pd, dl, dtype = g
    B, r, seed = 16, 8, 5
    t, N, I = _tensors(g)
    G, X, Wt = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    geom = _geom(g)
    dX = torch.full_like(X, 7.0)
    dW = torch.full_like(Wt, 7.0)
    ws = torch.empty(hlq.hlq_conv_workspace_bytes(geom, B, r, hlq.binding._dt(G), flags), dtype=torch.uint8, device=DEV)
    assert ws.numel() > 0
    print("conv case", g, "flags", flags, flush=True)
    hlq.hlq_conv2d_backward(G, X, Wt, geom, B, r, seed, flags, dX, dW, ws)
    torch.cuda.synchronize()
    ref = _oracle_pass(t, g, B, r, seed, flags)
    bf = dtype == "bf16"
    # the image gradient is judged per pixel over its channels when there are enough of them, else per image row
    cols_x = C if C >= 16 else W * C
    ex = row_rel_err(wl.as_f32_numpy(dX).reshape(-1, cols_x), ref["dX_img"].reshape(-1, cols_x), bf)
    ew = row_rel_err(wl.as_f32_numpy(dW).reshape(O, I), ref["dW_k"].reshape(O, I), bf)
    assert ex < TOL_OUT and ew < TOL_OUT, (ex, ew)
    # each output alone: the same dX bits, dW up to the order of its k splits; the library-owned workspace
    dX1 = torch.full_like(X, 3.0)
    dW1 = torch.full_like(Wt, 3.0)
    hlq.hlq_conv2d_backward(G, X, Wt, geom, B, r, seed, flags, dX1, None, ws)
    hlq.hlq_conv2d_backward(G, X, Wt, geom, B, r, seed, flags, None, dW1)
    torch.cuda.synchronize()
    assert torch.equal(dX1, dX) and same_up_to_split_order(dW1, dW)


def test_pointwise_convolution_is_the_linear_layer():
    g = GEOMS[2]
    Nb, H, W, C, O, kh, kw, st, pd, dl, dtype = g
    t, N, I = _tensors(g)
    G, X, Wt = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    dX, dW = torch.empty_like(X), torch.empty_like(Wt)
    hlq.hlq_conv2d_backward(G, X, Wt, _geom(g), 16, 8, 9, 0, dX, dW)
    dX2, dW2 = torch.empty((N, C), dtype=X.dtype, device=DEV), torch.empty((O, C), dtype=X.dtype, device=DEV)
    hlq.hlq_linear_backward_ex(G.reshape(N, O), X.reshape(N, C), None, Wt.reshape(O, C), N, C, O, 16, 8, 9, dX2, dW2)
    torch.cuda.synchronize()
    assert torch.equal(dX.reshape(N, C), dX2) and torch.equal(dW.reshape(O, C), dW2)


def test_rejections_leave_outputs_untouched():
    g = GEOMS[0]
    t, N, I = _tensors(g)
    G, X, Wt = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    dX, dW = torch.full_like(X, 7.0), torch.full_like(Wt, 7.0)
    small = torch.empty(1024, dtype=torch.uint8, device=DEV)
    for kwargs in (dict(B=20), dict(r=3), dict(workspace=small)):
        a = dict(B=16, r=8, workspace=None)
        a.update(kwargs)
        with pytest.raises(hlq.HlqError):
            hlq.hlq_conv2d_backward(G, X, Wt, _geom(g), a["B"], a["r"], 0, 0, dX, dW, a["workspace"])
    torch.cuda.synchronize()
    assert bool((dX == 7.0).all()) and bool((dW == 7.0).all())


@pytest.mark.parametrize("g,B,r,basis", [(GEOMS[0], 16, 8, 0), (GEOMS[9], 16, 4, 1), (GEOMS[0], 16, 8, 1), (GEOMS[1], 32, 16, 0),
                                         (GEOMS[9], 64, 32, 1), (GEOMS[4], 16, 8, 0), (GEOMS[8], 16, 2, 0),
                                         (GEOMS[7], 32, 8, 0), (GEOMS[10], 32, 32, 0), (GEOMS[3], 16, 16, 1)])
def test_compression_straight_from_the_image_equals_that_of_the_column_matrix(g, B, r, basis):
    Nb, H, W, C, O, kh, kw, st, pd, dl, dtype = g
    t, N, I = _tensors(g)
    Kc = N // B * r
    X = t["X"].to(DEV).contiguous()
    geom = _geom(g)
    cols = torch.empty((N, I), dtype=X.dtype, device=DEV)
    hlq.hlq_im2col(X, geom, cols)
    a, b = (torch.full((I, Kc), 3.0, dtype=torch.bfloat16, device=DEV) for _ in range(2))
    ca, cb = (torch.full((I, Kc), 3.0, dtype=torch.float32, device=DEV) for _ in range(2))
    hlq.hlq_hla_project_basis(cols, B, r, basis, a, ca)
    hlq.hlq_conv_compress_act(X, geom, B, r, basis, b, cb)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(ca, cb)
    # against the oracle's projection of its own column matrix
    ref = oracle.hla_f32(oracle.im2col(wl.as_f32_numpy(t["X"]), kh, kw, st, pd, dl), B, r, basis)
    scale = np.sqrt(B) * np.maximum(np.abs(ref).max(), 1e-30)
    assert np.max(np.abs(cb.cpu().numpy() - ref)) <= 1e-5 * scale
    if r % 4 == 0 and Kc % 16 == 0:
        qa, qb = (torch.full((I, Kc), 3, dtype=torch.int8, device=DEV) for _ in range(2))
        sa, sb = (torch.full((I,), 3.0, dtype=torch.float32, device=DEV) for _ in range(2))
        ws = torch.empty(hlq.hlq_hla_quantize_workspace_bytes(I), dtype=torch.uint8, device=DEV)
        hlq.hlq_hla_quantize_basis(cols, B, r, basis, 21, 2, qa, sa, ws)
        hlq.hlq_conv_compress_act_int8(X, geom, B, r, basis, 21, qb, sb, ws)
        torch.cuda.synchronize()
        assert torch.equal(qa, qb) and torch.equal(sa, sb)


def test_image_path_refuses_channel_counts_that_split_a_lane():
    g = GEOMS[5]                                                   # 4 channels, a lane owns 8 columns at B = 16
    t, N, I = _tensors(g)
    X = t["X"].to(DEV).contiguous()
    out = torch.full((I, N // 16 * 8), 3.0, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(hlq.HlqError):
        hlq.hlq_conv_compress_act(X, _geom(g), 16, 8, 0, out)
    hlq.hlq_conv_compress_act(X, _geom(g), 32, 16, 0, torch.empty((I, N // 32 * 16), dtype=torch.bfloat16, device=DEV))
    torch.cuda.synchronize()
    assert bool((out == 3.0).all())
