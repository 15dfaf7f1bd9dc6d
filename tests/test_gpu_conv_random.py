"""Seeded sweep of convolution geometries through the whole backward pass against the oracle: kernel
sizes 1 to 5 in either direction, strides, pads and dilations of 1 to 2 mixed freely, channel counts
that take the vector and the element-wise lanes, image sizes that leave ragged tiles everywhere."""
import numpy as np
import pytest

import oracle
from test_gpu_conv import test_convolution_backward_matches_oracle as _check

pytestmark = pytest.mark.gpu


def _geometries(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        Nb, H, W = int(rng.choice([2, 4, 8, 16])), int(rng.integers(6, 21)), int(rng.integers(6, 21))
        C, O = int(rng.choice([4, 8, 16, 24, 32, 64])), int(rng.choice([16, 32, 48, 64, 128, 272]))
        kh, kw = int(rng.choice([1, 2, 3, 5])), int(rng.choice([1, 2, 3, 5]))
        st = (int(rng.integers(1, 3)), int(rng.integers(1, 3)))
        pd = (int(rng.integers(0, 3)), int(rng.integers(0, 3)))
        dl = (int(rng.integers(1, 3)), int(rng.integers(1, 3)))
        if pd[0] > (kh - 1) * dl[0] or pd[1] > (kw - 1) * dl[1]:
            continue                                   # more padding than the kernel reaches
        Ho, Wo = oracle.conv_out_size(H, kh, st[0], pd[0], dl[0]), oracle.conv_out_size(W, kw, st[1], pd[1], dl[1])
        if Ho < 1 or Wo < 1 or (Nb * Ho * Wo) % 16 or (kh * kw * C) % 8:
            continue                                   # the layer's own shape rules (B = 16, r = 8)
        out.append((Nb, H, W, C, O, kh, kw, st, pd, dl, "bf16" if rng.random() < 0.7 else "f32"))
    return out


@pytest.mark.parametrize("g", _geometries(30, 5))
def test_random_geometry_matches_oracle(g):
    _check(g, 0)
