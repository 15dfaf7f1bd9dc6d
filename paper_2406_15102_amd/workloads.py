"""Seeded synthetic inputs shaped like the layers HLQ (arXiv 2406.15102) is applied to.

This module only draws random tensors; it contains none of the method's
arithmetic.  Both the HIP path and the CPU oracle are fed from here so that
they see the same bits.  The paper trains CNNs and ViTs on image datasets
(Sec. 7); those are not needed to exercise one layer's backward pass, so each
workload below is a stand-in with the layer's shape and a value distribution
chosen to stress what the method is for: outlier channels in X, per-token
spread in the output gradient, post-ReLU sparsity, heavy tails.

Every second distribution argument is a standard deviation.  Values are drawn
in fp32 with ``numpy.random.Generator(PCG64(seed))``, ``seed = 1000*id + k``
(k: 0 = X, 1 = W, 2 = G, 3 = auxiliary choices), and rounded once to bf16 for
the bf16 workloads, so the tensors handed out are exactly representable in the
dtype they are labelled with.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    id: int
    N: int          # tokens (batch x sequence, or batch x spatial positions)
    d_in: int
    d_out: int
    B: int          # Hadamard block order
    r: int          # kept bases per block
    dtype: str      # "bf16" | "f32"
    seed: int = 0   # stochastic-rounding seed handed to the backward call
    desc: str = ""


WORKLOADS = {
    "c1": Workload("c1", 1, 256, 256, 256, 16, 8, "f32", 0,
                   "small linear layer; X~N(0,1), W~N(0,.02), G~N(0,1e-3)"),
    "c2": Workload("c2", 2, 64 * 197, 768, 3072, 16, 8, "bf16", 0,
                   "ViT-B/16 MLP fc1; 2% of X channels x20; G per-token lognormal(0,.5) spread"),
    "c3": Workload("c3", 3, 64 * 14 * 14, 2304, 256, 16, 8, "bf16", 0,
                   "ResNet-50 stage-3 3x3 conv as im2col GEMM; X post-ReLU; W Kaiming-normal"),
    "c4": Workload("c4", 4, 2 * 2048, 4096, 11008, 16, 8, "bf16", 0,
                   "LLaMA-7B MLP up-proj; 0.5% of X channels x50; G per-token lognormal(0,1) spread"),
    "c4_b32": Workload("c4_b32", 4, 2 * 2048, 4096, 11008, 32, 16, "bf16", 0, "c4 with B=32, r=16"),
    "c4_b64": Workload("c4_b64", 4, 2 * 2048, 4096, 11008, 64, 32, "bf16", 0, "c4 with B=64, r=32"),
    "c5_r4": Workload("c5_r4", 5, 8192, 28672, 8192, 32, 4, "bf16", 0,
                      "70B-shaped MLP down-proj, one GPU's share; X Student-t(4)"),
    "c5_r8": Workload("c5_r8", 5, 8192, 28672, 8192, 32, 8, "bf16", 0, "c5 with r=8"),
    "c5_r16": Workload("c5_r16", 5, 8192, 28672, 8192, 32, 16, "bf16", 0, "c5 with r=16"),
}


# The twelve layer shapes (L, O, I) of the paper's latency table (Sec. 7, "Latency profiling
# results"), at batch 64 as in its memory table: N = 64 L.  p01-p06 are EfficientFormer-L1 layers
# (recipe of c2), p07-p12 ResNet-34 layers (recipe of c3).  The second ResNet shape is printed
# "(256, 128, 152)"; it is read as I = 1152 = 3*3*128, the only 3x3 layer with 128 channels.
_PAPER_LAYERS = [(196, 224, 896), (196, 896, 224), (196, 224, 864), (196, 864, 224), (784, 96, 432), (784, 96, 384),
                 (1024, 64, 576), (256, 128, 1152), (256, 128, 64), (64, 256, 1152), (64, 256, 128), (16, 512, 2304)]
for _k, (_L, _O, _I) in enumerate(_PAPER_LAYERS):
    _name = "p%02d" % (_k + 1)
    WORKLOADS[_name] = Workload(_name, 6 if _k < 6 else 7, 64 * _L, _I, _O, 16, 8, "bf16", 0,
                                "%s layer (L, O, I) = (%d, %d, %d) of the paper's latency table, batch 64"
                                % ("EfficientFormer-L1" if _k < 6 else "ResNet-34", _L, _O, _I))
_RECIPE = {6: 2, 7: 3}   # value distributions: as c2 (outlier channels, per-token spread) / as c3 (post-ReLU)


# Convolution geometry behind the im2col-shaped workloads: (Nb, H, W, C, kh, kw, stride, pad), channels-last.
# c3 is a 3x3 / 256-channel layer on 14x14 maps; the ResNet-34 rows of the latency table are read as
# its 3x3 layers (I = 9 C) and its 1x1 stride-2 shortcut projections (I = C), at batch 64.
CONV_GEOMS = {
    "c3": (64, 14, 14, 256, 3, 3, 1, 1),
    "p07": (64, 32, 32, 64, 3, 3, 1, 1),
    "p08": (64, 16, 16, 128, 3, 3, 1, 1),
    "p09": (64, 32, 32, 64, 1, 1, 2, 0),
    "p10": (64, 16, 16, 128, 3, 3, 2, 1),
    "p11": (64, 16, 16, 128, 1, 1, 2, 0),
    "p12": (64, 8, 8, 256, 3, 3, 2, 1),
}


def scaled(w: Workload, N: int | None = None, d_in: int | None = None, d_out: int | None = None,
           **kw) -> Workload:
    """Same recipe at another size (for parity cases the oracle finishes in seconds)."""
    return replace(w, N=N or w.N, d_in=d_in or w.d_in, d_out=d_out or w.d_out, **kw)


def _normal(rng, shape, std):
    return rng.standard_normal(shape, dtype=np.float32) * np.float32(std)


def generate(w: Workload, want=("X", "W", "G")):
    """Return {"X": [N,d_in], "W": [d_out,d_in], "G": [N,d_out]} as CPU torch tensors of w.dtype."""
    out = {}
    base = 1000 * w.id
    rid = _RECIPE.get(w.id, w.id)
    aux = np.random.Generator(np.random.PCG64(base + 3))
    if "X" in want:
        rng = np.random.Generator(np.random.PCG64(base + 0))
        if rid == 3:
            X = np.maximum(_normal(rng, (w.N, w.d_in), 1.0), np.float32(0))
        elif rid == 5:
            X = rng.standard_t(4.0, size=(w.N, w.d_in)).astype(np.float32)
        else:
            X = _normal(rng, (w.N, w.d_in), 1.0)
            if rid in (2, 4):
                frac, gain = (0.02, 20.0) if rid == 2 else (0.005, 50.0)
                n_out = max(1, int(round(frac * w.d_in)))
                ch = aux.choice(w.d_in, size=n_out, replace=False)
                X[:, ch] *= np.float32(gain)
        out["X"] = X
    if "W" in want:
        rng = np.random.Generator(np.random.PCG64(base + 1))
        std = {1: 0.02, 2: 0.02, 3: float(np.sqrt(2.0 / w.d_in)), 4: 0.02, 5: 0.01}[rid]
        out["W"] = _normal(rng, (w.d_out, w.d_in), std)
    if "G" in want:
        rng = np.random.Generator(np.random.PCG64(base + 2))
        std = {1: 1e-3, 2: 1e-3, 3: 1e-3, 4: 1e-4, 5: 1e-4}[rid]
        G = _normal(rng, (w.N, w.d_out), std)
        if rid in (2, 4):
            sigma = 0.5 if rid == 2 else 1.0
            G *= np.exp(np.float32(sigma) * rng.standard_normal((w.N, 1), dtype=np.float32))
        out["G"] = G
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    return {k: torch.from_numpy(v).to(tdt) for k, v in out.items()}


def generate_conv(Nb: int, H: int, W: int, C: int, O: int, kh: int, kw: int, Ho: int, Wo: int, dtype: str = "bf16"):
    """Channels-last tensors of a convolution layer, value recipe of c3 (post-ReLU input,
    Kaiming-normal filters, N(0, 1e-3) output gradient): {"X": [Nb,H,W,C], "W": [O,kh,kw,C],
    "G": [Nb,Ho,Wo,O]}.  The output extent (Ho, Wo) is the caller's to compute."""
    w = WORKLOADS["c3"]
    x = generate(scaled(w, N=Nb * H * W, d_in=C, dtype=dtype), want=("X",))["X"].reshape(Nb, H, W, C)
    t = generate(scaled(w, N=Nb * Ho * Wo, d_in=kh * kw * C, d_out=O, dtype=dtype), want=("W", "G"))
    return {"X": x, "W": t["W"].reshape(O, kh, kw, C), "G": t["G"].reshape(Nb, Ho, Wo, O)}


def as_f32_numpy(t: torch.Tensor) -> np.ndarray:
    """Widen (exactly) to fp32 numpy, the form the CPU oracle takes."""
    return t.detach().to("cpu", torch.float32).contiguous().numpy()
