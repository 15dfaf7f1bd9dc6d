"""hlq_quantize_w_static -- the entry point for callers that cannot allocate (its scratch is a
device array inside the library) -- against hlq_quantize_w on a caller workspace: same codes and
scales bit for bit, on two calls in a row, the second on a smaller weight (the array keeps the first
call's column maxima; each call must clear what it uses)."""
import pytest
import torch

import paper_2406_15102_amd as hlq
from paper_2406_15102_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(d_out, d_in, B, seed, bits, dtype):
    rng = torch.Generator(device="cpu").manual_seed(1000 + d_out + d_in)
    W = (torch.randn((d_out, d_in), generator=rng) * 0.02).to(dtype).to(DEV).contiguous()
    packed = bits == hlq.HLQ_BITS_4_PACKED
    cols = d_out // 2 if packed else d_out
    out = []
    for static in (False, True):
        WqT = torch.full((d_in, cols), 0x55, dtype=torch.uint8 if packed else torch.int8, device=DEV)
        sW = torch.full((d_in,), -1.0, dtype=torch.float32, device=DEV)
        if static:
            hlq.hlq_quantize_w_static(W, B, seed, WqT, sW, bits)
        else:
            ws = torch.empty(hlq.hlq_quantize_w_workspace_bytes(d_out, d_in), dtype=torch.uint8, device=DEV)
            hlq.hlq_quantize_w(W, B, seed, WqT, sW, ws, None, bits)
        torch.cuda.synchronize()
        out.append((WqT, sW))
    return out


def test_static_scratch_matches_caller_workspace_twice_in_a_row():
    # a weight spanning several workgroups both ways with ragged edges, then a smaller one whose
    # columns all had larger maxima in the first call
    for d_out, d_in, B, bits, dtype in ((1120, 776, 16, hlq.HLQ_BITS_4_PACKED, torch.bfloat16),
                                        (192, 264, 32, hlq.HLQ_BITS_4, torch.float32)):
        (q0, s0), (q1, s1) = _both(d_out, d_in, B, 9, bits, dtype)
        assert torch.equal(s0, s1), "scales differ (%d x %d)" % (d_out, d_in)
        assert torch.equal(q0, q1), "codes differ (%d x %d)" % (d_out, d_in)
        assert float(s0.min()) > 0.0


def test_static_scratch_refuses_what_does_not_fit():
    W = torch.zeros((64, 65536 + 8), dtype=torch.bfloat16, device=DEV)
    WqT = torch.empty((65536 + 8, 64), dtype=torch.int8, device=DEV)
    sW = torch.empty(65536 + 8, dtype=torch.float32, device=DEV)
    with pytest.raises(hlq.HlqError) as ei:
        hlq.hlq_quantize_w_static(W, 16, 0, WqT, sW)
    assert ei.value.status == 6
