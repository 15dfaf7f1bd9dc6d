"""The library's measurement switches (hlq_set_option) change how the work is laid out on the chip,
never what is computed: with either setting the whole path must give the same bits.  (That the
direct-to-LDS form of the products is right against the oracle is checked by the full-size
workloads, which take it by default; the persistent form is compared with it here.)"""
import pytest
import torch

import paper_2406_15102_amd as hlq
from paper_2406_15102_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run(w, G, X, W, seed=3, flags=0):
    N, I, O, B, r = w.N, w.d_in, w.d_out, w.B, w.r
    dX = torch.zeros((N, I), dtype=torch.bfloat16, device=DEV)
    dW = torch.zeros((O, I), dtype=torch.bfloat16, device=DEV)
    ws = torch.zeros(hlq.hlq_workspace_bytes_mode(N, I, O, B, r, False, flags), dtype=torch.uint8, device=DEV)
    hlq.hlq_linear_backward_mode(G, X, None, None, W, N, I, O, B, r, seed, flags, dX, dW, ws)
    torch.cuda.synchronize()
    return dX, dW


@pytest.mark.parametrize("B,r,flags", [(16, 8, 0), (32, 8, 0), (64, 32, 0), (16, 8, hlq.HLQ_FLAG_GW_INT8)])
def test_persistent_products_same_bits(B, r, flags):
    # 1024 + 128 tiles of 256 x 256 on 256 compute units: enough for the persistent form to be chosen
    w = wl.scaled(wl.WORKLOADS["c5_r8"], N=8192, d_in=8192, d_out=1024, B=B, r=r)
    t = wl.generate(w)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    try:
        hlq.hlq_set_option(hlq.HLQ_OPT_PERSISTENT_PRODUCTS, 0)
        dX0, dW0 = _run(w, G, X, W, flags=flags)
        hlq.hlq_set_option(hlq.HLQ_OPT_PERSISTENT_PRODUCTS, 1)
        dX1, dW1 = _run(w, G, X, W, flags=flags)
    finally:
        hlq.hlq_set_option(hlq.HLQ_OPT_PERSISTENT_PRODUCTS, 0)
    assert torch.equal(dX0, dX1) and torch.equal(dW0, dW1)
    assert float(dX1.float().abs().max()) > 0 and float(dW1.float().abs().max()) > 0


def test_persistent_products_ragged_edges_same_bits():
    # tiles that hang over both edges of either product (sizes that are no multiples of 256)
    w = wl.scaled(wl.WORKLOADS["c5_r8"], N=8192 - 64, d_in=8192 - 104, d_out=1024 + 64, B=32, r=16)
    t = wl.generate(w)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    try:
        hlq.hlq_set_option(hlq.HLQ_OPT_PERSISTENT_PRODUCTS, 0)
        dX0, dW0 = _run(w, G, X, W)
        hlq.hlq_set_option(hlq.HLQ_OPT_PERSISTENT_PRODUCTS, 1)
        dX1, dW1 = _run(w, G, X, W)
    finally:
        hlq.hlq_set_option(hlq.HLQ_OPT_PERSISTENT_PRODUCTS, 0)
    assert torch.equal(dX0, dX1) and torch.equal(dW0, dW1)


@pytest.mark.parametrize("B,r,N", [(16, 8, 2048), (32, 8, 2048 + 32), (64, 64, 2048), (16, 2, 2048 + 128)])
def test_shared_read_of_g_same_bits(B, r, N):
    # a G of 32 MB or more (the shared read is only taken for large tensors), token counts that are
    # and are not multiples of the 64-row groups
    w = wl.scaled(wl.WORKLOADS["c4"], N=N, d_in=1032, d_out=8192, B=B, r=r)   # a weight too large for the one-launch front
    t = wl.generate(w)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    try:
        hlq.hlq_set_option(hlq.HLQ_OPT_SHARED_G_READ, 0)
        dX0, dW0 = _run(w, G, X, W)
        hlq.hlq_set_option(hlq.HLQ_OPT_SHARED_G_READ, 1)
        dX1, dW1 = _run(w, G, X, W)
    finally:
        hlq.hlq_set_option(hlq.HLQ_OPT_SHARED_G_READ, 0)
    assert torch.equal(dX0, dX1) and torch.equal(dW0, dW1)


@pytest.mark.parametrize("B,r,N,d_out,d_in", [
    (16, 8, 2048, 8192, 4104),          # whole turns of both jobs
    (32, 8, 2048 + 32, 8192, 4104),     # workgroups of the quantiser left over after the last turn
    (64, 64, 2048, 8192, 4104),
    (16, 2, 2048 + 128, 8192, 4104),
    (16, 8, 1008, 11008, 4104),         # rows of 5.4 chunks a lane, projection workgroups left over
    (16, 4, 4096, 2048, 4104),          # short rows: several per workgroup of the quantiser
    (16, 8, 8192 + 16, 1024, 520),      # a small weight: everything in one launch, strips of W first
    (32, 16, 16384, 512, 264),
])
def test_front_interleave_same_bits(B, r, N, d_out, d_in):
    # the row quantiser's and the projections' workgroups in turns, or one job after the other
    w = wl.scaled(wl.WORKLOADS["c4"], N=N, d_in=d_in, d_out=d_out, B=B, r=r)
    t = wl.generate(w)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    try:
        hlq.hlq_set_option(hlq.HLQ_OPT_FRONT_INTERLEAVE, 0)
        dX0, dW0 = _run(w, G, X, W)
        hlq.hlq_set_option(hlq.HLQ_OPT_FRONT_INTERLEAVE, 1)
        dX1, dW1 = _run(w, G, X, W)
    finally:
        hlq.hlq_set_option(hlq.HLQ_OPT_FRONT_INTERLEAVE, 1)
    assert torch.equal(dX0, dX1) and torch.equal(dW0, dW1)
    assert float(dX1.float().abs().max()) > 0 and float(dW1.float().abs().max()) > 0


@pytest.mark.parametrize("B,r,N,d_out,d_in", [(16, 8, 2048, 8192, 4104), (32, 8, 2048 + 64, 4096, 1032), (16, 4, 4096, 2048, 4104)])
def test_front_interleave_integer_gw_same_bits(B, r, N, d_out, d_in):
    # integer g_w list: the row quantiser beside the passes that take the maxima, or in the launch before them
    w = wl.scaled(wl.WORKLOADS["c4"], N=N, d_in=d_in, d_out=d_out, B=B, r=r)
    t = wl.generate(w)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    try:
        hlq.hlq_set_option(hlq.HLQ_OPT_FRONT_INTERLEAVE, 0)
        dX0, dW0 = _run(w, G, X, W, flags=hlq.HLQ_FLAG_GW_INT8)
        hlq.hlq_set_option(hlq.HLQ_OPT_FRONT_INTERLEAVE, 1)
        dX1, dW1 = _run(w, G, X, W, flags=hlq.HLQ_FLAG_GW_INT8)
    finally:
        hlq.hlq_set_option(hlq.HLQ_OPT_FRONT_INTERLEAVE, 1)
    assert torch.equal(dX0, dX1) and torch.equal(dW0, dW1)
    assert float(dX1.float().abs().max()) > 0 and float(dW1.float().abs().max()) > 0


@pytest.mark.parametrize("N,d_in,d_out,B,r,flags", [
    (4096, 4096, 2048, 16, 8, 0),                                   # both products on 256-tiles, whole steps
    (4096 - 64, 4096 - 104, 2048, 32, 16, 0),                       # tiles that hang over the edges
    (4096, 4096, 2048, 16, 8, hlq.HLQ_FLAG_GW_INT8),                # integer g_w list: int8 operands for both
    (4096, 4096, 2048, 16, 8, hlq.HLQ_FLAG_GX_UNPACKED),            # one int8 per code for the g_x product
    (1024, 1024, 8192, 16, 8, 0),                                   # few tiles, long reduction for the g_x product
])
def test_direct_to_lds_same_bits(N, d_in, d_out, B, r, flags):
    w = wl.scaled(wl.WORKLOADS["c4"], N=N, d_in=d_in, d_out=d_out, B=B, r=r)
    t = wl.generate(w)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    try:
        hlq.hlq_set_option(hlq.HLQ_OPT_DIRECT_TO_LDS, 0)
        dX0, dW0 = _run(w, G, X, W, flags=flags)
        hlq.hlq_set_option(hlq.HLQ_OPT_DIRECT_TO_LDS, 1)
        dX1, dW1 = _run(w, G, X, W, flags=flags)
    finally:
        hlq.hlq_set_option(hlq.HLQ_OPT_DIRECT_TO_LDS, 1)
    assert torch.equal(dX0, dX1) and torch.equal(dW0, dW1)
    assert float(dX1.float().abs().max()) > 0 and float(dW1.float().abs().max()) > 0


@pytest.mark.parametrize("kind", ["int8", "int4", "bf16"])
@pytest.mark.parametrize("M,Nn,K,f32", [(4096, 4096, 1024, False), (4096 - 40, 4096 - 24, 2048, True),
                                         (512, 768, 32768, False)])
def test_direct_to_lds_products_same_bits(kind, M, Nn, K, f32):
    """The stage entry points of the products, operands through registers against straight into LDS:
    256-tiles with whole steps, ragged tile edges with fp32 output, a long reduction that is split."""
    gen = torch.Generator(device="cpu").manual_seed(M + K)
    out = torch.float32 if f32 else torch.bfloat16
    ws = torch.zeros(64 << 20, dtype=torch.uint8, device=DEV)
    if kind == "bf16":
        A = torch.randn((M, K), generator=gen).to(torch.bfloat16).to(DEV)
        Bm = torch.randn((Nn, K), generator=gen).to(torch.bfloat16).to(DEV)
        run = lambda C: hlq.hlq_bf16_gemm_nt(A, Bm, 1.0 / 16, C, ws)
    else:
        A = torch.randint(-7, 8, (M, K), generator=gen, dtype=torch.int8)
        Bm = torch.randint(-7, 8, (Nn, K), generator=gen, dtype=torch.int8)
        sA, sB = torch.rand(M, generator=gen).to(DEV), torch.rand(Nn, generator=gen).to(DEV)
        if kind == "int4":
            pack = lambda q: ((q[:, 0::2] & 15) | ((q[:, 1::2] & 15) << 4)).to(torch.uint8)
            A4, B4 = pack(A.to(torch.int16)).to(DEV), pack(Bm.to(torch.int16)).to(DEV)
            run = lambda C: hlq.hlq_int4_gemm_nt(A4, B4, sA, sB, 1.0 / 16, C, None, ws)
        else:
            Ad, Bd = A.to(DEV), Bm.to(DEV)
            run = lambda C: hlq.hlq_int8_gemm_nt(Ad, Bd, sA, sB, 1.0 / 16, C, None, ws)
    C0 = torch.zeros((M, Nn), dtype=out, device=DEV)
    C1 = torch.zeros((M, Nn), dtype=out, device=DEV)
    try:
        hlq.hlq_set_option(hlq.HLQ_OPT_DIRECT_TO_LDS, 0)
        run(C0)
        hlq.hlq_set_option(hlq.HLQ_OPT_DIRECT_TO_LDS, 1)
        run(C1)
        torch.cuda.synchronize()
    finally:
        hlq.hlq_set_option(hlq.HLQ_OPT_DIRECT_TO_LDS, 1)
    assert torch.equal(C0, C1)
    assert float(C1.float().abs().max()) > 0


@pytest.mark.parametrize("tile,splits", [(256, 1), (256, 2), (256, 3), (128, 1), (128, 4)])
def test_forced_plans_agree(tile, splits):
    """Every plan of the products computes the same pass: dX bit for bit, dW to the rounding of a
    different summation order; with the plan held fixed, operands through registers and straight
    into LDS give the same bits (this is what reaches the split-k form of the straight-into-LDS body)."""
    w = wl.scaled(wl.WORKLOADS["c4"], N=2048, d_in=1024 + 24, d_out=2048, B=16, r=8)   # whole k steps for both products, ragged tile edges
    t = wl.generate(w)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    dX_auto, dW_auto = _run(w, G, X, W)
    try:
        hlq.hlq_set_option(hlq.HLQ_OPT_PLAN_TILE, tile)
        hlq.hlq_set_option(hlq.HLQ_OPT_PLAN_SPLITS, splits)
        Kc = w.N // w.B * w.r
        plan = hlq.hlq_backward_products_plan(w.N, w.d_in, w.d_out, Kc, hlq.HLQ_BITS_4_PACKED, False, 1 << 28)
        assert plan[:3] == (tile, tile, splits)
        dX1, dW1 = _run(w, G, X, W)
        hlq.hlq_set_option(hlq.HLQ_OPT_DIRECT_TO_LDS, 0)
        dX0, dW0 = _run(w, G, X, W)
    finally:
        hlq.hlq_set_option(hlq.HLQ_OPT_DIRECT_TO_LDS, 1)
        hlq.hlq_set_option(hlq.HLQ_OPT_PLAN_TILE, 0)
        hlq.hlq_set_option(hlq.HLQ_OPT_PLAN_SPLITS, 0)
    assert torch.equal(dX0, dX1) and torch.equal(dW0, dW1)
    assert torch.equal(dX1, dX_auto)
    d = (dW1.float() - dW_auto.float()).abs()
    assert float((d / (dW_auto.float().abs() + 1e-6)).median()) < 1e-2 and float(d.max()) <= 2 ** -6 * float(dW_auto.float().abs().max())


@pytest.mark.parametrize("N,d_in,d_out", [(1024, 4096, 4352), (1024, 4096 - 24, 4352 - 32), (2048, 2048, 8192 + 256)])
def test_tail_tiles_same_bits(N, d_in, d_out):
    """The last rows of the g_w product in 192-row tiles (taken when its last round on 256-row tiles
    would be partly empty) against 256-row tiles throughout: the same bits.  256-tiles are forced so
    that the small g_x product does not move the plan to 128-tiles."""
    w = wl.scaled(wl.WORKLOADS["c4"], N=N, d_in=d_in, d_out=d_out, B=16, r=8)
    t = wl.generate(w)
    G, X, W = (t[k].to(DEV).contiguous() for k in ("G", "X", "W"))
    try:
        hlq.hlq_set_option(hlq.HLQ_OPT_PLAN_TILE, 256)
        hlq.hlq_set_option(hlq.HLQ_OPT_PLAN_SPLITS, 1)
        hlq.hlq_set_option(hlq.HLQ_OPT_TAIL_TILES, 0)
        dX0, dW0 = _run(w, G, X, W)
        hlq.hlq_set_option(hlq.HLQ_OPT_TAIL_TILES, 1)
        dX1, dW1 = _run(w, G, X, W)
    finally:
        hlq.hlq_set_option(hlq.HLQ_OPT_TAIL_TILES, 1)
        hlq.hlq_set_option(hlq.HLQ_OPT_PLAN_TILE, 0)
        hlq.hlq_set_option(hlq.HLQ_OPT_PLAN_SPLITS, 0)
    assert torch.equal(dX0, dX1) and torch.equal(dW0, dW1)
    assert float(dW1.float().abs().max()) > 0


@pytest.mark.parametrize("kind", ["int8", "bf16"])
@pytest.mark.parametrize("M,Nn,K,f32", [(4352, 4096, 512, False), (4352 - 40, 4096 - 24, 1024, True), (8192 + 300, 2048, 512, False)])
def test_tail_tiles_products_same_bits(kind, M, Nn, K, f32):
    """A product launched alone: 272 (or 272 ragged, or 264) tiles of 256 x 256 leave a last round of a few
    tiles, which the 192-row tiles take over."""
    gen = torch.Generator(device="cpu").manual_seed(M + K)
    out = torch.float32 if f32 else torch.bfloat16
    if kind == "bf16":
        A = torch.randn((M, K), generator=gen).to(torch.bfloat16).to(DEV)
        Bm = torch.randn((Nn, K), generator=gen).to(torch.bfloat16).to(DEV)
        run = lambda C: hlq.hlq_bf16_gemm_nt(A, Bm, 1.0 / 16, C, None)
    else:
        A = torch.randint(-127, 128, (M, K), generator=gen, dtype=torch.int8).to(DEV)
        Bm = torch.randint(-127, 128, (Nn, K), generator=gen, dtype=torch.int8).to(DEV)
        sA, sB = torch.rand(M, generator=gen).to(DEV), torch.rand(Nn, generator=gen).to(DEV)
        run = lambda C: hlq.hlq_int8_gemm_nt(A, Bm, sA, sB, 1.0 / 16, C, None, None)
    C0 = torch.zeros((M, Nn), dtype=out, device=DEV)
    C1 = torch.zeros((M, Nn), dtype=out, device=DEV)
    try:
        hlq.hlq_set_option(hlq.HLQ_OPT_TAIL_TILES, 0)
        run(C0)
        hlq.hlq_set_option(hlq.HLQ_OPT_TAIL_TILES, 1)
        run(C1)
        torch.cuda.synchronize()
    finally:
        hlq.hlq_set_option(hlq.HLQ_OPT_TAIL_TILES, 1)
    assert torch.equal(C0, C1)
    assert float(C1.float().abs().max()) > 0


def test_unknown_option_is_refused():
    with pytest.raises(hlq.HlqError) as ei:
        hlq.hlq_set_option(99, 1)
    assert ei.value.status == 2
    with pytest.raises(hlq.HlqError):
        hlq.hlq_set_option(hlq.HLQ_OPT_PLAN_TILE, 192)
    with pytest.raises(hlq.HlqError):
        hlq.hlq_set_option(hlq.HLQ_OPT_PLAN_SPLITS, 17)
