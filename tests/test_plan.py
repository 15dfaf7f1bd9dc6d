"""Regression guard for the cost model that lays out the two matrix products of a pass (tile sizes, k
split of the g_w product, dispatch order).  Its constants were fitted to a sweep of every plan over
these layer shapes on MI355X, where the picked plan measured within 2 % of the best one; a change
to the model that moves any of these picks has to come with a new sweep.  Host arithmetic only."""
import pytest

import paper_2406_15102_amd as hlq
from paper_2406_15102_amd import workloads as wl

# workload -> (tile edge of the g_x product, of the g_w product, k splits of the g_w product, g_w first)
MEASURED_PICKS = {
    "c2": (128, 128, 1, 1), "c3": (128, 128, 2, 1),
    "c4": (256, 256, 1, 0), "c4_b32": (256, 256, 1, 0), "c4_b64": (256, 256, 1, 0),
    "c5_r4": (256, 256, 1, 0), "c5_r8": (256, 256, 1, 0), "c5_r16": (256, 256, 1, 0),
    "p01": (128, 128, 6, 1), "p02": (128, 128, 4, 0), "p05": (128, 128, 12, 1), "p07": (128, 128, 12, 1),
    "p08": (128, 128, 6, 1), "p09": (128, 128, 16, 0), "p10": (128, 128, 6, 0), "p12": (128, 128, 1, 0),
}


@pytest.mark.parametrize("name", sorted(MEASURED_PICKS))
def test_pair_plan_picks_the_measured_plan(name):
    w = wl.WORKLOADS[name]
    Kc = w.N // w.B * w.r
    bits = hlq.HLQ_BITS_4_PACKED if w.d_out % 32 == 0 else hlq.HLQ_BITS_4
    plan = hlq.hlq_backward_products_plan(w.N, w.d_in, w.d_out, Kc, bits, False, 1 << 28)
    assert plan[:4] == MEASURED_PICKS[name], plan


def test_plan_properties():
    # without scratch the g_w product is never split; the split never exceeds its k steps
    for name in ("c3", "p05", "p09"):
        w = wl.WORKLOADS[name]
        Kc = w.N // w.B * w.r
        assert hlq.hlq_backward_products_plan(w.N, w.d_in, w.d_out, Kc, hlq.HLQ_BITS_4_PACKED, False, 0)[2] == 1
        s = hlq.hlq_backward_products_plan(w.N, w.d_in, w.d_out, Kc, hlq.HLQ_BITS_4_PACKED, False, 1 << 28)[2]
        assert 1 <= s <= (2 * Kc + 127) // 128
        assert s * w.d_out * w.d_in * 4 <= 1 << 28
    with pytest.raises(hlq.HlqError):
        hlq.hlq_backward_products_plan(4096, 4096, 11000, 2048, hlq.HLQ_BITS_4_PACKED)   # d_out % 32 for packed codes
