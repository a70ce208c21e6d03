"""A workspace whose arrival counters do not start at zero (abed_workspace_init forgotten, or a stale workspace) must
not make a checked call skip its cross-tile comparisons silently: flag bit 3 (ABED_FLAG_WORKSPACE) reports it.  The
outputs do not depend on the counters."""
import numpy as np
import pytest
import torch

import paper_2006_04984_amd as abed
from paper_2006_04984_amd import Variant
from gpu_helpers import GpuConv
from synth import ConvShape, int8_tensors

pytestmark = pytest.mark.gpu

# filters and batch both span several tiles: both counters are in use
SHAPE = ConvShape(20, 12, 12, 64, 160, 3, 3, 1, 1, 1, 1, "n20_k160")


@pytest.mark.parametrize("variant", [Variant.FUSED_OCG, Variant.FUSED_IOCG])
@pytest.mark.parametrize("fill", [0xff, 0x01], ids=["all_ones", "small_counts"])
def test_stale_counters_are_reported(oracle, variant, fill):
    s = SHAPE
    x, w = int8_tensors(s, 9700)
    g = GpuConv(s, variant)
    assert g.lay.grid_n > 1 and g.lay.grid_b > 1
    g.prepare(w)
    y, flags = g.run(x)
    assert not flags.any()                               # initialised workspace: clean
    ref = oracle.conv_int(x, w, s).astype(np.int32)
    assert np.array_equal(y, ref)
    g.ws.fill_(fill)                                     # counters now hold 0xffffffff / 0x01010101
    y, flags = g.run(x)
    assert np.array_equal(y, ref)
    assert (flags & 8).any(), "stale arrival counters went unnoticed"
    abed.workspace_init(g.ws)                            # and the remedy works
    y, flags = g.run(x)
    assert not flags.any() and np.array_equal(y, ref)
