"""Soak test of the cross-workgroup exchange of the layer-wide checked convolution (FC sums that span filter tiles,
IC sums that span batch tiles: partial residuals in the workspace, arrival counters, last arriver): a captured graph
of the checked layer is replayed 2000 times with alternating inputs and, every fifth time, an accumulator flip; every
replay's whole output and every flag word is compared on the device with what the oracle says for that input.  A lost
or stale partial, a counter that does not return to zero, or a flag wiped by another wave would show as a wrong flag
word in some replay."""
import numpy as np
import pytest
import torch

import paper_2006_04984_amd as abed
from synth import CONFIG2, int8_tensors, seed_for
from gpu_helpers import GpuConv, fold_flags, to_dev

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
REPLAYS = 2000


@pytest.mark.parametrize("li,variant", [(1, 4), (3, 4), (2, 3)], ids=["c128_28_ocg", "c512_7_ocg", "c256_14_partial"])
def test_exchange_soak(oracle, li, variant):
    s = CONFIG2[li]
    xa, w = int8_tensors(s, seed_for(2, li))
    xb, _ = int8_tensors(s, seed_for(2, li) + 77)
    g = GpuConv(s, variant)
    assert g.lay.grid_b > 1 and g.lay.grid_n > 1, "this layer must exchange both kinds of sums"
    g.prepare(w)
    idx = int(np.ravel_multi_index((s.N - 3, s.P // 2, 1, s.K - 5), (s.N, s.P, s.Q, s.K)))
    # what the oracle expects: outputs and folded flags of the four cases (input a / b, clean / flipped)
    exp_y, exp_f = {}, {}
    for name, x in (("a", xa), ("b", xb)):
        for flip in (None, (idx, 27)):
            r = oracle.abed_int8(x, w, s, acc_flip=flip)
            f, corner = fold_flags(r, s, g.lay)
            assert not corner.any()
            exp_y[name, flip is not None] = to_dev(r["y"].astype(np.int32))
            exp_f[name, flip is not None] = to_dev(f.reshape(-1).astype(np.int32))
        assert exp_f[name, True].any() and not exp_f[name, False].any()
    x_in = to_dev(xa).clone()
    xa_d, xb_d = to_dev(xa), to_dev(xb)
    epi = None
    stream = torch.cuda.Stream()
    bad = torch.zeros((2,), dtype=torch.int32, device=DEV)
    with torch.cuda.stream(stream):
        g.run(x_in)                                      # eager once (also sizes every buffer)
        graphs = {}
        for flipped in (False, True):
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr, stream=stream):
                abed.conv_int8(g.desc, x_in, g.w, g.wchk, g.xchk, True, g.y, g.variant, flags=g.flags, epilogue=epi,
                               workspace=g.ws, inject=(1, idx, 27) if flipped else None, stream=stream)
            graphs[flipped] = gr
        for r in range(REPLAYS):
            name = "ab"[r & 1]
            flipped = r % 5 == 4
            x_in.copy_(xa_d if name == "a" else xb_d)
            graphs[flipped].replay()
            bad[0] += (g.y != exp_y[name, flipped]).any().to(torch.int32)
            bad[1] += (g.flags[: g.lay.n_flag_words] != exp_f[name, flipped]).any().to(torch.int32)
            if r % 500 == 499:
                torch.cuda.synchronize()
                print("replays", r + 1, bad.tolist(), flush=True)
        torch.cuda.synchronize()
    assert bad.tolist() == [0, 0]
    # the arrival counters (the workspace's leading arrays) are back at zero
    cnt_bytes = (g.lay.grid_m * g.lay.grid_b * 4 + 255) // 256 * 256 + g.lay.grid_m * g.lay.grid_n * 4
    assert not g.ws[:cnt_bytes].any()
