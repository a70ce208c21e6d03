"""The library's calls inside a captured HIP graph (how the benchmark launches them): several replays,
with eager work and synchronisation in between and new input data each time, every replay checked
against the oracle.  Covers the state a call leaves for the next one (arrival counters back at zero,
flag words rewritten, partial sums overwritten)."""
import numpy as np
import pytest
import torch

import paper_2006_04984_amd as abed
from synth import ConvShape, int8_tensors

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_replays_match_the_oracle(oracle):
    from gpu_helpers import GpuConv
    from test_gpu_fic import GpuFic
    from test_gpu_ic2 import GpuIc2
    from test_gpu_fic_inloop import GpuFicInloop
    s = ConvShape(37, 9, 8, 32, 144, 3, 3, 1, 1, 1, 1, "graph_n37_k144")      # several batch and filter tiles: exchange on both axes
    x0, w = int8_tensors(s, 8080)
    g = GpuConv(s, 4); g.prepare(w)
    f = GpuFic(s, 4); f.prepare(w)
    i2 = GpuIc2(s, 4)
    fl = GpuFicInloop(s); fl.prepare(w)
    xd = torch.from_numpy(x0).to(DEV)
    wd = torch.from_numpy(w).to(DEV)
    g.x = f.x = i2.x = fl.x = xd
    i2.w = wd

    def step():
        abed.conv_int8(g.desc, xd, g.w, g.wchk, g.xchk, True, g.y, 4, flags=g.flags, workspace=g.ws)
        abed.fic_conv_int8(f.desc, xd, f.w, f.wsum, f.xrows, True, f.y, 4, f.result, f.flag, workspace=f.ws)
        abed.ic2_conv_int8(i2.desc, xd, wd, i2.xrows, True, i2.y, 4, i2.result, i2.flags, workspace=i2.ws)
        abed.fic_inloop_conv_int8(fl.desc, xd, fl.w, fl.wdig, fl.y, fl.result, fl.flag, workspace=fl.ws)

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        step()                                     # eager once (also warms up)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            step()
    torch.cuda.synchronize()
    for rep in range(4):
        x, _ = int8_tensors(s, 8080 + rep)
        xd.copy_(torch.from_numpy(x).to(DEV))      # eager work between the replays
        g.flags.fill_(-1); f.flag.fill_(-1); i2.flags.fill_(-1); fl.flag.fill_(-1); fl.result.fill_(-7)
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            graph.replay()
        torch.cuda.synchronize()
        ref = oracle.abed_int8(x, w, s)
        assert np.array_equal(g.y.cpu().numpy(), ref["y"]), rep
        assert not g.flags.cpu().numpy()[: g.lay.n_flag_words].any(), rep
        rf = oracle.abed_fic_int8(x, w, s)
        r = f.result.cpu().numpy()
        assert (int(r[0]), int(r[1]), int(f.flag.item())) == (rf["ocs"], rf["dot"], 0), rep
        r = fl.result.cpu().numpy()
        assert (int(r[0]), int(r[1]), int(fl.flag.item())) == (rf["ocs"], rf["dot"], 0), rep
        assert np.array_equal(fl.y.cpu().numpy(), rf["y"]), rep
        r2 = oracle.abed_ic2_int8(x, w, s)
        ri = i2.result.cpu().numpy()
        assert np.array_equal(ri[0], r2["osum"]) and np.array_equal(ri[1], r2["chk"]) and not i2.flags.cpu().numpy().any(), rep
