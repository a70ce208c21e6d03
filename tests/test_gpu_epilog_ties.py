"""The fused epilog of Sec. 4.3 on accumulators chosen to land on rounding ties and on the clamp's edges, through every
int8-output kernel of the library (pixel-group kernel, box kernel, the one-wave-per-SIMD kernel, checked and unchecked):
bit for bit against the oracle's epilog (convert, scale, bias as two separately rounded fp32 operations, ReLU, round to
nearest even, clamp).  The accumulators are made exact by one-hot filters: y[n,p,q,k] = m[k] * x[n,p,q,0]."""
import numpy as np
import pytest
import torch

import paper_2006_04984_amd as abed
from gpu_helpers import GpuConv
from synth import ConvShape

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def tie_problem(s, seed):
    g = np.random.Generator(np.random.PCG64(seed))
    x = np.zeros((s.N, s.H, s.W, s.C), dtype=np.int8)
    x[..., 0] = g.integers(-128, 128, size=(s.N, s.H, s.W), dtype=np.int64).astype(np.int8)
    w = np.zeros((s.K, s.R, s.S, s.C), dtype=np.int8)
    mult = g.choice(np.array([1, -1, 2, 3, 127, -128], dtype=np.int64), size=s.K)
    w[:, s.R // 2, s.S // 2, 0] = mult.astype(np.int8)
    # scales whose products with small integers are exact halves, quarters and values at the clamp's edges
    scale = g.choice(np.array([0.5, 1.5, 0.25, 1.0, 1.00390625, 0.0078125, 2.5], dtype=np.float32), size=s.K).astype(np.float32)
    bias = g.choice(np.array([0.0, 0.5, -0.5, 127.5, -128.5, 0.25], dtype=np.float32), size=s.K).astype(np.float32)
    return x, w, scale, bias


CASES = [(ConvShape(8, 8, 8, 64, 64, 3, 3, 1, 1, 1, 1, "3x3_c64"), {}),
         (ConvShape(8, 8, 8, 64, 64, 3, 3, 1, 1, 1, 1, "3x3_c64_box"), {"ABED_BOX": "1"}),
         (ConvShape(8, 8, 8, 64, 64, 3, 3, 1, 1, 1, 1, "3x3_c64_img"), {"ABED_IMG": "1"}),
         (ConvShape(5, 14, 14, 128, 128, 3, 3, 1, 1, 1, 1, "3x3_c128_img"), {"ABED_IMG": "1"}),
         (ConvShape(6, 9, 7, 32, 48, 1, 1, 1, 1, 0, 0, "1x1_c32_k48"), {}),
         (ConvShape(3, 11, 11, 16, 24, 5, 5, 2, 2, 2, 2, "5x5_stride2"), {})]


@pytest.mark.parametrize("relu", [True, False], ids=["relu", "norelu"])
@pytest.mark.parametrize("s,env", CASES, ids=lambda v: v.name if hasattr(v, "name") else "")
def test_epilog_on_ties_and_clamp_edges(oracle, monkeypatch, s, env, relu):
    print("case", s.name, relu, flush=True)
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    x, w, scale, bias = tie_problem(s, 9800 + s.C)
    ref = oracle.epilog_int8(oracle.conv_int(x, w, s), scale, bias, relu)
    assert len(np.unique(ref)) > 20                       # the case really spreads over the int8 range
    for variant in (0, 4):
        g = GpuConv(s, variant, int8_out=True)
        g.prepare(w)
        y, flags = g.run(x, epilogue=(scale, bias, relu))
        assert np.array_equal(y, ref), "variant %d" % variant
        if variant:
            assert not flags.any()
    if s.R == 3 and s.C % 64 == 0 and "ABED_IMG" not in env:
        # checksums local to a workgroup (the box kernel's checked form)
        lay = abed.get_layout(abed.desc_from_shape(s), 0, 4 | abed.LOCAL)
        xd, wd = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
        wchk = torch.zeros((lay.grid_n * lay.d_f, s.R, s.S, s.C), dtype=torch.int8, device=DEV)
        abed.filter_prepare_local_int8(abed.desc_from_shape(s), 4 | abed.LOCAL, wd, wchk)
        y = torch.empty((s.N, s.P, s.Q, s.K), dtype=torch.int8, device=DEV)
        flags = torch.zeros((lay.n_flag_words,), dtype=torch.int32, device=DEV)
        sc, bi = torch.from_numpy(scale).to(DEV), torch.from_numpy(bias).to(DEV)
        abed.conv_int8(abed.desc_from_shape(s), xd, wd, wchk, None, True, y, 4 | abed.LOCAL, flags=flags, epilogue=(sc, bi, relu))
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy(), ref) and int(flags.abs().max().item()) == 0
