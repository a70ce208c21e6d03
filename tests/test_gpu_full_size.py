"""GPU parity at the full sizes of the configured workloads, in the launch configuration the benchmark
and the evaluation runs time (automatic tile plan): outputs on sampled elements that the oracle
computes one by one, clean flags, and one accumulator flip whose flag words follow from the tile
layout alone (FC bit on the flipped element's batch tile, IC bit on its filter tile, nothing else)."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2006_04984_amd as abed
from synth import CONFIG2, CONFIG3, int8_tensors, requant_params, resnet50_layers, seed_for

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def sample_points(s, count, seed):
    rng = np.random.default_rng(seed)
    pts = np.stack([rng.integers(0, s.N, count), rng.integers(0, s.P, count), rng.integers(0, s.Q, count),
                    rng.integers(0, s.K, count)], axis=1)
    # the corners of the output tensor too: first and last image, pixel and filter
    pts[0] = (0, 0, 0, 0)
    pts[1] = (s.N - 1, s.P - 1, s.Q - 1, s.K - 1)
    return pts


def expected_flags(lay, s, idx, scheme):
    n, pix, k = idx // (s.P * s.Q * s.K), (idx // s.K) % (s.P * s.Q), idx % s.K
    exp = np.zeros((lay.grid_m, lay.grid_b, lay.grid_n), dtype=np.uint32)
    if scheme & 1:
        exp[pix // 16, n // lay.tile_batch, 0] |= 1
    if scheme & 2:
        exp[pix // 16, 0, k // lay.tile_n] |= 2
    return exp


@pytest.mark.parametrize("variant,scheme", [(0, 0), (4, 3), (5, 3), (3, 3), (4 | abed.ONLY_FC, 1), (4 | abed.ONLY_IC, 2)],
                         ids=["unchecked", "fused_ocg", "fused_iocg", "partial", "fc_only", "ic_only"])
@pytest.mark.parametrize("li", range(4))
def test_config2_layers(oracle, li, variant, scheme):
    from gpu_helpers import GpuConv
    s = CONFIG2[li]
    print("case", s.name, hex(variant), flush=True)
    x, w = int8_tensors(s, seed_for(2, li))
    g = GpuConv(s, variant)
    g.prepare(w)
    y, flags = g.run(x)
    pts = sample_points(s, 400, 17 + li)
    exp = oracle.conv_int_points(x, w, s, pts).astype(np.int32)
    assert np.array_equal(y[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]], exp)
    if scheme:
        assert not flags.any()
        idx = int(np.ravel_multi_index(tuple(pts[7]), (s.N, s.P, s.Q, s.K)))
        y2, f2 = g.run(x, inject=(1, idx, 29))
        assert y2[tuple(pts[7])] == np.int32(exp[7] ^ (1 << 29))
        assert np.array_equal(f2.reshape(g.lay.grid_m, g.lay.grid_b, g.lay.grid_n), expected_flags(g.lay, s, idx, scheme))


@pytest.mark.parametrize("int8_out", [False, True], ids=["i32out", "i8out"])
@pytest.mark.parametrize("li", range(5))
def test_config3_layers(oracle, li, int8_out):
    from gpu_helpers import GpuConv
    s = CONFIG3[li]
    print("case", s.name, int8_out, flush=True)
    x, w = int8_tensors(s, seed_for(3, li))
    scale, bias = requant_params(s, seed_for(3, li))
    pts = sample_points(s, 400, 31 + li)
    acc = oracle.conv_int_points(x, w, s, pts).astype(np.int32)
    exp = oracle.epilog_int8(acc, scale[pts[:, 3]], bias[pts[:, 3]], True) if int8_out else acc
    for variant in (0, 4):
        g = GpuConv(s, variant, int8_out=int8_out)
        g.prepare(w)
        y, flags = g.run(x, epilogue=(scale, bias, True) if int8_out else None)
        assert np.array_equal(y[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]], exp)
        assert variant == 0 or not flags.any()
        del g
        torch.cuda.empty_cache()


# one layer of every kind of the 53-layer network at its evaluation batch (the 3-channel stem aside):
# 3x3, 1x1 expanding (the tile plan goes 8 filter blocks wide), 1x1 reducing, strided 3x3, strided 1x1
RESNET_PICKS = [2, 3, 5, 12, 14, 29, 45]


@pytest.mark.parametrize("i", RESNET_PICKS)
def test_resnet50_layers_with_epilog(oracle, i):
    from gpu_helpers import GpuConv
    s = resnet50_layers(128)[i]
    print("case", i, s.name, flush=True)
    x, w = int8_tensors(s, 5000 + i)
    scale, bias = requant_params(s, 5000 + i)
    pts = sample_points(s, 300, 41 + i)
    acc = oracle.conv_int_points(x, w, s, pts).astype(np.int32)
    exp = oracle.epilog_int8(acc, scale[pts[:, 3]], bias[pts[:, 3]], True)
    xd, wd = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
    for variant in (0, 4, 4 | abed.ONLY_FC):
        g = GpuConv(s, variant, int8_out=True)
        g.prepare(wd)
        y, flags = g.run(xd, epilogue=(scale, bias, True))
        assert np.array_equal(y[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]], exp)
        assert variant == 0 or not flags.any()
        del g, y
        torch.cuda.empty_cache()
