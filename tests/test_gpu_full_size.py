"""GPU parity at the full sizes of the configured workloads, in the launch configuration the benchmark
and the evaluation runs time (automatic tile plan): the whole output tensor of every configured 3x3 and
1x1 layer against the oracle's, clean flags, and one accumulator flip whose flag words must equal the
oracle's mismatch maps folded onto the tile grid (FC bit on the flipped element's batch tile, IC bit on
its filter tile, nothing else).  The 53-layer network's picks are compared on sampled elements."""
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


ALL_VARIANTS = [(0, 0), (1, 3), (2, 3), (3, 3), (4, 3), (5, 3), (6, 0), (4 | abed.ONLY_FC, 1), (4 | abed.ONLY_IC, 2)]
ALL_IDS = ["unchecked", "unfused", "fused_write", "partial", "fused_ocg", "fused_iocg", "duplicate", "fc_only", "ic_only"]
_ref_cache = {}


def full_reference(oracle, cfg, li, s, x, w, flip=None):
    """The oracle's whole result for a configured layer (ConvOut and the element-level mismatch maps);
    the clean one is kept for the other variants of the same layer."""
    key = (cfg, li, flip)
    if key not in _ref_cache:
        if flip is None:
            for k in [k for k in _ref_cache if k[:2] != (cfg, li)]:
                del _ref_cache[k]
        _ref_cache[key] = oracle.abed_int8(x, w, s, acc_flip=flip)
    return _ref_cache[key]


@pytest.mark.parametrize("variant,scheme", ALL_VARIANTS, ids=ALL_IDS)
@pytest.mark.parametrize("li", range(4))
def test_config2_layers(oracle, li, variant, scheme):
    """Every variant on every configured 3x3 layer at full size: the WHOLE output tensor against the
    oracle's, all flag words clear, then one accumulator flip whose flag words must be the oracle's
    mismatch maps folded onto the tile grid."""
    from gpu_helpers import GpuConv, flags_match
    s = CONFIG2[li]
    print("case", s.name, hex(variant), flush=True)
    x, w = int8_tensors(s, seed_for(2, li))
    ref = full_reference(oracle, 2, li, s, x, w)
    g = GpuConv(s, variant)
    g.prepare(w)
    y, flags = g.run(x)
    assert np.array_equal(y, ref["y"])
    if variant == 6:
        assert flags[0] == 0 and np.array_equal(g.y2.cpu().numpy(), ref["y"])
    if scheme:
        assert not flags.any()
        pt = sample_points(s, 8, 17 + li)[7]
        idx = int(np.ravel_multi_index(tuple(pt), (s.N, s.P, s.Q, s.K)))
        bad = full_reference(oracle, 2, li, s, x, w, flip=(idx, 29))
        y2, f2 = g.run(x, inject=(1, idx, 29))
        assert np.array_equal(y2, bad["y"])
        assert flags_match(f2, bad, s, g.lay)
        assert np.array_equal(f2.reshape(g.lay.grid_m, g.lay.grid_b, g.lay.grid_n) & 3, expected_flags(g.lay, s, idx, scheme))


@pytest.mark.parametrize("int8_out", [False, True], ids=["i32out", "i8out"])
@pytest.mark.parametrize("li", range(5))
def test_config3_layers(oracle, li, int8_out):
    """The 1x1 layers at full size, unchecked and FusedOCG: the whole output tensor (raw ConvOut, or
    after the epilog) against the oracle's."""
    from gpu_helpers import GpuConv
    s = CONFIG3[li]
    print("case", s.name, int8_out, flush=True)
    x, w = int8_tensors(s, seed_for(3, li))
    scale, bias = requant_params(s, seed_for(3, li))
    acc = oracle.conv_int(x, w, s).astype(np.int32)
    exp = oracle.epilog_int8(acc, scale, bias, True) if int8_out else acc
    for variant in (0, 4):
        g = GpuConv(s, variant, int8_out=int8_out)
        g.prepare(w)
        y, flags = g.run(x, epilogue=(scale, bias, True) if int8_out else None)
        assert np.array_equal(y, exp)
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


def _distinct_resnet_layers():
    seen, out = set(), []
    for i, s in enumerate(resnet50_layers(128)):
        key = (s.H, s.W, s.C, s.K, s.R, s.S, s.stride_h, s.stride_w, s.pad_h, s.pad_w)
        if key not in seen:
            seen.add(key)
            out.append(i)
    return out


@pytest.mark.parametrize("i", _distinct_resnet_layers())
def test_resnet50_every_distinct_layer_whole_tensor(oracle, i):
    """Every distinct layer shape of the 53-layer network at its evaluation batch of 128 (the other layers repeat
    these shapes), FusedOCG with the fused int8 epilog: the WHOLE output tensor against the oracle's convolution and
    epilog, flags clear.  The 3-channel first layer goes through the library's channel padding."""
    from gpu_helpers import GpuConv
    s = resnet50_layers(128)[i]
    print("case", i, s.name, flush=True)
    x, w = int8_tensors(s, 5000 + i)
    scale, bias = requant_params(s, 5000 + i)
    exp = oracle.epilog_int8(oracle.conv_int(x, w, s).astype(np.int32), scale, bias, True)
    xd, wd = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
    sg = s
    if s.C % 16:
        sg = dataclasses.replace(s, C=16)
        xp = torch.empty((s.N, s.H, s.W, 16), dtype=torch.int8, device=DEV)
        wp = torch.empty((s.K, s.R, s.S, 16), dtype=torch.int8, device=DEV)
        abed.pad_channels(xd, xp, s.C, 16)
        abed.pad_channels(wd, wp, s.C, 16)
        xd, wd = xp, wp
    g = GpuConv(sg, 4, int8_out=True)
    g.prepare(wd)
    y, flags = g.run(xd, epilogue=(scale, bias, True))
    assert np.array_equal(y, exp)
    assert not flags.any()
    del g, y
    torch.cuda.empty_cache()
