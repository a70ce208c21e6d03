"""GPU parity with the reduction axis split over 2 and 4 wave groups per workgroup
(the tile plan's ABED_TILE_KG override), on shapes whose step counts are not
multiples of the group count, for int8 (bit-exact) and fp16 (tolerance)."""
import os

import numpy as np
import pytest

from synth import ConvShape, CONFIG1, int8_tensors, fp16_tensors, requant_params

pytestmark = pytest.mark.gpu

SHAPES = [
    CONFIG1[0],                                                                 # 144 bytes: 3 steps
    ConvShape(32, 9, 9, 64, 64, 3, 3, 1, 1, 1, 1, "n32_c64_k64_9x9"),           # 9 steps, fast loader path
    ConvShape(5, 7, 6, 16, 48, 3, 3, 2, 2, 1, 1, "n5_k48_stride2"),             # per-lane tap tracking
    ConvShape(12, 5, 5, 320, 80, 3, 3, 1, 1, 1, 1, "n12_c320_k80"),             # 45 steps
    ConvShape(9, 6, 6, 128, 144, 1, 1, 1, 1, 0, 0, "n9_1x1_c128"),              # 2 steps, fewer than the groups
]


@pytest.fixture(params=[2, 4], ids=lambda k: "kg%d" % k)
def wave_groups(request):
    os.environ["ABED_TILE_KG"] = str(request.param)
    yield request.param
    os.environ.pop("ABED_TILE_KG", None)
    os.environ.pop("ABED_TILE_WM", None)
    os.environ.pop("ABED_TILE_WK", None)


@pytest.mark.parametrize("variant", [0, 3, 4, 5])
@pytest.mark.parametrize("s", SHAPES, ids=lambda s: s.name)
def test_int8_clean_and_flip(oracle, wave_groups, s, variant):
    from gpu_helpers import GpuConv, fold_flags, flags_match
    if wave_groups == 4:
        os.environ["ABED_TILE_WM"], os.environ["ABED_TILE_WK"] = "2", "4"      # a shape compiled for 4 groups
    print("case", s.name, "variant", variant, "groups", wave_groups, flush=True)
    lo, hi = (-8, 7) if s.name.startswith("cfg1") else (-128, 127)
    x, w = int8_tensors(s, 5151, lo, hi)
    ref = oracle.abed_int8(x, w, s)
    g = GpuConv(s, variant)
    g.prepare(w)
    y, flags = g.run(x)
    assert np.array_equal(y, ref["y"])
    if variant:
        assert flags_match(flags, ref, s, g.lay) and not flags.any()
        idx, bit = (s.N * s.P * s.Q * s.K) // 3, 17
        ref = oracle.abed_int8(x, w, s, acc_flip=(idx, bit))
        y, flags = g.run(x, inject=(1, idx, bit))
        assert np.array_equal(y, ref["y"])
        assert flags.any() and flags_match(flags, ref, s, g.lay)


@pytest.mark.parametrize("s", [SHAPES[1], SHAPES[3]], ids=lambda s: s.name)
def test_int8_epilog_next_checksum(oracle, wave_groups, s):
    from gpu_helpers import GpuConv
    print("case", s.name, "groups", wave_groups, flush=True)
    x, w = int8_tensors(s, 5252)
    scale, bias = requant_params(s, 5252)
    ref = oracle.abed_int8(x, w, s, epilog=(scale, bias, True))
    g = GpuConv(s, 5, int8_out=True)
    g.prepare(w)
    y, flags = g.run(x, epilogue=(scale, bias, True))
    assert np.array_equal(y, ref["out8"]) and not flags.any()
    assert np.array_equal(g.xchk_next.cpu().numpy(), ref["xchk_next"])


@pytest.mark.parametrize("variant", [0, 4])
def test_fp16(oracle, wave_groups, variant):
    from test_gpu_fp16 import GpuConv16
    s = ConvShape(6, 8, 8, 96, 80, 3, 3, 1, 1, 1, 1, "fp16_n6_c96_k80")          # 27 steps of 32 halves
    print("case", s.name, "variant", variant, "groups", wave_groups, flush=True)
    x, w = fp16_tensors(s, 5353)
    ref = oracle.abed_fp16(x, w, s, rtol=1e-3, atol=1e-3)
    g = GpuConv16(s, variant)
    g.prepare(w)
    y, flags = g.run(x, rtol=1e-3, atol=1e-3)
    yr = ref["y"].astype(np.float64)
    assert np.all(np.abs(y.astype(np.float64) - yr) <= 1e-2 * np.abs(yr) + 1e-3)
    if variant:
        assert not flags.any()


@pytest.mark.parametrize("s", [SHAPES[1], SHAPES[2], SHAPES[3]], ids=lambda s: s.name)
def test_fic_fused(oracle, wave_groups, s):
    """The FIC scheme's fused option hosts its input checksum workgroups in the convolution's launch:
    with 2 or 4 wave groups those workgroups are 512 or 1024 threads wide and only 256 of them work."""
    from test_gpu_fic import GpuFic
    if wave_groups == 4:
        os.environ["ABED_TILE_WM"], os.environ["ABED_TILE_WK"] = "2", "4"
    print("case", s.name, "groups", wave_groups, flush=True)
    x, w = int8_tensors(s, 5454)
    ref = oracle.abed_fic_int8(x, w, s)
    g = GpuFic(s, 4)
    g.prepare(w)
    y, ocs, dot, flag = g.run(x)
    assert np.array_equal(y, ref["y"]) and (ocs, dot, flag) == (ref["ocs"], ref["dot"], 0)
    idx, bit = y.size // 5, 30
    ref2 = oracle.abed_fic_int8(x, w, s, acc_flip=(idx, bit))
    y2, ocs2, dot2, flag2 = g.run(x, inject=(1, idx, bit))
    assert np.array_equal(y2, ref2["y"]) and (ocs2, dot2, flag2) == (ref2["ocs"], ref2["dot"], 1)
