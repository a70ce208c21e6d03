"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by
element, bit-exact (integer work), on seeded inputs that span several tiles and
ragged tails.  Flags are compared after folding the oracle's maps on the tile layout."""
import numpy as np
import pytest

from synth import ConvShape, CONFIG1, int8_tensors, requant_params

pytestmark = pytest.mark.gpu

VARIANTS = [0, 1, 2, 3, 4, 5, 6]

SHAPES = [
    CONFIG1[0],
    ConvShape(32, 9, 9, 32, 64, 3, 3, 1, 1, 1, 1, "n32_c32_k64_9x9"),          # ragged pixel tail (81 = 10*8+1)
    ConvShape(5, 7, 6, 16, 48, 3, 3, 2, 2, 1, 1, "n5_k48_stride2"),            # padded batch, ragged filters
    ConvShape(16, 6, 5, 64, 128, 1, 1, 1, 1, 0, 0, "n16_1x1_k128"),
    ConvShape(64, 5, 5, 16, 320, 3, 3, 1, 1, 1, 1, "n64_k320_split"),          # filters span two tile columns
    ConvShape(128, 3, 4, 32, 64, 1, 1, 1, 1, 0, 0, "n128_1x1"),
    ConvShape(3, 10, 8, 16, 16, 3, 2, 1, 2, 1, 0, "n3_asym"),
    ConvShape(48, 4, 4, 80, 96, 3, 3, 1, 1, 1, 1, "n48_c80_k96"),              # C not a multiple of 64
    ConvShape(2, 12, 12, 16, 64, 7, 7, 2, 2, 3, 3, "7x7_s2"),
]


def lo_hi(s):
    return (-8, 7) if s.name.startswith("cfg1") else (-128, 127)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("s", SHAPES, ids=lambda s: s.name)
def test_clean_run_matches_oracle(oracle, s, variant):
    from gpu_helpers import GpuConv, fold_flags, flags_match
    print("case", s.name, "variant", variant, flush=True)
    x, w = int8_tensors(s, 4242, *lo_hi(s))
    ref = oracle.abed_int8(x, w, s)
    g = GpuConv(s, variant)
    g.prepare(w)
    y, flags = g.run(x)
    assert np.array_equal(y, ref["y"])
    if 1 <= variant <= 5:
        assert np.array_equal(g.wchk.cpu().numpy(), ref["wchk"])
        assert np.array_equal(g.xchk.cpu().numpy(), ref["xchk"])
        assert flags_match(flags, ref, s, g.lay) and not flags.any()
    if variant == 6:
        assert np.array_equal(g.y2.cpu().numpy(), ref["y"]) and flags[0] == 0


@pytest.mark.parametrize("variant", [0, 1, 2, 3, 4, 5, 6])
@pytest.mark.parametrize("s", [SHAPES[1], SHAPES[2], SHAPES[4]], ids=lambda s: s.name)
def test_epilog_matches_oracle(oracle, s, variant):
    from gpu_helpers import GpuConv, fold_flags, flags_match
    print("case", s.name, "variant", variant, flush=True)
    x, w = int8_tensors(s, 4343)
    scale, bias = requant_params(s, 4343)
    ref = oracle.abed_int8(x, w, s, epilog=(scale, bias, True))
    g = GpuConv(s, variant, int8_out=True)
    g.prepare(w)
    y, flags = g.run(x, epilogue=(scale, bias, True))
    assert np.array_equal(y, ref["out8"])
    if 1 <= variant <= 5:
        assert not flags.any()


@pytest.mark.parametrize("variant", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("s", [SHAPES[0], SHAPES[1], SHAPES[4]], ids=lambda s: s.name)
def test_accumulator_flip_is_flagged_in_the_right_tile(oracle, s, variant):
    from gpu_helpers import GpuConv, fold_flags, flags_match
    x, w = int8_tensors(s, 4444, *lo_hi(s))
    rng = np.random.default_rng(99)
    g = GpuConv(s, variant)
    g.prepare(w)
    for trial in range(4):
        idx = int(rng.integers(0, s.N * s.P * s.Q * s.K))
        bit = int(rng.integers(0, 32))
        print("case", s.name, "variant", variant, "flip", idx, bit, flush=True)
        ref = oracle.abed_int8(x, w, s, acc_flip=(idx, bit))
        y, flags = g.run(x, inject=(1, idx, bit))
        assert np.array_equal(y, ref["y"])
        exp, _ = fold_flags(ref, s, g.lay)
        assert exp.any()
        assert flags_match(flags, ref, s, g.lay)
