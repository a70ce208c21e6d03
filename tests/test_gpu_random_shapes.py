"""GPU parity on seeded random convolution shapes: extents that are not multiples of any tile size,
1 to 5 wide filters, strides and paddings, every checked variant and scheme selection, int32 and
int8 output, against the oracle element by element (bit-exact) with the flags folded on the tile grid."""
import numpy as np
import pytest

import paper_2006_04984_amd as abed
from synth import ConvShape, int8_tensors, requant_params

pytestmark = pytest.mark.gpu


def random_case(seed):
    rng = np.random.default_rng(seed)
    while True:
        R, S = int(rng.choice([1, 2, 3, 5])), int(rng.choice([1, 2, 3, 5]))
        sh, sw = int(rng.integers(1, 3)), int(rng.integers(1, 3))
        ph, pw = int(rng.integers(0, min(R, 3))), int(rng.integers(0, min(S, 3)))
        H, W = int(rng.integers(1, 13)), int(rng.integers(1, 13))
        if H + 2 * ph < R or W + 2 * pw < S:
            continue
        N = int(rng.choice([1, 2, 3, 5, 8, 13, 24, 33, 40]))
        C = int(rng.choice([16, 32, 48, 64, 80, 128]))
        K = int(rng.choice([1, 7, 13, 16, 30, 32, 47, 48, 64, 77, 96, 130, 144]))
        s = ConvShape(N, H, W, C, K, R, S, sh, sw, ph, pw, "rnd%d" % seed)
        variant = int(rng.choice([0, 1, 2, 3, 4, 5, 6, 4 | abed.ONLY_FC, 4 | abed.ONLY_IC, 3 | abed.ONLY_FC, 5 | abed.ONLY_IC,
                                  1 | abed.ONLY_IC, 2 | abed.ONLY_FC]))
        if variant in (4, 5, 4 | abed.ONLY_FC) and K % 16 and K % 16 + 2 <= 16 and rng.integers(0, 2):
            variant |= abed.PACKED_FC
        return s, variant, bool(rng.integers(0, 2))


@pytest.mark.parametrize("seed", range(60))
def test_random_shape(oracle, seed):
    from gpu_helpers import GpuConv, flags_match
    s, variant, int8_out = random_case(seed)
    print("case", seed, s, hex(variant), "int8_out", int8_out, flush=True)
    x, w = int8_tensors(s, 9000 + seed)
    epi = None
    if int8_out:
        scale, bias = requant_params(s, 9000 + seed)
        epi = (scale, bias, bool(seed & 1))
    ref = oracle.abed_int8(x, w, s, epilog=epi)
    g = GpuConv(s, variant, int8_out=int8_out)
    g.prepare(w)
    y, flags = g.run(x, epilogue=epi)
    assert np.array_equal(y, ref["out8"] if int8_out else ref["y"])
    base = variant & 0xff
    if 1 <= base <= 5:
        assert flags_match(flags, ref, s, g.lay) and not flags.any()
        if base == 5 and int8_out and g.lay.d_i:
            assert np.array_equal(g.xchk_next.cpu().numpy(), ref["xchk_next"])
        idx, bit = (s.N * s.P * s.Q * s.K) // 2, seed % 32
        ref2 = oracle.abed_int8(x, w, s, acc_flip=(idx, bit), epilog=epi)
        y2, f2 = g.run(x, epilogue=epi, inject=(1, idx, bit))
        assert np.array_equal(y2, ref2["out8"] if int8_out else ref2["y"])
        assert flags_match(f2, ref2, s, g.lay) and f2.any()
