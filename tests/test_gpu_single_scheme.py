"""GPU parity of the filter checksum scheme alone and of the batch checksum scheme alone (Sec. 3.1,
Sec. 3.2 option 1; the protection each gives is Table 1 of Sec. 3.4): outputs bit-exact, flags equal
to the oracle's mismatch map of that scheme folded on the tile grid, and the blind spots as the table
has them."""
import numpy as np
import pytest
import torch

import paper_2006_04984_amd as abed
from synth import ConvShape, CONFIG1, int8_tensors, fp16_tensors, requant_params

pytestmark = pytest.mark.gpu

SHAPES = [
    CONFIG1[0],
    ConvShape(32, 9, 9, 32, 64, 3, 3, 1, 1, 1, 1, "n32_c32_k64_9x9"),
    ConvShape(37, 7, 6, 16, 200, 3, 3, 2, 2, 1, 1, "n37_k200_stride2"),      # several batch and filter tiles, ragged
    ConvShape(9, 6, 6, 128, 144, 1, 1, 1, 1, 0, 0, "n9_1x1_c128"),
]
ONLY = {"fc": abed.ONLY_FC, "ic": abed.ONLY_IC}


@pytest.mark.parametrize("only", ["fc", "ic"])
@pytest.mark.parametrize("variant", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("s", SHAPES, ids=lambda s: s.name)
def test_clean_and_accumulator_flip(oracle, s, variant, only):
    from gpu_helpers import GpuConv, flags_match
    if variant == 5 and only == "fc":
        pytest.skip("the input-and-output-fused option hands on a batch checksum: not with FC alone")
    print("case", s.name, "variant", variant, only, flush=True)
    lo, hi = (-8, 7) if s.name.startswith("cfg1") else (-128, 127)
    x, w = int8_tensors(s, 6161, lo, hi)
    ref = oracle.abed_int8(x, w, s)
    g = GpuConv(s, variant | ONLY[only])
    assert (g.lay.d_f == 0) == (only == "ic") and (g.lay.d_i == 0) == (only == "fc")
    g.prepare(w)
    y, flags = g.run(x)
    assert np.array_equal(y, ref["y"]) and not flags.any()
    idx, bit = (s.N * s.P * s.Q * s.K) // 3, 21
    ref = oracle.abed_int8(x, w, s, acc_flip=(idx, bit))
    y, flags = g.run(x, inject=(1, idx, bit))
    assert np.array_equal(y, ref["y"])
    assert flags_match(flags, ref, s, g.lay)
    assert (flags & (1 if only == "fc" else 2)).any() and not (flags & ~np.uint32(1 if only == "fc" else 2)).any()


@pytest.mark.parametrize("only", ["fc", "ic"])
def test_epilog_output(oracle, only):
    from gpu_helpers import GpuConv, to_dev
    s = SHAPES[2]
    x, w = int8_tensors(s, 6262)
    scale, bias = requant_params(s, 6262)
    ref = oracle.abed_int8(x, w, s, epilog=(scale, bias, True))
    g = GpuConv(s, 4 | ONLY[only], int8_out=True)
    g.prepare(w)
    y, flags = g.run(x, epilogue=(scale, bias, True))
    assert np.array_equal(y, ref["out8"]) and not flags.any()


def test_next_layer_checksum_with_ic_alone(oracle):
    from gpu_helpers import GpuConv, to_dev
    s = SHAPES[1]
    x, w = int8_tensors(s, 6363)
    scale, bias = requant_params(s, 6363)
    ref = oracle.abed_int8(x, w, s, epilog=(scale, bias, True))
    g = GpuConv(s, 5 | abed.ONLY_IC, int8_out=True)
    g.prepare(w)
    y, flags = g.run(x, epilogue=(scale, bias, True))
    assert np.array_equal(y, ref["out8"]) and not flags.any()
    assert np.array_equal(g.xchk_next.cpu().numpy(), ref["xchk_next"])


def _flip_dev(t, flat_index, bit):
    t.view(torch.uint8).view(-1)[flat_index] ^= (1 << bit)


@pytest.mark.parametrize("only", ["fc", "ic"])
def test_blind_spots(oracle, only):
    """After the checksums were made: FC alone catches a filter flip and misses an input flip, IC alone
    the other way round (Table 1); the output is corrupted in every case."""
    from gpu_helpers import GpuConv, flags_match, to_dev
    s = SHAPES[1]
    x, w = int8_tensors(s, 6464, 1, 100)              # no zeros: every flip reaches an output
    clean = oracle.abed_int8(x, w, s)
    g = GpuConv(s, 4 | ONLY[only])
    g.prepare(w)
    y0, f0 = g.run(x)
    assert np.array_equal(y0, clean["y"]) and not f0.any()
    rng = np.random.default_rng(11)
    for site in ("x", "w"):
        t = g.x if site == "x" else g.w
        idx, bit = int(rng.integers(0, t.numel())), int(rng.integers(0, 8))
        print("only", only, "site", site, idx, bit, flush=True)
        _flip_dev(t, idx, bit)
        y, f = g.run(g.x, compute_xchk=False)
        arrs = dict(x=x.copy(), w=w.copy())
        oracle.flip_bit(arrs[site], idx, bit)
        ref = oracle.abed_int8(arrs["x"], arrs["w"], s, wchk=clean["wchk"], xchk=clean["xchk"])
        assert np.array_equal(y, ref["y"]) and (y != clean["y"]).any()
        assert flags_match(f, ref, s, g.lay)
        caught = (only == "fc") == (site == "w")
        assert f.any() == caught
        _flip_dev(t, idx, bit)


@pytest.mark.parametrize("only", ["fc", "ic"])
def test_fp16(oracle, only):
    from test_gpu_fp16 import GpuConv16
    s = ConvShape(6, 8, 8, 96, 80, 3, 3, 1, 1, 1, 1, "fp16_n6_c96_k80")
    x, w = fp16_tensors(s, 6565)
    ref = oracle.abed_fp16(x, w, s, rtol=1e-3, atol=1e-3)
    g = GpuConv16(s, 4 | ONLY[only])
    g.prepare(w)
    y, flags = g.run(x, rtol=1e-3, atol=1e-3)
    yr = ref["y"].astype(np.float64)
    assert np.all(np.abs(y.astype(np.float64) - yr) <= 1e-2 * np.abs(yr) + 1e-3)
    assert not flags.any()
    idx = y.size // 2
    y2, flags2 = g.run(x, rtol=1e-3, atol=1e-3, inject=(1, idx, 14))       # exponent bit: far beyond the threshold
    assert flags2.any() and not (flags2 & ~np.uint32(1 if only == "fc" else 2)).any()
