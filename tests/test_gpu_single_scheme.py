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


PACKED_SHAPES = [
    ConvShape(32, 9, 9, 32, 60, 3, 3, 1, 1, 1, 1, "k60"),                  # digits in rows 12, 13 of block 3
    ConvShape(37, 7, 6, 16, 205, 3, 3, 2, 2, 1, 1, "k205_stride2"),         # several filter tiles; digits in rows 13, 14
    ConvShape(9, 6, 6, 128, 13, 1, 1, 1, 1, 0, 0, "k13_1x1"),               # one block
    ConvShape(20, 5, 5, 64, 30, 3, 3, 1, 1, 1, 1, "k30"),                   # digits fill the block (rows 14, 15)
]


@pytest.mark.parametrize("scheme", ["fc", "both"])
@pytest.mark.parametrize("variant", [4, 5])
@pytest.mark.parametrize("s", PACKED_SHAPES, ids=lambda s: s.name)
def test_packed_checksum_filters(oracle, s, variant, scheme):
    """The checksum filters in the free rows of the last block of 16 filters (Sec. 6.2: reserved space
    for the filter checksums): outputs and flags are those of the plain layout."""
    from gpu_helpers import GpuConv, flags_match
    if variant == 5 and scheme == "fc":
        pytest.skip("no batch checksum to hand on with FC alone")
    print("case", s.name, "variant", variant, scheme, flush=True)
    x, w = int8_tensors(s, 6767)
    ref = oracle.abed_int8(x, w, s)
    v = variant | abed.PACKED_FC | (abed.ONLY_FC if scheme == "fc" else 0)
    g = GpuConv(s, v)
    g.prepare(w)
    assert g.wchk.data_ptr() == g.w.data_ptr() + s.K * s.R * s.S * s.C
    y, flags = g.run(x)
    assert np.array_equal(y, ref["y"]) and not flags.any()
    assert np.array_equal(g.wchk.cpu().numpy(), ref["wchk"])
    for idx, bit in ((y.size // 3, 21), (y.size - 1, 31), (s.K - 1, 0)):
        ref2 = oracle.abed_int8(x, w, s, acc_flip=(idx, bit))
        y2, f2 = g.run(x, inject=(1, idx, bit))
        assert np.array_equal(y2, ref2["y"]) and f2.any() and flags_match(f2, ref2, s, g.lay)
    if scheme == "both":
        # a corrupted checksum image disagrees with the checksum filters too: IC bit and corner bit,
        # the latter from the digit columns that now sit among the real filters' columns
        g.xchk.view(torch.uint8).view(-1)[5] ^= 0x04
        xc = ref["xchk"].copy(); oracle.flip_bit(xc, 5, 2)
        ref3 = oracle.abed_int8(x, w, s, xchk=xc)
        y3, f3 = g.run(x, compute_xchk=False)
        assert np.array_equal(y3, ref["y"]) and flags_match(f3, ref3, s, g.lay) and (f3 & 4).any()
    # a filter corrupted after its checksum was made
    g.w.view(torch.uint8).view(-1)[77] ^= 0x10
    w2 = w.copy(); oracle.flip_bit(w2, 77, 4)
    ref4 = oracle.abed_int8(x, w2, s, wchk=ref["wchk"])
    y4, f4 = g.run(x)
    assert np.array_equal(y4, ref4["y"]) and flags_match(f4, ref4, s, g.lay) and (f4 & 1).any()


def test_packed_needs_one_buffer():
    from gpu_helpers import GpuConv
    s = PACKED_SHAPES[0]
    g = GpuConv(s, 4 | abed.PACKED_FC)
    g.w = torch.zeros((s.K, s.R, s.S, s.C), dtype=torch.int8, device="cuda:0")     # wchk elsewhere
    with pytest.raises(abed.AbedError) as e:
        g.run(torch.zeros((s.N, s.H, s.W, s.C), dtype=torch.int8, device="cuda:0"))
    assert e.value.status == 1


@pytest.mark.parametrize("variant", [1, 2, 3, 4])
def test_nine_wide_tiles_for_the_filter_checksum_alone(oracle, variant):
    """256 filters + the block of checksum filters = 17 filter blocks: with a long reduction axis and a grid of
    200 tiles or more the plan takes tiles 9 blocks wide (two filter tiles instead of five)."""
    from gpu_helpers import GpuConv, flags_match
    s = ConvShape(64, 14, 14, 128, 256, 3, 3, 1, 1, 1, 1, "n64_c128_k256_14x14")
    x, w = int8_tensors(s, 6464)
    ref = oracle.abed_int8(x, w, s)
    g = GpuConv(s, variant | abed.ONLY_FC)
    assert (g.lay.tile_batch, g.lay.tile_n, g.lay.grid_n) == (8, 144, 2)
    g.prepare(w)
    y, flags = g.run(x)
    assert np.array_equal(y, ref["y"]) and not flags.any()
    idx, bit = (s.N * s.P * s.Q * s.K) // 3 + 200, 30
    ref = oracle.abed_int8(x, w, s, acc_flip=(idx, bit))
    y, flags = g.run(x, inject=(1, idx, bit))
    assert np.array_equal(y, ref["y"]) and flags_match(flags, ref, s, g.lay) and flags.any()
    # the same shape with both schemes keeps its 4-wide tiles
    assert abed.get_layout(g.desc, 0, variant).tile_n in (64, 80)
