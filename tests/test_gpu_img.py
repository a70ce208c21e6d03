"""GPU parity for the one-wave-per-SIMD 3x3 convolution kernel (opt-in, ABED_IMG=1; unchecked; int32 ConvOut, or int8
after the epilog of Sec. 4.3): whole output tensors, bit for bit, against the oracle's 7-loop convolution (Sec. 2.2)
and its requantised outputs, on shapes that cover
both wave layouts (regions of up to 64 and up to 128 positions), ragged regions, paddings 0..2, several
chunks of channels, several filter tiles, several batches per workgroup and a batch tail."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2006_04984_amd as abed
from synth import CONFIG2, ConvShape, int8_tensors, requant_params

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

SHAPES = [ConvShape(8, 8, 8, 64, 64, 3, 3, 1, 1, 1, 1, "n8_8x8"),
          ConvShape(5, 16, 16, 128, 64, 3, 3, 1, 1, 1, 1, "n5_16x16_two_chunks"),
          ConvShape(9, 7, 7, 128, 128, 3, 3, 1, 1, 1, 1, "n9_7x7_two_tiles"),
          ConvShape(6, 14, 14, 64, 128, 3, 3, 1, 1, 1, 1, "n6_14x14"),
          ConvShape(3, 28, 28, 64, 64, 3, 3, 1, 1, 1, 1, "n3_28x28"),
          ConvShape(37, 12, 12, 192, 64, 3, 3, 1, 1, 1, 1, "n37_three_chunks_many_batches"),
          ConvShape(11, 11, 13, 64, 64, 3, 3, 1, 1, 1, 1, "n11_11x13_ragged"),
          ConvShape(5, 12, 7, 256, 64, 3, 3, 1, 1, 0, 2, "n5_c256_pad0x2"),
          ConvShape(3, 17, 9, 64, 128, 3, 3, 1, 1, 2, 0, "n3_pad2x0"),
          ConvShape(1, 9, 9, 64, 192, 3, 3, 1, 1, 1, 1, "n1_three_tiles")]


def run_plain(s, x, w, epilogue=None):
    desc = abed.desc_from_shape(s)
    xd, wd = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
    y = torch.full((s.N, s.P, s.Q, s.K), -3, dtype=torch.int8 if epilogue else torch.int32, device=DEV)
    epi = None
    if epilogue:
        sc, bi = torch.from_numpy(epilogue[0]).to(DEV), torch.from_numpy(epilogue[1]).to(DEV)
        epi = (sc, bi, epilogue[2])
    abed.conv_int8(desc, xd, wd, None, None, False, y, 0, epilogue=epi)
    torch.cuda.synchronize()
    return y.cpu().numpy()


@pytest.mark.parametrize("s", SHAPES, ids=lambda s: s.name)
def test_img_kernel_matches_oracle(oracle, monkeypatch, s):
    print("case", s.name, flush=True)
    monkeypatch.setenv("ABED_IMG", "1")
    x, w = int8_tensors(s, 9100 + s.N)
    ref = oracle.conv_int(x, w, s)
    assert np.array_equal(run_plain(s, x, w), ref.astype(np.int32))
    sc, bi = requant_params(s, 9100 + s.N)
    for relu in (True, False):
        assert np.array_equal(run_plain(s, x, w, epilogue=(sc, bi, relu)), oracle.epilog_int8(ref, sc, bi, relu))


@pytest.mark.parametrize("i", range(4))
def test_img_kernel_config2_layers_whole_tensor(oracle, monkeypatch, i):
    """The configured 3x3 layers at their real size (32 images), every output element."""
    s = CONFIG2[i]
    print("case", s.name, flush=True)
    monkeypatch.setenv("ABED_IMG", "1")
    x, w = int8_tensors(s, 9200 + i)
    ref = oracle.conv_int(x, w, s)
    assert np.array_equal(run_plain(s, x, w), ref.astype(np.int32))
    sc, bi = requant_params(s, 9200 + i)
    assert np.array_equal(run_plain(s, x, w, epilogue=(sc, bi, True)), oracle.epilog_int8(ref, sc, bi, True))
