"""GPU parity for the one-wave-per-SIMD 3x3 convolution kernel (opt-in, ABED_IMG=1; unchecked, int32 ConvOut):
whole output tensors, bit for bit, against the oracle's 7-loop convolution (Sec. 2.2), on shapes that cover
both wave layouts (regions of up to 64 and up to 128 positions), ragged regions, paddings 0..2, several
chunks of channels, several filter tiles, several batches per workgroup and a batch tail."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2006_04984_amd as abed
from synth import CONFIG2, ConvShape, int8_tensors

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


def run_plain(s, x, w):
    desc = abed.desc_from_shape(s)
    xd, wd = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
    y = torch.full((s.N, s.P, s.Q, s.K), -3, dtype=torch.int32, device=DEV)
    abed.conv_int8(desc, xd, wd, None, None, False, y, 0)
    torch.cuda.synchronize()
    return y.cpu().numpy()


@pytest.mark.parametrize("s", SHAPES, ids=lambda s: s.name)
def test_img_kernel_matches_oracle(oracle, monkeypatch, s):
    print("case", s.name, flush=True)
    monkeypatch.setenv("ABED_IMG", "1")
    x, w = int8_tensors(s, 9100 + s.N)
    assert np.array_equal(run_plain(s, x, w), oracle.conv_int(x, w, s).astype(np.int32))


@pytest.mark.parametrize("i", range(4))
def test_img_kernel_config2_layers_whole_tensor(oracle, monkeypatch, i):
    """The configured 3x3 layers at their real size (32 images), every output element."""
    s = CONFIG2[i]
    print("case", s.name, flush=True)
    monkeypatch.setenv("ABED_IMG", "1")
    x, w = int8_tensors(s, 9200 + i)
    assert np.array_equal(run_plain(s, x, w), oracle.conv_int(x, w, s).astype(np.int32))
