"""Pins for the fp16 oracle (Sec. 7 of the paper): library witness for the
double-precision convolution, exactness of the hi/lo checksum split, the
linearity identities to rounding level, and the threshold rule on hand cases."""
import numpy as np
import pytest
import torch

from synth import ConvShape, fp16_tensors

SHAPES = [ConvShape(3, 6, 5, 8, 5, 3, 2, 1, 1, 1, 0, "asym_a"),
          ConvShape(2, 7, 9, 8, 4, 2, 3, 2, 1, 0, 2, "asym_b"),
          ConvShape(4, 6, 6, 16, 8, 3, 3, 1, 1, 1, 1, "3x3")]


def torch_conv_f64(x, w, s):
    xt = torch.from_numpy(np.asarray(x, dtype=np.float64)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(np.asarray(w, dtype=np.float64)).permute(0, 3, 1, 2)
    y = torch.nn.functional.conv2d(xt, wt, stride=(s.stride_h, s.stride_w), padding=(s.pad_h, s.pad_w))
    return y.permute(0, 2, 3, 1).contiguous().numpy()


@pytest.mark.parametrize("s", SHAPES, ids=lambda s: s.name)
def test_conv_f64_vs_torch(oracle, s):
    x, w = fp16_tensors(s, 21)
    np.testing.assert_allclose(oracle.conv_f64(x, w, s), torch_conv_f64(x, w, s), rtol=1e-12, atol=1e-12)


def test_conv_f64_small_integers_exact(oracle):
    """Small integers are exact in fp16 and in double: the double path must equal integer arithmetic."""
    s = SHAPES[0]
    g = np.random.default_rng(1)
    x = g.integers(-8, 8, (s.N, s.H, s.W, s.C)).astype(np.float16)
    w = g.integers(-8, 8, (s.K, s.R, s.S, s.C)).astype(np.float16)
    assert np.array_equal(oracle.conv_f64(x, w, s), oracle.conv_int(x.astype(np.int32), w.astype(np.int32), s).astype(np.float64))


def test_hi_lo_split(oracle):
    g = np.random.default_rng(2)
    s = g.standard_normal(10000) * 16.0
    hl = oracle.split_hi_lo(s)
    assert hl.dtype == np.float16 and hl.shape == (2, 10000)
    err = np.abs(hl[0].astype(np.float64) + hl[1].astype(np.float64) - s)
    # one fp16 keeps 11 bits; the pair keeps about 22 (less when lo is subnormal)
    assert np.all(err <= np.abs(s) * 2.0 ** -21 + 2.0 ** -25)
    assert np.all(np.abs(hl[0].astype(np.float64) - s) <= np.abs(s) * 2.0 ** -11 + 2.0 ** -25)


@pytest.mark.parametrize("s", SHAPES, ids=lambda s: s.name)
def test_clean_run_identities(oracle, s):
    x, w = fp16_tensors(s, 22)
    r = oracle.abed_fp16(x, w, s, rtol=1e-3, atol=1e-3)
    # the identities of Sec. 3 hold to the precision of the hi/lo checksums
    np.testing.assert_allclose(r["rs"], r["yf"], rtol=0, atol=1e-4)
    np.testing.assert_allclose(r["cs"], r["yi"], rtol=0, atol=1e-4)
    np.testing.assert_allclose(r["yf"].sum(0), r["yfi"], rtol=0, atol=1e-4)
    assert not (r["fc_bad"].any() or r["ic_bad"].any() or r["corner_bad"].any())
    # library witness for the extra fmaps
    wsum = np.asarray(w, dtype=np.float64).sum(0, keepdims=True)
    np.testing.assert_allclose(r["yf"], torch_conv_f64(x, wsum, s)[..., 0], rtol=0, atol=1e-4)


def test_threshold_rule_hand_cases(oracle):
    # |s-c| > rtol*max(|s|,|c|) + atol
    s = np.array([100.0, 100.0, 0.0, 0.0, -50.0, np.inf, np.nan])
    c = np.array([100.05, 100.2, 0.0005, 0.002, 50.0, 1.0, 1.0])
    bad = oracle.threshold_bad(s, c, 1e-3, 1e-3)
    assert list(bad[:5]) == [False, True, False, True, True]


def test_output_flip_detection(oracle):
    """A flip of a high exponent bit of one output moves one row sum and one column sum far
    beyond the threshold; a flip of the lowest mantissa bit stays below it (Sec. 7: errors are
    detected when they move the value by more than the threshold)."""
    s = SHAPES[2]
    x, w = fp16_tensors(s, 23)
    idx = ((1 * s.P + 2) * s.Q + 3) * s.K + 4
    r = oracle.abed_fp16(x, w, s, 1e-3, 1e-3, acc_flip=(idx, 14))
    assert r["fc_bad"][1, 2, 3] and r["fc_bad"].sum() == 1
    assert r["ic_bad"][2, 3, 4] and r["ic_bad"].sum() == 1
    r = oracle.abed_fp16(x, w, s, 1e-3, 1e-3, acc_flip=(idx, 0))
    assert not r["fc_bad"].any() and not r["ic_bad"].any()
