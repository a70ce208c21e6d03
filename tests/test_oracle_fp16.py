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
    # an infinity or a NaN on either side is a mismatch, whatever the tolerance works out to
    assert list(bad[5:]) == [True, True]
    assert list(oracle.threshold_bad(np.array([1.0, 1.0, np.inf]), np.array([np.inf, np.nan, np.inf]), 1e-3, 1e-3)) == [True] * 3
    assert list(oracle.threshold_bad(np.array([np.nan]), np.array([1.0]), 0.0, np.inf)) == [True]


def test_l1_threshold_hand_cases(oracle):
    """Threshold relative to the L1 norm of the reduced elements: tol = rtol * sum|y| + atol."""
    # two elements that cancel: s = 1e-4 against a checksum of 0.  Relative to the values the tolerance is
    # 1e-3 * 1e-4 and the check fails; relative to sum|y| = 1.9999 it is 2e-3 and the check passes
    y = np.array([1.0, -0.9999])
    assert oracle.threshold_bad(y.sum(), 0.0, 1e-3, 0.0)
    assert not oracle.threshold_bad(y.sum(), 0.0, 1e-3, 0.0, mag=np.abs(y).sum())
    # no cancellation: both readings agree (2 against 2.01: tolerance 2.01e-3 and 2e-3)
    y = np.array([1.0, 1.0])
    assert oracle.threshold_bad(y.sum(), 2.01, 1e-3, 0.0) and oracle.threshold_bad(y.sum(), 2.01, 1e-3, 0.0, mag=2.0)
    assert not oracle.threshold_bad(y.sum(), 2.001, 1e-3, 0.0, mag=2.0)
    # the boundary itself passes (<=), one ulp beyond fails; atol adds
    assert not oracle.threshold_bad(0.5, 0.0, 0.25, 0.0, mag=2.0)
    assert oracle.threshold_bad(np.nextafter(0.5, 1.0), 0.0, 0.25, 0.0, mag=2.0)
    assert not oracle.threshold_bad(0.75, 0.0, 0.25, 0.25, mag=2.0)
    # margins have the sign of the decision
    assert oracle.threshold_margin(0.75, 0.0, 0.25, 0.0, mag=2.0) == 0.25
    assert oracle.threshold_margin(3.0, 1.0, 0.5, 0.0) == 0.5
    # non-finite sums or norms are mismatches
    assert oracle.threshold_bad(np.inf, 1.0, 1e-3, 0.0, mag=np.inf) and oracle.threshold_bad(1.0, 1.0, 1e-3, 0.0, mag=np.nan)


@pytest.mark.parametrize("s", SHAPES, ids=lambda s: s.name)
def test_l1_threshold_on_convolutions(oracle, s):
    x, w = fp16_tensors(s, 24)
    r = oracle.abed_fp16(x, w, s, rtol=1e-5, atol=0.0, l1=True)
    # the norms are what they say: recomputed from the library convolution
    y = torch_conv_f64(x, w, s)
    np.testing.assert_allclose(r["rs_abs"], np.abs(y).sum(3), rtol=1e-12)
    np.testing.assert_allclose(r["cs_abs"], np.abs(y).sum(0), rtol=1e-12)
    assert np.all(r["rs_abs"] >= np.abs(r["rs"])) and np.all(r["cs_abs"] >= np.abs(r["cs"]))
    # clean data: the only error is the hi/lo rounding of the checksums (2^-22 relative), far below 1e-5 of the norm
    assert not (r["fc_bad"].any() or r["ic_bad"].any() or r["corner_bad"].any())
    # same data, same tolerance relative to the values: never fewer mismatches on clean data (sum|y| >= |sum y|, and
    # the checksum side equals the sum to rounding)
    lit = oracle.abed_fp16(x, w, s, rtol=1e-5, atol=0.0)
    assert np.all(lit["fc_margin"] >= r["fc_margin"] - 1e-9) and np.all(lit["ic_margin"] >= r["ic_margin"] - 1e-9)
    # an exponent-bit flip is found and localised under both readings; the lowest mantissa bit under neither at 1e-3
    idx = ((1 * s.P + 1) * s.Q + 2) * s.K + 3
    for l1 in (False, True):
        f = oracle.abed_fp16(x, w, s, 1e-3, 1e-3, acc_flip=(idx, 14), l1=l1)
        assert f["fc_bad"][1, 1, 2] and f["fc_bad"].sum() == 1 and f["ic_bad"][1, 2, 3] and f["ic_bad"].sum() == 1
        f = oracle.abed_fp16(x, w, s, 1e-3, 1e-3, acc_flip=(idx, 0), l1=l1)
        assert not (f["fc_bad"].any() or f["ic_bad"].any())


@pytest.mark.parametrize("l1", [False, True])
def test_corner_mismatch(oracle, l1):
    """A corrupted checksum tensor shows in the corner (Sec. 2.1: the checksum row and column are checked against
    each other): the checksum image enters yi and yfi, so the IC comparison fails where the element is used while
    sum_k yi still agrees with yfi; but sum_n yf, made from the real images, no longer agrees with yfi."""
    s = SHAPES[2]
    x, w = fp16_tensors(s, 25)
    clean = oracle.abed_fp16(x, w, s, 1e-3, 1e-3, l1=l1)
    assert not clean["corner_bad"].any()
    xchk = clean["xchk"].copy()
    h0, w0, c0 = 2, 3, 5
    oracle.flip_bit(xchk[0], (h0 * s.W + w0) * s.C + c0, 14)           # a high exponent bit of the hi part
    r = oracle.abed_fp16(x, w, s, 1e-3, 1e-3, xchk=xchk, l1=l1)
    # output positions whose 3x3 window (pad 1, stride 1) covers (h0, w0)
    cover = np.zeros((s.P, s.Q), dtype=bool)
    cover[max(h0 - 1, 0):h0 + 2, max(w0 - 1, 0):w0 + 2] = True
    assert np.array_equal(r["corner_bad"], cover)
    assert not r["fc_bad"].any()                                       # the real rows and their filter checksum are intact
    assert np.array_equal(r["ic_bad"].any(axis=2), cover)              # the column check sees the bad checksum image
    # the same for a corrupted checksum filter: every position uses every filter element (up to padding)
    wchk = clean["wchk"].copy()
    oracle.flip_bit(wchk[0], (1 * s.S + 1) * s.C + 2, 14)              # centre tap: used at every output position
    r = oracle.abed_fp16(x, w, s, 1e-3, 1e-3, wchk=wchk, l1=l1)
    assert r["corner_bad"].all() and r["fc_bad"].all() and not r["ic_bad"].any()


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


def test_next_layer_checksum_chains(oracle):
    """The batch checksum handed to the next layer (Sec. 4.3) is the checksum that layer would make from its own
    input: chaining two layers, layer 2's default input checksum equals layer 1's xchk_next bit for bit, and a
    clean second layer raises no flag with it."""
    s1 = ConvShape(5, 6, 6, 8, 16, 3, 3, 1, 1, 1, 1, "l1")
    s2 = ConvShape(5, 6, 6, 16, 8, 1, 1, 1, 1, 0, 0, "l2")
    x, w1 = fp16_tensors(s1, 31)
    _, w2 = fp16_tensors(s2, 32)
    r1 = oracle.abed_fp16(x, w1, s1, 1e-3, 1e-3)
    nxt = r1["xchk_next"]
    assert nxt.dtype == np.float16 and nxt.shape == (2, s1.P, s1.Q, s1.K)
    total = r1["y"].astype(np.float64).sum(axis=0)
    assert np.all(np.abs(nxt.astype(np.float64).sum(0) - total) <= np.abs(total) * 2.0 ** -21 + 2.0 ** -25)
    r2_own = oracle.abed_fp16(r1["y"], w2, s2, 1e-3, 1e-3)
    assert np.array_equal(r2_own["xchk"].view(np.uint16), nxt.view(np.uint16))
    r2 = oracle.abed_fp16(r1["y"], w2, s2, 1e-3, 1e-3, xchk=nxt)
    assert not (r2["fc_bad"].any() or r2["ic_bad"].any() or r2["corner_bad"].any())
    # an output of layer 1 corrupted after its checksum was handed on shows in layer 2's batch check
    ybad = r1["y"].copy()
    oracle.flip_bit(ybad, ((2 * s1.P + 3) * s1.Q + 1) * s1.K + 4, 13)
    r2b = oracle.abed_fp16(ybad, w2, s2, 1e-3, 1e-3, xchk=nxt)
    assert r2b["ic_bad"][3, 1].any() and not np.delete(r2b["ic_bad"].reshape(36, -1), 3 * 6 + 1, axis=0).any()
