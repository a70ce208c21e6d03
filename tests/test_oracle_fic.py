"""Pins of the FIC part of the oracle (Sec. 3.3): the input patch checksum, the dot
product with the filter checksum and the scalar comparison, against values that
do not come from the oracle's own formula: a hand-worked all-ones case, a
bounds-checked brute force, the independent 7-loop convolution, and the algebra
of single faults."""
import os

import numpy as np
import pytest

from synth import ConvShape, CONFIG1, int8_tensors

HERE = os.path.dirname(os.path.abspath(__file__))

SHAPES = [
    ConvShape(2, 5, 4, 3, 4, 3, 3, 1, 1, 1, 1, "3x3_p1"),
    ConvShape(3, 7, 6, 2, 5, 3, 2, 2, 1, 1, 0, "3x2_s2x1"),
    ConvShape(2, 9, 8, 4, 3, 7, 7, 2, 2, 3, 3, "7x7_s2_p3"),
    ConvShape(4, 3, 5, 8, 6, 1, 1, 1, 1, 0, 0, "1x1"),
    ConvShape(1, 6, 6, 2, 2, 3, 3, 2, 2, 0, 0, "3x3_s2_p0"),
]


def brute_patch(x, s):
    """X[r,s,c] by six plain loops with explicit bounds checks (no padded copy, no slicing)."""
    X = np.zeros((s.R, s.S, s.C), dtype=np.int64)
    for n in range(s.N):
        for p in range(s.P):
            for q in range(s.Q):
                for r in range(s.R):
                    for c in range(s.S):
                        h, w_ = p * s.stride_h - s.pad_h + r, q * s.stride_w - s.pad_w + c
                        if 0 <= h < s.H and 0 <= w_ < s.W:
                            X[r, c] += x[n, h, w_].astype(np.int64)
    return X


@pytest.mark.parametrize("s", SHAPES, ids=lambda s: s.name)
def test_patch_checksum_against_brute_force(oracle, s):
    x, _ = int8_tensors(s, 7)
    assert np.array_equal(oracle.patch_checksum(x, s), brute_patch(x, s))


def test_patch_checksum_all_ones_hand_worked(oracle):
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "fic_ones_3x3_pad1.txt")) if l.strip() and not l.startswith("#")]
    table = np.array([[int(v) for v in r] for r in rows[:3]])
    total = int(rows[3][0])
    s = ConvShape(3, 5, 4, 2, 7, 3, 3, 1, 1, 1, 1)
    x = np.ones((s.N, s.H, s.W, s.C), dtype=np.int8)
    w = np.ones((s.K, s.R, s.S, s.C), dtype=np.int8)
    X = oracle.patch_checksum(x, s)
    assert np.array_equal(X[:, :, 0], table) and np.array_equal(X[:, :, 1], table)
    res = oracle.abed_fic_int8(x, w, s)
    assert res["dot"] == total and res["ocs"] == total and not res["bad"]


@pytest.mark.parametrize("s", SHAPES + [CONFIG1[0]], ids=lambda s: s.name)
def test_dot_product_equals_sum_of_outputs(oracle, s):
    """Sec. 3.3: <input checksum, filter checksum> = sum of all outputs, with the outputs from the
    independent seven-loop convolution and the dot product re-done here in Python integers."""
    x, w = int8_tensors(s, 21)
    res = oracle.abed_fic_int8(x, w, s)
    y = oracle.conv_int(x, w, s)
    assert res["ocs"] == int(y.sum())
    wsum = w.astype(np.int64).sum(axis=0)
    dot = sum(int(a) * int(b) for a, b in zip(brute_patch(x, s).ravel(), wsum.ravel()))
    assert res["dot"] == dot == res["ocs"] and not res["bad"]


def test_widths_of_sec_4_1(oracle):
    """Input checksum entries need 8 + log2(PQN) bits, the filter checksum 8 + log2(K); int32 holds
    both for the largest configured layers, and the dot product stays far inside int64."""
    from synth import CONFIG2, CONFIG3, resnet50_layers
    for s in CONFIG2 + CONFIG3 + resnet50_layers(128):
        assert 128 * s.N * s.P * s.Q < 2 ** 31 and 128 * s.K < 2 ** 31
        assert 128 * s.N * s.P * s.Q * 128 * s.K * s.C * s.R * s.S < 2 ** 63
    s = ConvShape(2, 4, 4, 2, 3, 3, 3, 1, 1, 1, 1)
    x = np.full((s.N, s.H, s.W, s.C), -128, dtype=np.int8)
    assert oracle.patch_checksum(x, s).min() == -128 * s.N * s.P * s.Q      # the bound is attained in the middle tap


def test_single_faults_are_detected_and_cancelling_pairs_are_not(oracle):
    s = SHAPES[0]
    x, w = int8_tensors(s, 33)
    clean = oracle.abed_fic_int8(x, w, s)
    g = np.random.default_rng(3)
    for _ in range(16):
        idx, bit = int(g.integers(0, s.N * s.P * s.Q * s.K)), int(g.integers(0, 32))
        r = oracle.abed_fic_int8(x, w, s, acc_flip=(idx, bit))
        assert r["bad"] and abs(r["ocs"] - clean["ocs"]) == 2 ** bit and r["dot"] == clean["dot"]
    # a filter corrupted after its checksum was made (Table 1: FIC covers the filters) ...
    w2 = w.copy(); w2[1, 1, 1, 0] ^= 0x10
    r = oracle.abed_fic_int8(x, w2, s, wsum=clean["wsum"])
    assert r["bad"] == (not np.array_equal(r["y"], clean["y"]))
    assert r["bad"]
    # ... and an input corrupted after its checksum was made (it covers the inputs too)
    x2 = x.copy(); x2[1, 2, 1, 2] ^= 0x04
    r = oracle.abed_fic_int8(x2, w, s, xpatch=clean["xpatch"])
    assert r["bad"]
    # a corrupted checksum flags a clean output (verification-path fault)
    xp = clean["xpatch"].copy(); xp[0, 0, 0] += 1
    r = oracle.abed_fic_int8(x, w, s, xpatch=xp)
    assert np.array_equal(r["y"], clean["y"]) and r["bad"] == bool(clean["wsum"][0, 0, 0] != 0)
    # the one scalar cannot see two errors that cancel: +2^b in one accumulator, -2^b in another
    y = clean["y"].astype(np.int64).ravel()
    b = 3
    i = int(np.flatnonzero(((y >> b) & 1) == 0)[0])      # flipping bit b adds 2^b here ...
    j = int(np.flatnonzero(((y >> b) & 1) == 1)[0])      # ... and removes it there
    y2 = clean["y"].copy()
    oracle.flip_bit(y2, i, b)
    oracle.flip_bit(y2, j, b)
    assert not np.array_equal(y2, clean["y"]) and int(y2.astype(np.int64).sum()) == clean["dot"]


@pytest.mark.parametrize("s", SHAPES, ids=lambda s: s.name)
def test_patch_checksum_from_the_batch_sum(oracle, s):
    """The input checksum is linear in x: made from the batch-summed image it equals the one made
    from the images (brute force again as the witness), which is what lets a layer's fused kernel
    hand the next layer the batch sum of its own output (Sec. 4.3)."""
    x, _ = int8_tensors(s, 9)
    xsum = x.astype(np.int64).sum(axis=0)
    assert np.array_equal(oracle.patch_checksum(xsum, s), brute_patch(x, s))


def test_next_layer_checksum_from_the_epilog_output(oracle):
    """Two chained layers: the batch sum of the first layer's int8 output, handed over, gives the
    second layer the same dot product as its own pass over that output."""
    from synth import requant_params
    s1 = ConvShape(6, 8, 8, 16, 32, 3, 3, 1, 1, 1, 1, "a")
    s2 = ConvShape(6, 8, 8, 32, 16, 3, 3, 2, 2, 1, 1, "b")
    x, w1 = int8_tensors(s1, 41)
    _, w2 = int8_tensors(s2, 42)
    scale, bias = requant_params(s1, 41)
    r1 = oracle.abed_fic_int8(x, w1, s1, epilog=(scale, bias, True))
    assert np.array_equal(r1["xsum_next"], r1["out8"].astype(np.int64).sum(axis=0))
    direct = oracle.abed_fic_int8(r1["out8"], w2, s2)
    handed = oracle.abed_fic_int8(r1["out8"], w2, s2, xpatch=oracle.patch_checksum(r1["xsum_next"], s2))
    assert handed["dot"] == direct["dot"] == direct["ocs"] and not handed["bad"]
