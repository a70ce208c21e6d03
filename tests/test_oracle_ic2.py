"""Pins of the oracle's IC option 2 (Sec. 3.2: the input checksum tensor convolved with the K filters
gives K values that the reduced output fmaps must equal), against values that do not come from the
oracle's own formula: the hand-worked all-ones case, a brute-force checksum with the dot products
redone in Python integers, a matrix product for the 1x1 case, the relation to the FIC scalar, and
the algebra of single faults with the blind spot Table 1 (Sec. 3.4) lists."""
import os

import numpy as np
import pytest

from synth import ConvShape, CONFIG1, int8_tensors
from test_oracle_fic import SHAPES, brute_patch

HERE = os.path.dirname(os.path.abspath(__file__))


def test_all_ones_hand_worked(oracle):
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "fic_ones_3x3_pad1.txt")) if l.strip() and not l.startswith("#")]
    total = int(rows[3][0])                         # sum of all outputs of the 7-filter all-ones layer
    s = ConvShape(3, 5, 4, 2, 7, 3, 3, 1, 1, 1, 1)
    x = np.ones((s.N, s.H, s.W, s.C), dtype=np.int8)
    w = np.ones((s.K, s.R, s.S, s.C), dtype=np.int8)
    res = oracle.abed_ic2_int8(x, w, s)
    assert total % s.K == 0
    assert res["chk"].tolist() == [total // s.K] * s.K and res["osum"].tolist() == [total // s.K] * s.K
    assert not res["bad"].any()


@pytest.mark.parametrize("s", SHAPES + [CONFIG1[0]], ids=lambda s: s.name)
def test_k_values_equal_reduced_outputs(oracle, s):
    """Left side from the oracle's convolution, right side from this file's brute-force checksum and
    Python integers."""
    x, w = int8_tensors(s, 17)
    res = oracle.abed_ic2_int8(x, w, s)
    X = brute_patch(x, s)
    for k in range(s.K):
        want = sum(int(a) * int(b) for a, b in zip(X.ravel(), w[k].ravel()))
        assert int(res["chk"][k]) == want
        assert int(res["osum"][k]) == want
    assert not res["bad"].any()
    # the K values add up to the one value of the FIC scheme (Sec. 3.3)
    fic = oracle.abed_fic_int8(x, w, s)
    assert int(res["chk"].sum()) == fic["dot"] and int(res["osum"].sum()) == fic["ocs"]


def test_1x1_is_a_matrix_product(oracle):
    s = ConvShape(5, 4, 6, 16, 9, 1, 1, 1, 1, 0, 0)
    x, w = int8_tensors(s, 23)
    res = oracle.abed_ic2_int8(x, w, s)
    colsum = x.astype(np.int64).reshape(-1, s.C).sum(axis=0)            # every pixel is met exactly once
    assert np.array_equal(res["chk"], w.reshape(s.K, s.C).astype(np.int64) @ colsum)


def test_single_faults(oracle):
    s = SHAPES[0]
    x, w = int8_tensors(s, 33, 1, 100)               # no zero weights or inputs
    clean = oracle.abed_ic2_int8(x, w, s)
    g = np.random.default_rng(5)
    for _ in range(16):
        idx, bit = int(g.integers(0, s.N * s.P * s.Q * s.K)), int(g.integers(0, 32))
        r = oracle.abed_ic2_int8(x, w, s, acc_flip=(idx, bit))
        k = idx % s.K
        assert r["bad"].tolist() == [j == k for j in range(s.K)]
        assert abs(int(r["osum"][k]) - int(clean["osum"][k])) == 2 ** bit and np.array_equal(r["chk"], clean["chk"])
    # an input corrupted after its checksum was made reaches every filter (weights are non-zero)
    x2 = x.copy(); x2[1, 2, 1, 2] ^= 0x04
    r = oracle.abed_ic2_int8(x2, w, s, xpatch=clean["xpatch"])
    assert r["bad"].all()
    # a corrupted filter is outside this scheme's reach: both sides are computed with it
    w2 = w.copy(); w2[1, 1, 1, 0] ^= 0x10
    r = oracle.abed_ic2_int8(x, w2, s)
    assert not np.array_equal(r["y"], clean["y"]) and not r["bad"].any()
    # two errors that cancel inside one filter's sum are invisible, in different filters they are not
    y = clean["y"].astype(np.int64)
    b = 2
    zero = np.argwhere(((y >> b) & 1) == 0)
    one = np.argwhere(((y >> b) & 1) == 1)
    i = zero[0]
    same = one[one[:, 3] == i[3]][0]
    other = one[one[:, 3] != i[3]][0]
    for j, seen in ((same, False), (other, True)):
        y2 = clean["y"].copy()
        y2[tuple(i)] ^= (1 << b)
        y2[tuple(j)] ^= (1 << b)
        osum = y2.astype(np.int64).sum(axis=(0, 1, 2))
        assert (osum != clean["chk"]).any() == seen
