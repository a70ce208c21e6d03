"""Pins for the oracle of the traditional ABFT-GEMM baseline (Sec. 5.3, with the row + column scheme of
Sec. 2.1): a hand-worked 2x2 case, the library matrix product, the checksum identities on the exact values,
single-fault localisation (one bad row, one bad column: the correction capability), digit bounds."""
import numpy as np
import pytest

from oracle import abft_gemm_oracle as ab
from oracle import abed_oracle as ao


def test_hand_worked_case():
    # A = [[1, 2], [3, 4]], B rows are the output columns: B = [[1, 0], [2, -1]]
    # C = A . B^T = [[1, 0], [3, 2]]; column checksum of A = [4, 6]; checksum of B's rows = [3, -1]
    # last column of C' = A . [3, -1] = [1, 5] = row sums of C; last row = [4, 6] . B^T = [4, 2] = column sums; corner = 4*3 - 6 = 6
    A = np.array([[1, 2], [3, 4]], dtype=np.int8)
    B = np.array([[1, 0], [2, -1]], dtype=np.int8)
    r = ab.abft_gemm_int8(A, B)
    assert r["C"].tolist() == [[1, 0], [3, 2]]
    assert r["csA"].tolist() == [4, 6] and r["rsB"].tolist() == [3, -1]
    assert (r["d_a"], r["d_b"]) == (2, 2)                       # two int8 values can sum beyond one int8
    assert r["Ap"].tolist() == [[1, 2], [3, 4], [4, 6], [0, 0]]
    assert r["Bp"].tolist() == [[1, 0], [2, -1], [3, -1], [0, 0]]
    assert r["Cp"].tolist() == [[1, 0, 1, 0], [3, 2, 5, 0], [4, 2, 6, 0], [0, 0, 0, 0]]
    assert not r["row_bad"].any() and not r["col_bad"].any() and not r["corner_bad"]


@pytest.mark.parametrize("M,Kg,Ng,seed", [(37, 24, 19, 1), (300, 64, 5, 2), (5, 7, 300, 3)])
def test_against_library_product_and_identities(M, Kg, Ng, seed):
    g = np.random.default_rng(seed)
    A = g.integers(-128, 128, (M, Kg)).astype(np.int8)
    B = g.integers(-128, 128, (Ng, Kg)).astype(np.int8)
    r = ab.abft_gemm_int8(A, B)
    C = A.astype(np.int64) @ B.astype(np.int64).T
    assert np.array_equal(r["C"], C.astype(np.int32))           # small enough not to wrap
    # digits: int8 rows that recombine to the exact checksums, and as few as the bit budget of Sec. 4.1 allows
    assert r["Ap"].dtype == np.int8 and r["Ap"].shape == (M + r["d_a"], Kg)
    assert np.array_equal(ao.recombine_digits(list(r["Ap"][M:])), A.astype(np.int64).sum(0))
    assert np.array_equal(ao.recombine_digits(list(r["Bp"][Ng:])), B.astype(np.int64).sum(0))
    assert r["d_a"] == (2 if M <= 257 else 3) and r["d_b"] == (2 if Ng <= 257 else 3)
    # the identities behind the scheme, on the exact values: checksum column = row sums, checksum row = column sums
    E = r["Cp_exact"]
    assert np.array_equal(ao.recombine_digits([E[:M, Ng + d] for d in range(r["d_b"])]), C.sum(1))
    assert np.array_equal(ao.recombine_digits([E[M + d, :Ng] for d in range(r["d_a"])]), C.sum(0))
    assert not r["row_bad"].any() and not r["col_bad"].any() and not r["corner_bad"]


def test_single_fault_is_located():
    g = np.random.default_rng(7)
    M, Kg, Ng = 70, 32, 40
    A = g.integers(-128, 128, (M, Kg)).astype(np.int8)
    B = g.integers(-128, 128, (Ng, Kg)).astype(np.int8)
    for (i, j, bit) in [(0, 0, 0), (69, 39, 31), (13, 7, 17)]:
        r = ab.abft_gemm_int8(A, B, stored_flip=(i, j, bit))
        assert np.flatnonzero(r["row_bad"]).tolist() == [i] and np.flatnonzero(r["col_bad"]).tolist() == [j]
        assert not r["corner_bad"]
        # the difference of the two sums is the error itself: the classical correction
        clean = ab.abft_gemm_int8(A, B)["C"]
        assert (int(r["C"][i, j]) - int(clean[i, j])) % 2 ** 32 == (1 << bit if (int(clean[i, j]) >> bit) & 1 == 0 else -(1 << bit)) % 2 ** 32
    # a fault in a checksum entry: its own line and the corner, no data line of the other kind
    r = ab.abft_gemm_int8(A, B, stored_flip=(5, Ng, 9))          # the checksum column, row 5
    assert np.flatnonzero(r["row_bad"]).tolist() == [5] and not r["col_bad"].any() and r["corner_bad"]
    r = ab.abft_gemm_int8(A, B, stored_flip=(M + 1, 3, 2))        # the second digit of the checksum row, column 3
    assert np.flatnonzero(r["col_bad"]).tolist() == [3] and not r["row_bad"].any() and r["corner_bad"]


def test_sums_that_wrap():
    """Kg = 4096 at full-range values: outputs reach 2^26, 300 of them in a line exceed 2^31; the wrapped
    comparisons still hold on clean data and still see a one-bit fault."""
    g = np.random.default_rng(9)
    A = np.full((300, 4096), 127, dtype=np.int8)
    B = np.full((300, 4096), 127, dtype=np.int8)
    B[::7] = -128
    r = ab.abft_gemm_int8(A, B)
    assert np.abs(r["Cp_exact"][:300, :300].sum(1)).max() > 2 ** 31
    assert not r["row_bad"].any() and not r["col_bad"].any() and not r["corner_bad"]
    r = ab.abft_gemm_int8(A, B, stored_flip=(11, 12, 31))
    assert r["row_bad"].sum() == 1 and r["col_bad"].sum() == 1
