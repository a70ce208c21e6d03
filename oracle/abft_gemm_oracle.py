"""CPU oracle for the traditional ABFT technique applied at the GEMM level, the comparison system of
Sec. 5.3 (method) and Sec. 6.3 (results) of the paper, with the row + column checksum scheme that
Sec. 2.1 recalls.

TEST INFRASTRUCTURE ONLY (see abed_oracle.py): only tests/ and the benchmark's cpu_baseline leg may
import this module; the product path never does and shares no code with it.

The GEMM is C[M, Ng] = A[M, Kg] . B[Ng, Kg]^T on int8 operands with exact integer accumulation
(a convolution lowered to a GEMM has M = N*P*Q, Kg = C*R*S, Ng = K).  The tasks, in the paper's order:

 (1)-(2) larger operands with room for checksums, the data copied into them:
         A' = [A ; column checksum of A], B' = [B ; row checksum of B];
 (3)     the checksums: csA[k] = sum_m A[m, k],  rsB[k] = sum_n B[n, k]  (exact), stored as balanced
         base-256 int8 digit rows (Sec. 4.1 applied to the two checksum vectors: the sums do not
         fit the operand type);
 (4)     the larger GEMM C' = A' . B'^T: its last d_b columns are the digits' products with A (the
         row checksums of C in digit form), its last d_a rows those with B (the column checksums);
 (5)     verification: the output is reduced once along rows and once along columns, and each sum is
         compared with the recombined checksum entries; the corner (digit rows x digit columns)
         against the sums of the checksum column and of the checksum row;
 (6)     C' without its checksum rows and columns is the result.

All comparisons are made mod 2^32 (as everywhere in this build; the exact int64 values are kept
beside them).  A single wrong element of C shows as exactly one bad row and one bad column, which
is what gives the classical scheme its correction capability (Sec. 2.1).
"""
import numpy as np

from .abed_oracle import num_digits_for_count, split_digits, recombine_digits, wrap32


def abft_gemm_int8(A, B, stored_flip=None):
    """Tasks (1)-(6) above.  A: int8 [M, Kg]; B: int8 [Ng, Kg] (one row per output column, as filters are
    stored).  stored_flip = (row, column, bit) flips one bit of the stored int32 C' between tasks (4) and (5)
    (row < M + d_a, column < Ng + d_b).
    Returns a dict: C (int32 [M, Ng], task 6), Cp (the larger output, int32), csA / rsB (exact sums), d_a / d_b,
    Ap / Bp (the larger operands), row_bad [M], col_bad [Ng], corner_bad (bool)."""
    A = np.asarray(A, dtype=np.int8)
    B = np.asarray(B, dtype=np.int8)
    M, Kg = A.shape
    Ng = B.shape[0]
    assert B.shape[1] == Kg
    csA = A.astype(np.int64).sum(axis=0)                 # column checksum of A: one value per k
    rsB = B.astype(np.int64).sum(axis=0)                 # checksum over the rows of B (the columns of C)
    d_a, d_b = num_digits_for_count(M), num_digits_for_count(Ng)
    Ap = np.concatenate([A, split_digits(csA, d_a)], axis=0)          # [M + d_a, Kg]
    Bp = np.concatenate([B, split_digits(rsB, d_b)], axis=0)          # [Ng + d_b, Kg]
    Cp64 = Ap.astype(np.int64) @ Bp.astype(np.int64).T                # task 4, exact
    Cp = wrap32(Cp64).copy()
    if stored_flip is not None:
        r, c, bit = stored_flip
        Cp.view(np.uint32)[r, c] ^= np.uint32(1 << bit)
    C = Cp[:M, :Ng]
    # task 5: rows, then columns, then the corner; mod 2^32
    row_sum = wrap32(C.astype(np.int64).sum(axis=1))
    row_chk = wrap32(recombine_digits([Cp[:M, Ng + d] for d in range(d_b)]))
    col_sum = wrap32(C.astype(np.int64).sum(axis=0))
    col_chk = wrap32(recombine_digits([Cp[M + d, :Ng] for d in range(d_a)]))
    corner = wrap32(recombine_digits([recombine_digits([Cp[M + i, Ng + j] for j in range(d_b)]) for i in range(d_a)]))
    # the checksum column summed over the rows, the checksum row summed over the columns
    corner_bad = bool(wrap32(row_chk.astype(np.int64).sum()) != corner) or bool(wrap32(col_chk.astype(np.int64).sum()) != corner)
    return dict(C=C.copy(), Cp=Cp, Cp_exact=Cp64, csA=csA, rsB=rsB, d_a=d_a, d_b=d_b, Ap=Ap, Bp=Bp,
                row_bad=row_sum != row_chk, col_bad=col_sum != col_chk, corner_bad=corner_bad)
