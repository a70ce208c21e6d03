"""GPU parity for the traditional ABFT-GEMM baseline (Sec. 5.3; row + column checksums of Sec. 2.1) against its
oracle: result, the whole larger output incl. checksum rows and columns, clean flags, and single faults in the
stored output located by one bad row and one bad column."""
import numpy as np
import pytest
import torch

import paper_2006_04984_amd as abed
from oracle import abft_gemm_oracle as ab

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


class AbftGemm:
    def __init__(self, M, Ng, Kg):
        self.M, self.Ng, self.Kg = M, Ng, Kg
        self.lay = abed.abft_gemm_get_layout(M, Ng, Kg)
        self.ws = torch.full((self.lay.workspace_bytes,), 0x5a, dtype=torch.uint8, device=DEV)
        self.C = torch.full((M, Ng), -7, dtype=torch.int32, device=DEV)
        self.flags = torch.full((8,), -1, dtype=torch.int32, device=DEV)

    def run(self, A, B, inject=None):
        self.A, self.B = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
        abed.abft_gemm_int8(self.M, self.Ng, self.Kg, self.A, self.B, self.C, self.flags, self.ws, inject=inject)
        torch.cuda.synchronize()
        L = self.lay
        cp = self.ws[L.c_offset: L.c_offset + L.rows_padded * L.ld_c * 4].view(torch.int32).reshape(L.rows_padded, L.ld_c)
        return self.C.cpu().numpy(), cp.cpu().numpy(), self.flags.cpu().numpy().view(np.uint32)


@pytest.mark.parametrize("M,Kg,Ng,full", [(70, 32, 40, False), (1000, 576, 64, False), (300, 4096, 300, True),
                                           (6272, 256, 64, False), (513, 64, 257, False)])
def test_abft_gemm_matches_oracle(M, Kg, Ng, full):
    print("case", M, Kg, Ng, flush=True)
    g = np.random.default_rng(M + Kg)
    if full:        # sums that wrap: extreme values
        A = np.full((M, Kg), 127, dtype=np.int8)
        B = np.full((Ng, Kg), 127, dtype=np.int8)
        B[::7] = -128
    else:
        A = g.integers(-128, 128, (M, Kg)).astype(np.int8)
        B = g.integers(-128, 128, (Ng, Kg)).astype(np.int8)
    ref = ab.abft_gemm_int8(A, B)
    h = AbftGemm(M, Ng, Kg)
    assert (h.lay.d_a, h.lay.d_b) == (ref["d_a"], ref["d_b"])
    C, cp, flags = h.run(A, B)
    assert np.array_equal(C, ref["C"])
    # the larger output: data, checksum rows and columns, corner; zeros in the padding
    da, db = ref["d_a"], ref["d_b"]
    assert np.array_equal(cp[: M + da, : Ng + db], ref["Cp"])
    assert not cp[M + da:, :].any() and not cp[:, Ng + db:].any()
    assert flags[:3].tolist() == [0, 0, 0]
    # single faults in the stored output between the larger GEMM and the verification
    for (i, j, bit) in [(0, 0, 0), (M - 1, Ng - 1, 31), (M // 2, Ng // 3, 13)]:
        bad = ab.abft_gemm_int8(A, B, stored_flip=(i, j, bit))
        C2, _, f2 = h.run(A, B, inject=(2, i * h.lay.ld_c + j, bit))
        assert np.array_equal(C2, bad["C"])
        assert f2[0] == 3 and f2[1] == 1 and f2[2] == 1 and (f2[3], f2[4]) == (i, j)
        assert np.flatnonzero(bad["row_bad"]).tolist() == [i] and np.flatnonzero(bad["col_bad"]).tolist() == [j]
    # a fault in a checksum entry: its line and the corner
    bad = ab.abft_gemm_int8(A, B, stored_flip=(5, Ng, 9))
    _, _, f2 = h.run(A, B, inject=(2, 5 * h.lay.ld_c + Ng, 9))
    assert f2[0] == 5 and f2[1] == 1 and f2[2] == 0 and f2[3] == 5
    assert bad["corner_bad"] and bad["row_bad"].sum() == 1 and not bad["col_bad"].any()
    bad = ab.abft_gemm_int8(A, B, stored_flip=(M + 1, 3, 2))
    _, _, f2 = h.run(A, B, inject=(2, (M + 1) * h.lay.ld_c + 3, 2))
    assert f2[0] == 6 and f2[1] == 0 and f2[2] == 1 and f2[4] == 3
    assert bad["corner_bad"] and bad["col_bad"].sum() == 1 and not bad["row_bad"].any()
    # a corrupted operand after the checksums were made is caught too: rerun only tasks 4-6 with a changed A'
    T = abed.ABFT_TASKS
    abed.abft_gemm_int8(M, Ng, Kg, h.A, h.B, h.C, h.flags, h.ws, tasks=T["copy_in"] | T["checksums"])
    h.ws[7 * Kg + 3] ^= 0x40                     # element (7, 3) of the larger A
    abed.abft_gemm_int8(M, Ng, Kg, h.A, h.B, h.C, h.flags, h.ws, tasks=T["gemm"] | T["verify"] | T["copy_out"])
    torch.cuda.synchronize()
    f3 = h.flags.cpu().numpy().view(np.uint32)
    # row 7 of the output changes in every column whose B has a non-zero element 3: the column check sees it, the row
    # check does not (the row's checksum entry is computed from the same corrupted row)
    assert f3[0] & 2 and not f3[0] & 1
