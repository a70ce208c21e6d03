"""Helpers for the GPU parity tests: run the HIP path through the C-ABI binding,
run the oracle on the same inputs, fold the oracle's element-level mismatch
maps onto the library's tile layout."""
import numpy as np
import torch

import paper_2006_04984_amd as abed
from paper_2006_04984_amd import Variant

DEV = "cuda:0"


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


class GpuConv:
    """Buffers and calls for one convolution shape on the GPU."""

    def __init__(self, shape, variant, int8_out=False):
        # variant may carry a scheme selection bit (abed.ONLY_FC / abed.ONLY_IC)
        self.shape, self.variant, self.int8_out = shape, int(variant), int8_out
        self.desc = abed.desc_from_shape(shape)
        self.lay = abed.get_layout(self.desc, 0, self.variant)
        s = shape
        self.y = torch.empty((s.N, s.P, s.Q, s.K), dtype=torch.int8 if int8_out else torch.int32, device=DEV)
        self.y2 = torch.empty_like(self.y) if self.variant == int(Variant.DUPLICATE) else None
        self.flags = torch.full((max(1, self.lay.n_flag_words),), 0xdeadbeef, dtype=torch.int64, device=DEV).to(torch.int32)
        self.ws = torch.empty((max(256, self.lay.workspace_bytes),), dtype=torch.uint8, device=DEV)
        abed.workspace_init(self.ws)
        self.wchk = torch.empty((self.lay.d_f, s.R, s.S, s.C), dtype=torch.int8, device=DEV)
        self.xchk = torch.empty((self.lay.d_i, s.H, s.W, s.C), dtype=torch.int8, device=DEV)
        self.xchk_next = torch.empty((self.lay.d_i, s.P, s.Q, s.K), dtype=torch.int8, device=DEV)

    def prepare(self, w):
        self.w = w if torch.is_tensor(w) else to_dev(w)
        if self.variant & abed.PACKED_FC:
            # filters and checksum filters in one buffer, the checksum filters right behind the K filters
            both = torch.empty((self.shape.K + self.lay.d_f, self.shape.R, self.shape.S, self.shape.C), dtype=torch.int8, device=DEV)
            both[: self.shape.K].copy_(self.w)
            self.w, self.wchk = both[: self.shape.K], both[self.shape.K:]
        if self.lay.d_f:                       # none with the batch checksum scheme alone
            abed.filter_prepare_int8(self.desc, self.w, self.wchk)

    def run(self, x, compute_xchk=True, epilogue=None, inject=None):
        self.x = x if torch.is_tensor(x) else to_dev(x)
        epi = None
        if epilogue is not None:
            self.scale, self.bias = to_dev(epilogue[0]), to_dev(epilogue[1])
            epi = (self.scale, self.bias, epilogue[2])
        abed.conv_int8(self.desc, self.x, self.w, self.wchk, self.xchk, compute_xchk, self.y, self.variant,
                       flags=self.flags, epilogue=epi, xchk_next=self.xchk_next if epi is not None else None,
                       workspace=self.ws, inject=inject, y2=self.y2)
        torch.cuda.synchronize()
        return self.y.cpu().numpy(), self.flags.cpu().numpy().view(np.uint32)[: self.lay.n_flag_words]


def fold_flags(res, shape, lay):
    """Oracle mismatch maps -> expected flag words [grid_m][grid_b][grid_n] for bits 0 and 1,
    and the per-pixel-group corner bit [grid_m] (bit 2 may sit on any word of the group).  With one
    scheme alone (lay.d_i or lay.d_f zero) only that scheme's map is folded and there is no corner."""
    s = shape
    out = np.zeros((lay.grid_m, lay.grid_b, lay.grid_n), dtype=np.uint32)
    corner = np.zeros((lay.grid_m,), dtype=bool)
    PQ = s.P * s.Q
    fc = res["fc_bad"].reshape(s.N, PQ)
    ic = res["ic_bad"].reshape(PQ, s.K)
    co = res["corner_bad"].reshape(PQ)
    for tm in range(lay.grid_m):
        lo, hi = tm * lay.tile_pixels, min(PQ, (tm + 1) * lay.tile_pixels)
        corner[tm] = co[lo:hi].any() and lay.d_f > 0 and lay.d_i > 0
        for tb in range(lay.grid_b if lay.d_f > 0 else 0):
            if fc[tb * lay.tile_batch:(tb + 1) * lay.tile_batch, lo:hi].any():
                out[tm, tb, 0] |= 1
        for tn in range(lay.grid_n if lay.d_i > 0 else 0):
            if ic[lo:hi, tn * lay.tile_n:(tn + 1) * lay.tile_n].any():
                out[tm, 0, tn] |= 2
    return out, corner


def flags_match(flags, res, shape, lay):
    exp, corner = fold_flags(res, shape, lay)
    f = flags.reshape(lay.grid_m, lay.grid_b, lay.grid_n)
    return np.array_equal(f & 3, exp) and np.array_equal(((f & 4) != 0).any(axis=(1, 2)), corner) and not (f & ~np.uint32(7)).any()
