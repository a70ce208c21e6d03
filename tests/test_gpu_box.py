"""GPU parity for the convolution kernel that keeps the checksums local to a workgroup (ABED_LOCAL):
outputs bit for bit against the oracle's convolution; flag words against the oracle's mismatch maps of
every (batch tile, filter tile) sub-problem - the schemes of Sec. 3.1 and Sec. 3.2 option 1 applied to the
tile's own filters and the tile's own images - folded onto the boxes of 8x8 pixels."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2006_04984_amd as abed
from synth import CONFIG2, ConvShape, int8_tensors, requant_params, seed_for

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
V_BOTH = 4 | abed.LOCAL
V_FC = 4 | abed.LOCAL | abed.ONLY_FC
V_IC = 4 | abed.LOCAL | abed.ONLY_IC

SHAPES = [ConvShape(8, 8, 8, 64, 64, 3, 3, 1, 1, 1, 1, "n8_8x8_c64_k64"),
          ConvShape(11, 11, 13, 64, 64, 3, 3, 1, 1, 1, 1, "n11_11x13_ragged"),
          ConvShape(20, 9, 10, 128, 128, 3, 3, 1, 1, 1, 1, "n20_c128_k128_two_tiles_two_chunks"),
          ConvShape(5, 12, 7, 256, 64, 3, 3, 1, 1, 0, 2, "n5_c256_pad0x2"),
          ConvShape(9, 7, 7, 512, 192, 3, 3, 1, 1, 1, 1, "n9_7x7_c512_k192"),
          ConvShape(3, 17, 9, 64, 128, 3, 3, 1, 1, 2, 0, "n3_pad2x0")]


class BoxConv:
    def __init__(self, s, variant, int8_out=False):
        self.s, self.variant = s, int(variant)
        self.desc = abed.desc_from_shape(s)
        self.lay = abed.get_layout(self.desc, 0, self.variant)
        assert self.lay.local_checksums == 1 and self.lay.tile_box == 8 and self.lay.workspace_bytes == 0
        self.y = torch.empty((s.N, s.P, s.Q, s.K), dtype=torch.int8 if int8_out else torch.int32, device=DEV)
        self.flags = torch.full((self.lay.n_flag_words,), 0x5a5a5a5a, dtype=torch.int32, device=DEV)
        self.wchk = torch.zeros((max(1, self.lay.grid_n * self.lay.d_f), s.R, s.S, s.C), dtype=torch.int8, device=DEV)

    def prepare(self, w):
        self.w = torch.from_numpy(w).to(DEV)
        abed.filter_prepare_local_int8(self.desc, self.variant, self.w, self.wchk)
        torch.cuda.synchronize()

    def run(self, x, inject=None, epilogue=None):
        self.x = x if torch.is_tensor(x) else torch.from_numpy(x).to(DEV)
        epi = None
        if epilogue is not None:
            self.scale, self.bias = torch.from_numpy(epilogue[0]).to(DEV), torch.from_numpy(epilogue[1]).to(DEV)
            epi = (self.scale, self.bias, epilogue[2])
        self.y.fill_(-3)
        abed.conv_int8(self.desc, self.x, self.w, self.wchk, None, True, self.y, self.variant, flags=self.flags,
                       epilogue=epi, inject=inject)
        torch.cuda.synchronize()
        L = self.lay
        return self.y.cpu().numpy(), self.flags.cpu().numpy().view(np.uint32).reshape(L.grid_m, L.grid_b, L.grid_n)


def expected_local_flags(oracle, x, w, s, lay, acc_flip=None, wchk=None):
    """Flag words [box][batch tile][filter tile]: the oracle run on every (batch tile, filter tile)
    sub-problem with that tile's own checksums, its element maps folded onto the boxes."""
    bx = (s.Q + 7) // 8
    exp = np.zeros((lay.grid_m, lay.grid_b, lay.grid_n), dtype=np.uint32)
    for tb in range(lay.grid_b):
        n0, n1 = tb * lay.tile_batch, min(s.N, (tb + 1) * lay.tile_batch)
        for tn in range(lay.grid_n):
            k0, k1 = tn * lay.tile_n, (tn + 1) * lay.tile_n
            sub = dataclasses.replace(s, N=n1 - n0, K=k1 - k0)
            flip = None
            if acc_flip is not None:
                n, p, q, k = np.unravel_index(acc_flip[0], (s.N, s.P, s.Q, s.K))
                if n0 <= n < n1 and k0 <= k < k1:
                    flip = (int(np.ravel_multi_index((n - n0, p, q, k - k0), (sub.N, s.P, s.Q, sub.K))), acc_flip[1])
            wc = None if wchk is None else wchk[tn * 2:(tn + 1) * 2]
            r = oracle.abed_int8(x[n0:n1], w[k0:k1], sub, wchk=wc, acc_flip=flip)
            fc = r["fc_bad"].any(axis=0) if lay.d_f else np.zeros((s.P, s.Q), bool)       # [P][Q]
            ic = r["ic_bad"].any(axis=2) if lay.d_i else np.zeros((s.P, s.Q), bool)
            co = r["corner_bad"] if (lay.d_f and lay.d_i) else np.zeros((s.P, s.Q), bool)
            for tm in range(lay.grid_m):
                by, bxx = divmod(tm, bx)
                sl = (slice(by * 8, by * 8 + 8), slice(bxx * 8, bxx * 8 + 8))
                exp[tm, tb, tn] = (1 if fc[sl].any() else 0) | (2 if ic[sl].any() else 0) | (4 if co[sl].any() else 0)
    return exp


@pytest.mark.parametrize("variant", [V_BOTH, V_FC, V_IC], ids=["fc_ic", "fc", "ic"])
@pytest.mark.parametrize("rng_len,eh", [(0, 2), (8, 2), (0, 1), (4, 1)], ids=["autorange", "range8", "halfwg_autorange", "halfwg_range4"])
@pytest.mark.parametrize("s", SHAPES, ids=lambda s: s.name)
def test_box_clean_and_flips(oracle, monkeypatch, s, rng_len, eh, variant):
    """eh = 1: workgroups of four waves and batches of four entries, two workgroups per CU."""
    print("case", s.name, rng_len, eh, hex(variant), flush=True)
    if rng_len:
        monkeypatch.setenv("ABED_BOX_RANGE", str(rng_len))
    monkeypatch.setenv("ABED_BOX_EH", str(eh))
    if eh == 1 and variant != V_FC and s.C > 128:
        # the batch checksum of the half-size workgroups keeps at most two chunks of sums in registers
        with pytest.raises(abed.AbedError) as e:
            abed.get_layout(abed.desc_from_shape(s), 0, variant)
        assert e.value.status == 2
        return
    x, w = int8_tensors(s, 7100 + s.N)
    g = BoxConv(s, variant)
    g.prepare(w)
    y, flags = g.run(x)
    assert np.array_equal(y, oracle.conv_int(x, w, s).astype(np.int32))
    assert not flags.any()
    rng = np.random.default_rng(s.N * 31 + s.C)
    total = s.N * s.P * s.Q * s.K
    for trial in range(4):
        idx = int(rng.integers(0, total)) if trial else total - 1
        bit = int(rng.integers(0, 32))
        print("flip", idx, bit, flush=True)
        y2, f2 = g.run(x, inject=(1, idx, bit))
        exp_y = oracle.conv_int(x, w, s).astype(np.int32)
        exp_y.reshape(-1).view(np.uint32)[idx] ^= np.uint32(1 << bit)
        assert np.array_equal(y2, exp_y)
        exp = expected_local_flags(oracle, x, w, s, g.lay, acc_flip=(idx, bit))
        assert exp.any() and np.array_equal(f2, exp)


def test_box_filter_flip_is_caught_by_fc(oracle):
    """A filter corrupted after its tile's checksum was made: FC fires on every row it changes, in that
    filter tile only; the batch checksum (made from the same inputs) does not see it (Table 1 of Sec. 3.4)."""
    s = SHAPES[2]
    x, w = int8_tensors(s, 7300)
    g = BoxConv(s, V_BOTH)
    g.prepare(w)
    wchk = g.wchk.cpu().numpy()
    wbad = w.copy()
    wbad[100, 1, 2, 5] ^= np.int8(0x10)
    g.w = torch.from_numpy(wbad).to(DEV)
    y, flags = g.run(x)
    assert np.array_equal(y, oracle.conv_int(x, wbad, s).astype(np.int32))
    exp = expected_local_flags(oracle, x, wbad, s, g.lay, wchk=wchk)
    assert np.array_equal(flags & 1, exp & 1) and (flags[:, :, 100 // g.lay.tile_n] & 1).any()
    assert not (flags & 2).any() and not flags[:, :, 1 - 100 // g.lay.tile_n].any()


def test_box_unchecked_matches_oracle(oracle, monkeypatch):
    """The unchecked convolution routed to the box kernel (both filter tile widths)."""
    monkeypatch.setenv("ABED_BOX", "1")
    for s, fbr, eh in ((SHAPES[1], 4, 2), (SHAPES[2], 4, 2), (SHAPES[2], 8, 2), (SHAPES[4], 4, 2),
                       (SHAPES[1], 4, 1), (SHAPES[2], 4, 1), (SHAPES[4], 4, 1)):
        monkeypatch.setenv("ABED_BOX_FBR", str(fbr))
        monkeypatch.setenv("ABED_BOX_EH", str(eh))
        x, w = int8_tensors(s, 7400)
        desc = abed.desc_from_shape(s)
        y = torch.full((s.N, s.P, s.Q, s.K), -9, dtype=torch.int32, device=DEV)
        abed.conv_int8(desc, torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV), None, None, False, y, 0)
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy(), oracle.conv_int(x, w, s).astype(np.int32)), (s.name, fbr, eh)


def test_box_epilog_int8(oracle):
    s = SHAPES[2]
    x, w = int8_tensors(s, 7500)
    scale, bias = requant_params(s, 7500)
    g = BoxConv(s, V_BOTH, int8_out=True)
    g.prepare(w)
    y, flags = g.run(x, epilogue=(scale, bias, True))
    acc = oracle.conv_int(x, w, s).astype(np.int32)
    assert np.array_equal(y, oracle.epilog_int8(acc, scale, bias, True)) and not flags.any()


@pytest.mark.parametrize("li", range(4))
def test_box_config2_full_size(oracle, li):
    """The configured 3x3 layers at full size: whole output tensor, clean flags, one accumulator flip."""
    s = CONFIG2[li]
    print("case", s.name, flush=True)
    x, w = int8_tensors(s, seed_for(2, li))
    g = BoxConv(s, V_BOTH)
    g.prepare(w)
    y, flags = g.run(x)
    ref = oracle.conv_int(x, w, s).astype(np.int32)
    assert np.array_equal(y, ref)
    assert not flags.any()
    idx = int(np.ravel_multi_index((s.N - 1, s.P // 2, s.Q - 1, s.K // 3), (s.N, s.P, s.Q, s.K)))
    y2, f2 = g.run(x, inject=(1, idx, 30))
    ref.reshape(-1).view(np.uint32)[idx] ^= np.uint32(1 << 30)
    assert np.array_equal(y2, ref)
    exp = expected_local_flags(oracle, x, w, s, g.lay, acc_flip=(idx, 30))
    assert np.array_equal(f2, exp) and (exp == 3).sum() == 1 and (exp != 0).sum() == 1
