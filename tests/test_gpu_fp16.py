"""GPU parity for the fp16 path (Sec. 7; the options of Sec. 4.3: unfused, fused write, fused partial reduction, fused
output checksum generation): outputs against the double-precision oracle within
1e-2 relative / 1e-3 absolute; flags against the oracle's threshold test wherever the oracle's
margin is outside a guard band (the kernel sums in fp32 in its own order, so inside the band
either answer is right)."""
import numpy as np
import pytest
import torch

import paper_2006_04984_amd as abed
from synth import ConvShape, CONFIG4, fp16_tensors

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

SHAPES = [ConvShape(16, 9, 9, 32, 64, 3, 3, 1, 1, 1, 1, "n16_c32_k64_9x9"),
          ConvShape(5, 7, 6, 16, 48, 3, 3, 2, 2, 1, 1, "n5_k48_stride2"),
          ConvShape(40, 5, 5, 64, 144, 1, 1, 1, 1, 0, 0, "n40_1x1_k144_split"),
          ConvShape(3, 10, 8, 8, 16, 3, 2, 1, 2, 1, 0, "n3_asym_c8")]


class GpuConv16:
    def __init__(self, s, variant, out_fp32=False):
        self.s, self.variant, self.out_fp32 = s, variant, out_fp32
        self.desc = abed.desc_from_shape(s)
        self.lay = abed.get_layout(self.desc, 1, variant)
        self.y = torch.empty((s.N, s.P, s.Q, s.K), dtype=torch.float32 if out_fp32 else torch.float16, device=DEV)
        self.y2 = torch.empty_like(self.y) if variant == 6 else None
        if (variant & 0xff) == 5:          # the next layer's checksum images come back through y2
            self.y2 = torch.full((2, s.P, s.Q, s.K), 7.0, dtype=torch.float16, device=DEV)
        self.flags = torch.full((max(1, self.lay.n_flag_words),), -1, dtype=torch.int32, device=DEV)
        self.ws = torch.zeros((max(256, self.lay.workspace_bytes),), dtype=torch.uint8, device=DEV)
        abed.workspace_init(self.ws)
        self.wchk = torch.empty((2, s.R, s.S, s.C), dtype=torch.float16, device=DEV)
        self.xchk = torch.empty((2, s.H, s.W, s.C), dtype=torch.float16, device=DEV)

    def prepare(self, w):
        self.w = torch.from_numpy(w).to(DEV)
        abed.filter_prepare_fp16(self.desc, self.w, self.wchk)

    def run(self, x, rtol=1e-3, atol=1e-3, compute_xchk=True, inject=None):
        self.x = x if torch.is_tensor(x) else torch.from_numpy(x).to(DEV)
        abed.conv_fp16(self.desc, self.x, self.w, self.wchk, self.xchk, compute_xchk, self.y, self.variant, rtol, atol,
                       flags=self.flags, out_fp32=self.out_fp32, workspace=self.ws, inject=inject, y2=self.y2)
        torch.cuda.synchronize()
        return self.y.cpu().numpy(), self.flags.cpu().numpy().view(np.uint32)[: self.lay.n_flag_words]


def fold_margin(res, s, lay, thresh):
    """Flag words expected if every check whose oracle margin exceeds `thresh` fires."""
    PQ = s.P * s.Q
    out = np.zeros((lay.grid_m, lay.grid_b, lay.grid_n), dtype=np.uint32)
    fc = (~(res["fc_margin"] <= thresh)).reshape(s.N, PQ)
    ic = (~(res["ic_margin"] <= thresh)).reshape(PQ, s.K)
    for tm in range(lay.grid_m):
        lo, hi = tm * 16, min(PQ, tm * 16 + 16)
        for tb in range(lay.grid_b):
            if fc[tb * lay.tile_batch:(tb + 1) * lay.tile_batch, lo:hi].any():
                out[tm, tb, 0] |= 1
        for tn in range(lay.grid_n):
            if ic[lo:hi, tn * lay.tile_n:(tn + 1) * lay.tile_n].any():
                out[tm, 0, tn] |= 2
    return out


def check_outputs(y, ref):
    exact = ref["y_exact"]
    err = np.abs(y.astype(np.float64) - exact)
    assert np.all(err <= 1e-2 * np.abs(exact) + 1e-3), float(err.max())


@pytest.mark.parametrize("out_fp32", [False, True])
@pytest.mark.parametrize("variant", [0, 1, 2, 3, 4, 5, 6])
@pytest.mark.parametrize("s", SHAPES, ids=lambda s: s.name)
def test_fp16_clean(oracle, s, variant, out_fp32):
    print("case", s.name, variant, out_fp32, flush=True)
    x, w = fp16_tensors(s, 6161)
    g = GpuConv16(s, variant, out_fp32)
    g.prepare(w)
    y, flags = g.run(x, rtol=1e-3, atol=1e-2)
    wchk, xchk = g.wchk.cpu().numpy(), g.xchk.cpu().numpy()
    checked = 1 <= variant <= 5
    ref = oracle.abed_fp16(x, w, s, 1e-3, 1e-2, wchk=wchk if checked else None, xchk=xchk if checked else None)
    check_outputs(y, ref)
    if checked:
        # the checksum tensors themselves: hi + lo reproduces the sums to fp32 accuracy
        wsum = w.astype(np.float64).sum(0)
        xsum = x.astype(np.float64).sum(0)
        assert np.all(np.abs(wchk.astype(np.float64).sum(0) - wsum) <= 2.0 ** -20 * np.abs(wsum) + 2.0 ** -24)
        assert np.all(np.abs(xchk.astype(np.float64).sum(0) - xsum) <= 2.0 ** -18 * np.abs(xsum) + 1e-6)
        assert ref["fc_margin"].max() < -5e-3 and ref["ic_margin"].max() < -5e-3
        assert not flags.any()
    if variant == 5:
        # the handed-on batch checksum: hi + lo against the oracle's sum of the fp16 outputs (the kernel sums in fp32
        # and may round an output the other way where the exact value lies on a rounding boundary: one fp16 ulp of slack)
        nxt = g.y2.cpu().numpy().astype(np.float64).sum(0)
        want = ref["xchk_next"].astype(np.float64).sum(0)
        ulp = np.abs(ref["y"].astype(np.float64)).max(axis=0) * 2.0 ** -10
        assert np.all(np.abs(nxt - want) <= np.abs(want) * 2.0 ** -18 + 1e-5 + ulp)
    if variant == 6:
        assert flags[0] == 0 and torch.equal(g.y, g.y2)


@pytest.mark.parametrize("rtol,atol,l1,guard", [(1e-3, 1e-2, False, 2e-3), (1e-3, 0.0, True, 2e-3), (1e-4, 0.0, True, 2e-4)],
                         ids=["values_1e-3_floor_1e-2", "l1_1e-3", "l1_1e-4"])
@pytest.mark.parametrize("base", [4, 1, 2, 3, 5], ids=["ocg", "unfused", "write", "partial", "iocg"])
@pytest.mark.parametrize("s", [SHAPES[0], SHAPES[2]], ids=lambda s: s.name)
def test_fp16_flip_detection_and_threshold(oracle, s, rtol, atol, l1, guard, base):
    """Flips of one output bit: those the oracle puts clearly above the threshold must be flagged in
    the right tile, those clearly below must not; with the threshold relative to the compared values and
    relative to the sum of magnitudes (no absolute floor)."""
    x, w = fp16_tensors(s, 6262)
    variant = base | (abed.L1_THRESHOLD if l1 else 0)
    g = GpuConv16(s, variant)
    g.prepare(w)
    y, flags = g.run(x, rtol, atol)
    wchk, xchk = g.wchk.cpu().numpy(), g.xchk.cpu().numpy()
    ref = oracle.abed_fp16(x, w, s, rtol, atol, wchk=wchk, xchk=xchk, l1=l1)
    assert ref["fc_margin"].max() < -guard and ref["ic_margin"].max() < -guard and not flags.any()
    rng = np.random.default_rng(11)
    decided = 0
    for trial in range(24 if base == 4 else 12):
        idx = int(rng.integers(0, s.N * s.P * s.Q * s.K))
        bit = int(rng.integers(0, 16))
        print("flip", s.name, idx, bit, flush=True)
        y, flags = g.run(x, rtol, atol, compute_xchk=False, inject=(1, idx, bit))
        ref = oracle.abed_fp16(x, w, s, rtol, atol, wchk=wchk, xchk=xchk, acc_flip=(idx, bit), l1=l1)
        f = flags.reshape(g.lay.grid_m, g.lay.grid_b, g.lay.grid_n) & 3
        must = fold_margin(ref, s, g.lay, guard)
        may = fold_margin(ref, s, g.lay, -guard)
        assert np.all((f & must) == must), "a flip above the threshold was missed"
        assert np.all((f & ~may) == 0), "a flag without a mismatch"
        decided += int(np.array_equal(must, may))
    assert decided >= (12 if base == 4 else 6)


def test_fp16_nonfinite_is_a_mismatch(oracle):
    """A flip that turns an output into an infinity or a NaN (exponent all ones) is flagged under both readings of
    the threshold, also where a tolerance computed from the values would itself be infinite."""
    s = SHAPES[0]
    x, w = fp16_tensors(s, 6363)
    ref = oracle.abed_fp16(x, w, s, 1e-3, 0.0)
    # an element whose fp16 exponent field is 01111 (1 <= |y| < 2): flipping bit 14 gives 11111 = Inf / NaN
    h = ref["y"].reshape(-1).view(np.uint16)
    idx = int(np.flatnonzero(((h >> 10) & 31) == 15)[0])
    for l1 in (False, True):
        g = GpuConv16(s, 4 | (abed.L1_THRESHOLD if l1 else 0))
        g.prepare(w)
        y, flags = g.run(x, 1e-3, 1e-2, inject=(1, idx, 14))
        assert not np.isfinite(y.reshape(-1)[idx])
        r = oracle.abed_fp16(x, w, s, 1e-3, 1e-2, acc_flip=(idx, 14), l1=l1)
        assert r["fc_bad"].sum() == 1 and r["ic_bad"].sum() == 1
        f = flags.reshape(g.lay.grid_m, g.lay.grid_b, g.lay.grid_n)
        n, rem = divmod(idx, s.P * s.Q * s.K)
        pix, k = divmod(rem, s.K)
        assert f[pix // 16, n // g.lay.tile_batch, 0] & 1 and f[pix // 16, 0, k // g.lay.tile_n] & 2


def test_fp16_config4_full_tensor(oracle):
    """The fp16 layer of the benchmark configuration at full size, whole tensor against the oracle; no flag on a
    clean run at the stated relative threshold of 1e-3, neither with a floor of 2e-2 on the value-relative reading
    nor with no floor at all on the magnitude-relative one, and the oracle agrees in both cases."""
    s = CONFIG4[0]
    x, w = fp16_tensors(s, 4000)
    for l1, atol in ((False, 2e-2), (True, 0.0)):
        print("config4", l1, flush=True)
        g = GpuConv16(s, 4 | (abed.L1_THRESHOLD if l1 else 0))
        g.prepare(w)
        y, flags = g.run(x, rtol=1e-3, atol=atol)
        ref = oracle.abed_fp16(x, w, s, 1e-3, atol, wchk=g.wchk.cpu().numpy(), xchk=g.xchk.cpu().numpy(), l1=l1)
        check_outputs(y, ref)
        assert np.isfinite(y).all()
        assert not (ref["fc_bad"].any() or ref["ic_bad"].any() or ref["corner_bad"].any())
        assert ref["fc_margin"].max() < -2e-3 and ref["ic_margin"].max() < -2e-3
        assert not flags.any()


def test_fp16_iocg_chain(oracle):
    """Two layers chained through the handed-on checksum (Sec. 4.3): layer 2 runs with compute_xchk = 0 on the images
    layer 1 emitted, raises no flag on clean data and flags a layer-1 output corrupted in memory between the layers."""
    s1 = ConvShape(40, 9, 9, 32, 64, 3, 3, 1, 1, 1, 1, "l1")      # several batch tiles: the sums span tiles
    s2 = ConvShape(40, 9, 9, 64, 48, 1, 1, 1, 1, 0, 0, "l2")
    x, w1 = fp16_tensors(s1, 6464)
    _, w2 = fp16_tensors(s2, 6465)
    g1 = GpuConv16(s1, 5)
    assert g1.lay.grid_b > 1
    g1.prepare(w1)
    y1, f1 = g1.run(x, 1e-3, 1e-2)
    assert not f1.any()
    g2 = GpuConv16(s2, 4)
    g2.prepare(w2)
    g2.xchk = g1.y2
    y2, f2 = g2.run(g1.y, 1e-3, 1e-2, compute_xchk=False)
    ref2 = oracle.abed_fp16(y1, w2, s2, 1e-3, 1e-2, wchk=g2.wchk.cpu().numpy(), xchk=g1.y2.cpu().numpy())
    check_outputs(y2, ref2)
    assert ref2["ic_margin"].max() < -2e-3 and not f2.any()
    ybad = g1.y.clone()
    idx = ((7 * s1.P + 4) * s1.Q + 2) * s1.K + 9
    ybad.view(-1).view(torch.int16)[idx] ^= 1 << 13
    _, f3 = g2.run(ybad, 1e-3, 1e-2, compute_xchk=False)
    pix = 4 * s1.Q + 2
    f3 = f3.reshape(g2.lay.grid_m, g2.lay.grid_b, g2.lay.grid_n)
    assert (f3[pix // 16, 0, :] & 2).any() and not (np.delete(f3, pix // 16, axis=0) & 2).any()
