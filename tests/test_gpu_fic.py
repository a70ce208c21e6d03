"""GPU parity of the FIC scheme (Sec. 3.3) through the C ABI against the oracle: the filter
checksum, the row-wise input checksum (folded here to the filter-sized checksum the oracle
defines), the two 64-bit scalars, the flag and the outputs, bit-exact; single faults in the
accumulators, the stored ConvOut, the filters and the inputs."""
import numpy as np
import pytest
import torch

from synth import ConvShape, CONFIG1, CONFIG2, int8_tensors, requant_params

pytestmark = pytest.mark.gpu

DEV = "cuda:0"

SHAPES = [
    CONFIG1[0],
    ConvShape(32, 9, 9, 64, 64, 3, 3, 1, 1, 1, 1, "n32_c64_k64_9x9"),
    ConvShape(5, 7, 6, 16, 48, 3, 3, 2, 2, 1, 1, "n5_k48_stride2"),
    ConvShape(16, 6, 5, 64, 128, 1, 1, 1, 1, 0, 0, "n16_1x1_k128"),
    ConvShape(3, 10, 8, 16, 16, 3, 2, 1, 2, 1, 0, "n3_asym"),
    ConvShape(48, 4, 4, 80, 96, 3, 3, 1, 1, 1, 1, "n48_c80_k96"),
    ConvShape(2, 12, 12, 16, 64, 7, 7, 2, 2, 3, 3, "7x7_s2"),
    ConvShape(12, 5, 5, 320, 80, 3, 3, 1, 1, 1, 1, "n12_c320_k80"),
]


class GpuFic:
    def __init__(self, s, variant, int8_out=False):
        import paper_2006_04984_amd as abed
        self.abed, self.s, self.variant = abed, s, variant
        self.desc = abed.desc_from_shape(s)
        self.lay = abed.fic_get_layout(self.desc, variant)
        self.y = torch.empty((s.N, s.P, s.Q, s.K), dtype=torch.int8 if int8_out else torch.int32, device=DEV)
        self.wsum = torch.empty((s.R, s.S, s.C), dtype=torch.int32, device=DEV)
        self.xrows = torch.empty((self.lay.xrows_parts, s.H, s.S, s.C), dtype=torch.int32, device=DEV)
        self.result = torch.full((2,), -12345, dtype=torch.int64, device=DEV)
        self.flag = torch.full((1,), 77, dtype=torch.int32, device=DEV)
        self.ws = torch.empty((max(256, self.lay.workspace_bytes),), dtype=torch.uint8, device=DEV)
        abed.workspace_init(self.ws)

    def prepare(self, w):
        self.w = torch.from_numpy(w).to(DEV)
        self.abed.fic_filter_prepare_int8(self.desc, self.w, self.wsum)

    def run(self, x, compute=True, epilogue=None, inject=None, xsum_in=None, xsum_next=None):
        self.x = x if torch.is_tensor(x) else torch.from_numpy(x).to(DEV)
        epi = None
        if epilogue is not None:
            self.scale, self.bias = torch.from_numpy(epilogue[0]).to(DEV), torch.from_numpy(epilogue[1]).to(DEV)
            epi = (self.scale, self.bias, epilogue[2])
        self.abed.fic_conv_int8(self.desc, self.x, self.w, self.wsum, self.xrows, compute, self.y, self.variant,
                                self.result, self.flag, epilogue=epi, workspace=self.ws, inject=inject,
                                xsum_in=xsum_in, xsum_next=xsum_next)
        torch.cuda.synchronize()
        r = self.result.cpu().numpy()
        return self.y.cpu().numpy(), int(r[0]), int(r[1]), int(self.flag.item())


def fold_rows(xrows, s):
    """Row-wise input checksum -> the filter-sized one: X[r] = sum of xrows over the input rows filter row r meets."""
    X = np.zeros((s.R, s.S, s.C), dtype=np.int64)
    for r in range(s.R):
        for p in range(s.P):
            h = p * s.stride_h - s.pad_h + r
            if 0 <= h < s.H:
                X[r] += xrows[h]
    return X


@pytest.mark.parametrize("variant", [1, 4])
@pytest.mark.parametrize("s", SHAPES, ids=lambda s: s.name)
def test_clean_run_and_accumulator_flip(oracle, s, variant):
    print("case", s.name, "variant", variant, flush=True)
    lo, hi = (-8, 7) if s.name.startswith("cfg1") else (-128, 127)
    x, w = int8_tensors(s, 6161, lo, hi)
    ref = oracle.abed_fic_int8(x, w, s)
    g = GpuFic(s, variant)
    g.prepare(w)
    y, ocs, dot, flag = g.run(x)
    assert np.array_equal(y, ref["y"])
    assert np.array_equal(g.wsum.cpu().numpy(), ref["wsum"])
    assert np.array_equal(fold_rows(g.xrows.cpu().numpy().astype(np.int64).sum(axis=0), s), ref["xpatch"])
    assert (ocs, dot, flag) == (ref["ocs"], ref["dot"], 0)
    rng = np.random.default_rng(11)
    for _ in range(3):
        idx, bit = int(rng.integers(0, y.size)), int(rng.integers(0, 32))
        print("  flip", idx, bit, flush=True)
        ref2 = oracle.abed_fic_int8(x, w, s, acc_flip=(idx, bit))
        y2, ocs2, dot2, flag2 = g.run(x, inject=(1, idx, bit))
        assert np.array_equal(y2, ref2["y"])
        assert (ocs2, dot2, flag2) == (ref2["ocs"], ref2["dot"], 1)
    # a second clean call on the same buffers clears the flag again
    assert g.run(x)[1:] == (ref["ocs"], ref["dot"], 0)


@pytest.mark.parametrize("variant", [1, 4])
@pytest.mark.parametrize("s", [SHAPES[1], SHAPES[2], SHAPES[7]], ids=lambda s: s.name)
def test_epilog_output(oracle, s, variant):
    print("case", s.name, "variant", variant, flush=True)
    x, w = int8_tensors(s, 6262)
    scale, bias = requant_params(s, 6262)
    ref = oracle.abed_fic_int8(x, w, s, epilog=(scale, bias, True))
    g = GpuFic(s, variant, int8_out=True)
    g.prepare(w)
    y, ocs, dot, flag = g.run(x, epilogue=(scale, bias, True))
    assert np.array_equal(y, ref["out8"]) and (ocs, dot, flag) == (ref["ocs"], ref["dot"], 0)


def test_stored_flip_filter_flip_input_flip(oracle):
    s = SHAPES[1]
    x, w = int8_tensors(s, 6363)
    clean = oracle.abed_fic_int8(x, w, s)
    # stored ConvOut corrupted between the kernels: only the unfused option reads it back
    g = GpuFic(s, 1)
    g.prepare(w)
    idx, bit = 1234, 9
    y, ocs, dot, flag = g.run(x, inject=(2, idx, bit))
    exp = clean["y"].copy(); oracle.flip_bit(exp, idx, bit)
    assert np.array_equal(y, exp) and flag == 1 and abs(ocs - clean["ocs"]) == 2 ** bit and dot == clean["dot"]
    # a filter corrupted after its checksum was made
    g = GpuFic(s, 4)
    g.prepare(w)
    w2 = w.copy(); w2[3, 1, 2, 5] ^= 0x20
    g.w = torch.from_numpy(w2).to(DEV)
    ref = oracle.abed_fic_int8(x, w2, s, wsum=clean["wsum"])
    y, ocs, dot, flag = g.run(x)
    assert np.array_equal(y, ref["y"]) and (ocs, dot, flag) == (ref["ocs"], ref["dot"], 1) and ref["bad"]
    # an input corrupted after its checksum was made
    g = GpuFic(s, 4)
    g.prepare(w)
    g.abed.fic_input_checksum_int8(g.desc, 4, torch.from_numpy(x).to(DEV), g.xrows)
    x2 = x.copy(); x2[7, 4, 4, 17] ^= 0x08
    ref = oracle.abed_fic_int8(x2, w, s, xpatch=clean["xpatch"])
    y, ocs, dot, flag = g.run(x2, compute=False)
    assert np.array_equal(y, ref["y"]) and (ocs, dot, flag) == (ref["ocs"], ref["dot"], 1) and ref["bad"]


def test_full_size_layer_scalars(oracle):
    """A config-2 layer at full size in the launch configuration the benchmark times: the two 64-bit
    scalars against the oracle, outputs on sampled points."""
    s = CONFIG2[1]
    x, w = int8_tensors(s, 2001)
    g = GpuFic(s, 4)
    g.prepare(w)
    y, ocs, dot, flag = g.run(x)
    X = oracle.patch_checksum(x, s)
    ref_dot = int((X * oracle.filter_checksum(w)).sum())
    assert dot == ref_dot and ocs == ref_dot and flag == 0
    rng = np.random.default_rng(5)
    pts = np.stack([rng.integers(0, s.N, 500), rng.integers(0, s.P, 500), rng.integers(0, s.Q, 500), rng.integers(0, s.K, 500)], axis=1)
    exp = oracle.conv_int_points(x, w, s, pts)
    assert np.array_equal(y[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]], exp.astype(np.int32))


def test_unsupported_variants_are_refused():
    import paper_2006_04984_amd as abed
    d = abed.desc_from_shape(SHAPES[1])
    for v in (0, 2, 3, 6):
        with pytest.raises(abed.AbedError) as e:
            abed.fic_get_layout(d, v)
        assert e.value.status == 2


CHAINS = [
    (ConvShape(6, 8, 8, 16, 32, 3, 3, 1, 1, 1, 1, "a3x3"), ConvShape(6, 8, 8, 32, 48, 3, 3, 2, 2, 1, 1, "b3x3s2")),
    (ConvShape(40, 9, 7, 64, 80, 1, 1, 1, 1, 0, 0, "a1x1_n40"), ConvShape(40, 9, 7, 80, 64, 3, 3, 1, 1, 1, 1, "b3x3_n40")),
    (ConvShape(3, 12, 12, 16, 16, 7, 7, 2, 2, 3, 3, "a7x7s2"), ConvShape(3, 6, 6, 16, 32, 1, 1, 1, 1, 0, 0, "b1x1")),
]


@pytest.mark.parametrize("sa,sb", CHAINS, ids=lambda s: s.name)
def test_next_layer_checksum_is_handed_over(oracle, sa, sb):
    """The option that also fuses the next layer's input checksum generation (Sec. 4.3): layer A adds
    the batch sum of its int8 output to xsum; layer B makes its input checksum from xsum instead of a
    pass over A's output, and leaves xsum zero.  Twice in a row on the same buffers."""
    print("case", sa.name, "->", sb.name, flush=True)
    x, wa = int8_tensors(sa, 7171)
    _, wb = int8_tensors(sb, 7272)
    scale, bias = requant_params(sa, 7171)
    ra = oracle.abed_fic_int8(x, wa, sa, epilog=(scale, bias, True))
    rb = oracle.abed_fic_int8(ra["out8"], wb, sb)
    ga, gb = GpuFic(sa, 5, int8_out=True), GpuFic(sb, 5)
    ga.prepare(wa); gb.prepare(wb)
    xsum = torch.zeros((sa.P, sa.Q, sa.K), dtype=torch.int32, device=DEV)
    for rep in range(2):
        ya, ocs, dot, flag = ga.run(x, epilogue=(scale, bias, True), xsum_next=xsum)
        assert np.array_equal(ya, ra["out8"]) and (ocs, dot, flag) == (ra["ocs"], ra["dot"], 0)
        assert np.array_equal(xsum.cpu().numpy(), ra["xsum_next"])
        yb, ocs, dot, flag = gb.run(ga.y, xsum_in=xsum)
        assert np.array_equal(yb, rb["y"]) and (ocs, dot, flag) == (rb["ocs"], rb["dot"], 0)
        assert not xsum.any()
    # B's input corrupted after A made the sum: B's check fires
    ga.run(x, epilogue=(scale, bias, True), xsum_next=xsum)
    bad = ga.y.clone()
    bad.view(-1)[bad.numel() // 2] ^= 0x10
    ref = oracle.abed_fic_int8(bad.cpu().numpy(), wb, sb, xpatch=rb["xpatch"])
    yb, ocs, dot, flag = gb.run(bad, xsum_in=xsum)
    assert np.array_equal(yb, ref["y"]) and (ocs, dot, flag) == (ref["ocs"], ref["dot"], int(ref["bad"])) and ref["bad"]


def test_deferred_verification_of_several_layers(oracle):
    """The comparisons of several layers made in one launch after all of them ran (the paper leaves the
    comparison to the host, Sec. 4.3): per layer the two scalars and the flag, one layer with a flip."""
    import paper_2006_04984_amd as abed
    picks = [(SHAPES[1], 4, None), (SHAPES[2], 4, (1, 100, 20)), (SHAPES[5], 1, None), (SHAPES[3], 5, None)]
    layers, refs = [], []
    for s, variant, inject in picks:
        x, w = int8_tensors(s, 7070 + len(layers))
        g = GpuFic(s, variant)
        g.prepare(w)
        g.x = torch.from_numpy(x).to(DEV)
        abed.fic_conv_int8(g.desc, g.x, g.w, g.wsum, g.xrows, True, g.y, variant, None, None, workspace=g.ws, inject=inject)
        layers.append(g)
        refs.append(oracle.abed_fic_int8(x, w, s, acc_flip=inject[1:] if inject else None))
    results = torch.full((len(picks), 2), -1, dtype=torch.int64, device=DEV)
    flags = torch.full((len(picks),), 99, dtype=torch.int32, device=DEV)
    abed.fic_verify([g.desc for g in layers], [p[1] for p in picks], [g.ws for g in layers], results, flags)
    torch.cuda.synchronize()
    r, f = results.cpu().numpy(), flags.cpu().numpy()
    for i, (g, ref) in enumerate(zip(layers, refs)):
        assert np.array_equal(g.y.cpu().numpy(), ref["y"])
        assert (int(r[i, 0]), int(r[i, 1]), int(f[i])) == (ref["ocs"], ref["dot"], int(ref["bad"]))
    assert f.tolist() == [0, 1, 0, 0]


def test_deferred_needs_both_null():
    import paper_2006_04984_amd as abed
    s = SHAPES[1]
    g = GpuFic(s, 4)
    x, w = int8_tensors(s, 1)
    g.prepare(w)
    g.x = torch.from_numpy(x).to(DEV)
    with pytest.raises(abed.AbedError) as e:
        abed.fic_conv_int8(g.desc, g.x, g.w, g.wsum, g.xrows, True, g.y, 4, g.result, None, workspace=g.ws)
    assert e.value.status == 1
