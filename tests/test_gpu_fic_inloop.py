"""GPU parity of the FIC scheme (Sec. 3.3) with the input side formed in the convolution's main loop,
through the C ABI against the oracle: the digits of the filter checksum, the two 64-bit scalars (the same
numbers as the scheme's other options give), the flag and the outputs, bit-exact; single faults in the
accumulators and the filters; the comparison deferred to abed_fic_verify."""
import dataclasses

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
    ConvShape(32, 7, 7, 512, 512, 3, 3, 1, 1, 1, 1, "wave_groups_512at7"),
    ConvShape(8, 14, 14, 256, 1024, 1, 1, 1, 1, 0, 0, "wide_1x1_k1024"),
]


class GpuFicInloop:
    def __init__(self, s, int8_out=False):
        import paper_2006_04984_amd as abed
        self.abed, self.s = abed, s
        self.desc = abed.desc_from_shape(s)
        self.lay = abed.fic_inloop_get_layout(self.desc)
        self.y = torch.empty((s.N, s.P, s.Q, s.K), dtype=torch.int8 if int8_out else torch.int32, device=DEV)
        self.wdig = torch.full((self.lay.wdig_bytes,), 99, dtype=torch.int8, device=DEV)
        self.result = torch.full((2,), -12345, dtype=torch.int64, device=DEV)
        self.flag = torch.full((1,), 77, dtype=torch.int32, device=DEV)
        self.ws = torch.empty((max(256, self.lay.workspace_bytes),), dtype=torch.uint8, device=DEV)
        abed.workspace_init(self.ws)

    def prepare(self, w):
        self.w = torch.from_numpy(w).to(DEV)
        self.abed.fic_inloop_filter_prepare_int8(self.desc, self.w, self.wdig)

    def run(self, x, epilogue=None, inject=None, deferred=False):
        self.x = x if torch.is_tensor(x) else torch.from_numpy(x).to(DEV)
        epi = None
        if epilogue is not None:
            self.scale, self.bias = torch.from_numpy(epilogue[0]).to(DEV), torch.from_numpy(epilogue[1]).to(DEV)
            epi = (self.scale, self.bias, epilogue[2])
        self.abed.fic_inloop_conv_int8(self.desc, self.x, self.w, self.wdig, self.y, None if deferred else self.result,
                                       None if deferred else self.flag, epilogue=epi, workspace=self.ws, inject=inject)
        torch.cuda.synchronize()
        r = self.result.cpu().numpy()
        return self.y.cpu().numpy(), int(r[0]), int(r[1]), int(self.flag.item())


def digits_value(wdig, s):
    """[3][pad] digits -> the values they stand for, and the padding."""
    crs = s.R * s.S * s.C
    d = wdig.reshape(3, -1).astype(np.int64)
    return (d[0] + 256 * d[1] + 65536 * d[2])[:crs].reshape(s.R, s.S, s.C), d[:, crs:]


@pytest.mark.parametrize("s", SHAPES, ids=lambda s: s.name)
def test_clean_run_and_accumulator_flip(oracle, s):
    print("case", s.name, flush=True)
    lo, hi = (-8, 7) if s.name.startswith("cfg1") else (-128, 127)
    x, w = int8_tensors(s, 7171, lo, hi)
    ref = oracle.abed_fic_int8(x, w, s)
    g = GpuFicInloop(s)
    g.prepare(w)
    val, tail = digits_value(g.wdig.cpu().numpy(), s)
    assert np.array_equal(val, ref["wsum"]) and not tail.any()
    y, ocs, dot, flag = g.run(x)
    assert np.array_equal(y, ref["y"])
    assert (ocs, dot, flag) == (ref["ocs"], ref["dot"], 0)
    rng = np.random.default_rng(12)
    for _ in range(3):
        idx, bit = int(rng.integers(0, y.size)), int(rng.integers(0, 32))
        print("  flip", idx, bit, flush=True)
        ref2 = oracle.abed_fic_int8(x, w, s, acc_flip=(idx, bit))
        y2, ocs2, dot2, flag2 = g.run(x, inject=(1, idx, bit))
        assert np.array_equal(y2, ref2["y"])
        assert (ocs2, dot2, flag2) == (ref2["ocs"], ref2["dot"], 1)
    # a second clean call on the same buffers clears the flag again
    assert g.run(x)[1:] == (ref["ocs"], ref["dot"], 0)


def test_extreme_values(oracle):
    """All inputs and filters at -128: the largest digit products and sums the shape can produce."""
    s = ConvShape(8, 6, 6, 128, 96, 3, 3, 1, 1, 1, 1, "extreme")
    x = np.full((s.N, s.H, s.W, s.C), -128, dtype=np.int8)
    w = np.full((s.K, s.R, s.S, s.C), -128, dtype=np.int8)
    ref = oracle.abed_fic_int8(x, w, s)
    g = GpuFicInloop(s)
    g.prepare(w)
    y, ocs, dot, flag = g.run(x)
    assert np.array_equal(y, ref["y"]) and (ocs, dot, flag) == (ref["ocs"], ref["dot"], 0)


@pytest.mark.parametrize("s", [SHAPES[1], SHAPES[2], SHAPES[7]], ids=lambda s: s.name)
def test_epilog_output(oracle, s):
    print("case", s.name, flush=True)
    x, w = int8_tensors(s, 7272)
    scale, bias = requant_params(s, 7272)
    ref = oracle.abed_fic_int8(x, w, s, epilog=(scale, bias, True))
    g = GpuFicInloop(s, int8_out=True)
    g.prepare(w)
    y, ocs, dot, flag = g.run(x, epilogue=(scale, bias, True))
    assert np.array_equal(y, ref["out8"]) and (ocs, dot, flag) == (ref["ocs"], ref["dot"], 0)


def test_filter_flip_after_the_checksum(oracle):
    s = SHAPES[1]
    x, w = int8_tensors(s, 7373)
    clean = oracle.abed_fic_int8(x, w, s)
    g = GpuFicInloop(s)
    g.prepare(w)
    w2 = w.copy(); w2[3, 1, 2, 5] ^= 0x20
    g.w = torch.from_numpy(w2).to(DEV)
    ref = oracle.abed_fic_int8(x, w2, s, wsum=clean["wsum"])
    y, ocs, dot, flag = g.run(x)
    assert np.array_equal(y, ref["y"]) and (ocs, dot, flag) == (ref["ocs"], ref["dot"], 1) and ref["bad"]


def test_deferred_verification_with_other_options(oracle):
    """Layers run by this entry point and by abed_fic_conv_int8, compared in one abed_fic_verify launch."""
    import paper_2006_04984_amd as abed
    from test_gpu_fic import GpuFic
    shapes = [SHAPES[1], SHAPES[3], SHAPES[5]]
    gs, refs, variants = [], [], []
    for i, s in enumerate(shapes):
        x, w = int8_tensors(s, 7400 + i)
        inject = (1, 17, 5) if i == 2 else None
        refs.append(oracle.abed_fic_int8(x, w, s, acc_flip=(17, 5) if inject else None))
        if i == 1:
            g = GpuFic(s, 4)
            g.prepare(w)
            abed.fic_conv_int8(g.desc, torch.from_numpy(x).to(DEV), g.w, g.wsum, g.xrows, True, g.y, 4, None, None, workspace=g.ws)
            variants.append(4)
        else:
            g = GpuFicInloop(s)
            g.prepare(w)
            g.run(x, inject=inject, deferred=True)
            variants.append(abed.FIC_INLOOP)
        gs.append(g)
    res = torch.zeros((len(gs), 2), dtype=torch.int64, device=DEV)
    flags = torch.full((len(gs),), 9, dtype=torch.int32, device=DEV)
    abed.fic_verify([g.desc for g in gs], variants, [g.ws for g in gs], res, flags)
    torch.cuda.synchronize()
    r, f = res.cpu().numpy(), flags.cpu().numpy()
    for i, ref in enumerate(refs):
        assert (int(r[i, 0]), int(r[i, 1]), int(f[i])) == (ref["ocs"], ref["dot"], 1 if i == 2 else 0)


def test_full_size_layers_sampled(oracle):
    """Config-2 layers at full size: the two scalars against the oracle's (which computes them whole), flag clean."""
    for s in (CONFIG2[0], CONFIG2[3]):
        print("case", s.name, flush=True)
        x, w = int8_tensors(s, 7500)
        ref = oracle.abed_fic_int8(x, w, s)
        g = GpuFicInloop(s)
        g.prepare(w)
        y, ocs, dot, flag = g.run(x)
        assert (ocs, dot, flag) == (ref["ocs"], ref["dot"], 0) and np.array_equal(y, ref["y"])


def test_errors():
    import paper_2006_04984_amd as abed
    s = SHAPES[1]
    g = GpuFicInloop(s)
    x, w = int8_tensors(s, 1)
    g.prepare(w)
    xd = torch.from_numpy(x).to(DEV)
    with pytest.raises(abed.AbedError):      # workspace too small
        abed.fic_inloop_conv_int8(g.desc, xd, g.w, g.wdig, g.y, g.result, g.flag, workspace=g.ws[:256])
    with pytest.raises(abed.AbedError):      # result without flag
        abed.fic_inloop_conv_int8(g.desc, xd, g.w, g.wdig, g.y, g.result, None, workspace=g.ws)
    with pytest.raises(abed.AbedError):      # a stored-output fault needs an unfused option
        abed.fic_inloop_conv_int8(g.desc, xd, g.w, g.wdig, g.y, g.result, g.flag, workspace=g.ws, inject=(2, 0, 0))
    big = dataclasses.replace(s, C=1024)     # 9216 elements along the reduction axis: the digits do not fit beside the tile
    with pytest.raises(abed.AbedError):
        abed.fic_inloop_get_layout(abed.desc_from_shape(big))


def _random_shape(seed):
    rng = np.random.default_rng(seed)
    while True:
        R, S = int(rng.choice([1, 2, 3, 5])), int(rng.choice([1, 2, 3, 5]))
        sh, sw = int(rng.integers(1, 3)), int(rng.integers(1, 3))
        ph, pw = int(rng.integers(0, min(R, 3))), int(rng.integers(0, min(S, 3)))
        H, W = int(rng.integers(1, 13)), int(rng.integers(1, 13))
        if H + 2 * ph < R or W + 2 * pw < S:
            continue
        N = int(rng.choice([1, 2, 3, 5, 8, 13, 24, 33, 40]))
        C = int(rng.choice([16, 32, 48, 64, 80, 128, 272]))
        K = int(rng.choice([1, 7, 13, 16, 30, 32, 47, 48, 64, 77, 96, 130, 144, 272]))
        return ConvShape(N, H, W, C, K, R, S, sh, sw, ph, pw, "rnd%d" % seed), bool(rng.integers(0, 2))


@pytest.mark.parametrize("seed", range(40))
def test_random_shape(oracle, seed):
    """Seeded random shapes (extents that fit no tile size, both digit counts, both loader paths), int32 or int8
    output: outputs and both scalars against the oracle, clean and with one accumulator flip."""
    s, int8_out = _random_shape(seed)
    print("case", seed, s, "int8_out", int8_out, flush=True)
    x, w = int8_tensors(s, 9500 + seed)
    epi = None
    if int8_out:
        scale, bias = requant_params(s, 9500 + seed)
        epi = (scale, bias, bool(seed & 1))
    ref = oracle.abed_fic_int8(x, w, s, epilog=epi)
    g = GpuFicInloop(s, int8_out=int8_out)
    g.prepare(w)
    y, ocs, dot, flag = g.run(x, epilogue=epi)
    assert np.array_equal(y, ref["out8"] if int8_out else ref["y"])
    assert (ocs, dot, flag) == (ref["ocs"], ref["dot"], 0)
    idx, bit = (s.N * s.P * s.Q * s.K) // 2, seed % 32
    ref2 = oracle.abed_fic_int8(x, w, s, acc_flip=(idx, bit), epilog=epi)
    y2, ocs2, dot2, flag2 = g.run(x, epilogue=epi, inject=(1, idx, bit))
    assert np.array_equal(y2, ref2["out8"] if int8_out else ref2["y"])
    assert (ocs2, dot2, flag2) == (ref2["ocs"], ref2["dot"], 1)


def test_lane_sums_in_groups_of_four(oracle, monkeypatch):
    """A tile shape and reduction axis for which a lane's accumulators no longer add up inside 32 bits
    (R*S*C * 4*WM*WK * 2^14 >= 2^31): the output sum is then formed in groups of four.  Both FIC forms."""
    import paper_2006_04984_amd as abed
    from test_gpu_fic import GpuFic
    monkeypatch.setenv("ABED_TILE_WM", "2")
    monkeypatch.setenv("ABED_TILE_WK", "8")
    monkeypatch.setenv("ABED_TILE_KG", "1")
    s = ConvShape(16, 7, 7, 512, 256, 3, 3, 1, 1, 1, 1, "c512_k256_2x8_tiles")
    x, w = int8_tensors(s, 7600)
    ref = oracle.abed_fic_int8(x, w, s)
    g = GpuFicInloop(s)
    assert (abed.get_layout(g.desc, 0, 0).tile_batch, abed.get_layout(g.desc, 0, 0).tile_n) == (8, 128)
    g.prepare(w)
    y, ocs, dot, flag = g.run(x)
    assert np.array_equal(y, ref["y"]) and (ocs, dot, flag) == (ref["ocs"], ref["dot"], 0)
    r = GpuFic(s, 4)
    r.prepare(w)
    y, ocs, dot, flag = r.run(x)
    assert np.array_equal(y, ref["y"]) and (ocs, dot, flag) == (ref["ocs"], ref["dot"], 0)
    # the largest magnitudes: every product 16384
    x[:] = -128
    w[:] = -128
    ref = oracle.abed_fic_int8(x, w, s)
    g.prepare(w)
    y, ocs, dot, flag = g.run(x)
    assert np.array_equal(y, ref["y"]) and (ocs, dot, flag) == (ref["ocs"], ref["dot"], 0)
