"""GPU tests of the fused next-layer checksum (variant 5) and of the error
coverage of the checks under single-bit flips in every tensor (Sec. 3.4 Table 1,
Sec. 5.4 / 6.4 injections), against the oracle given the same corrupted tensors."""
import numpy as np
import pytest
import torch

from synth import ConvShape, CONFIG1, int8_tensors, requant_params

pytestmark = pytest.mark.gpu

S1 = ConvShape(32, 9, 9, 32, 64, 3, 3, 1, 1, 1, 1, "n32_c32_k64_9x9")
S2 = ConvShape(64, 5, 5, 16, 320, 3, 3, 1, 1, 1, 1, "n64_k320_split")
S3 = ConvShape(6, 8, 8, 16, 32, 3, 3, 1, 1, 1, 1, "n6_small")


@pytest.mark.parametrize("s", [S1, S2, S3], ids=lambda s: s.name)
def test_next_layer_checksum(oracle, s):
    """Variant 5 emits the digits of sum_n out8[n] (Sec. 4.3, the fused input/output checksum option)."""
    from gpu_helpers import GpuConv
    x, w = int8_tensors(s, 5151)
    scale, bias = requant_params(s, 5151)
    ref = oracle.abed_int8(x, w, s, epilog=(scale, bias, True))
    g = GpuConv(s, 5, int8_out=True)
    g.prepare(w)
    y, flags = g.run(x, epilogue=(scale, bias, True))
    assert np.array_equal(y, ref["out8"]) and not flags.any()
    got = g.xchk_next.cpu().numpy()
    assert np.array_equal(oracle.recombine_digits(list(got)), ref["xsum_next"])
    assert np.array_equal(got, ref["xchk_next"])


def test_chained_layers_reuse_the_emitted_checksum(oracle):
    """Two convolutions in a row: the second takes its batch checksum from the first kernel
    (no ICG launch) and still verifies clean; a flip in the tensor between the layers is caught."""
    from gpu_helpers import GpuConv, to_dev
    s1 = ConvShape(32, 8, 8, 32, 64, 3, 3, 1, 1, 1, 1, "l1")
    s2 = ConvShape(32, 8, 8, 64, 32, 1, 1, 1, 1, 0, 0, "l2")
    x, w1 = int8_tensors(s1, 5252)
    _, w2 = int8_tensors(s2, 5253)
    scale, bias = requant_params(s1, 5252)
    g1 = GpuConv(s1, 5, int8_out=True); g1.prepare(w1)
    y1, f1 = g1.run(x, epilogue=(scale, bias, True))
    g2 = GpuConv(s2, 4); g2.prepare(w2)
    g2.xchk.copy_(g1.xchk_next)
    y2, f2 = g2.run(g1.y, compute_xchk=False)
    ref2 = oracle.abed_int8(y1, w2, s2)
    assert np.array_equal(y2, ref2["y"]) and not f1.any() and not f2.any()
    # corrupt the intermediate tensor after the first layer emitted its checksum
    bad = g1.y.clone()
    bad.view(torch.uint8).view(-1)[12345] ^= 0x10
    y2b, f2b = g2.run(bad, compute_xchk=False)
    assert (y2b != y2).any() and (f2b & 2).any() and not (f2b & 1).any()


def flip_dev(t, flat_index, bit):
    u = t.view(torch.uint8).view(-1)
    u[flat_index] ^= (1 << bit)


@pytest.mark.parametrize("variant", [1, 2, 3, 4])
def test_coverage_matrix_on_gpu(oracle, variant):
    """Flips in x, w, wchk, xchk after the checksums were generated: FC must miss input flips and
    catch filter flips, IC the other way round, checksum flips raise a flag with clean outputs."""
    from gpu_helpers import GpuConv, flags_match
    s = S1
    x, w = int8_tensors(s, 5353, 1, 100)
    g = GpuConv(s, variant)
    g.prepare(w)
    y0, f0 = g.run(x)                                  # generates xchk too
    clean = oracle.abed_int8(x, w, s)
    assert not f0.any()
    rng = np.random.default_rng(7)
    for site in ("x", "w", "wchk", "xchk"):
        for _ in range(3):
            t = {"x": g.x, "w": g.w, "wchk": g.wchk, "xchk": g.xchk}[site]
            idx, bit = int(rng.integers(0, t.numel())), int(rng.integers(0, 8))
            print("variant", variant, "site", site, idx, bit, flush=True)
            flip_dev(t, idx, bit)
            y, f = g.run(g.x, compute_xchk=False)
            arrs = dict(x=x.copy(), w=w.copy(), wchk=clean["wchk"].copy(), xchk=clean["xchk"].copy())
            oracle.flip_bit(arrs[site], idx, bit)
            ref = oracle.abed_int8(arrs["x"], arrs["w"], s, wchk=arrs["wchk"], xchk=arrs["xchk"])
            assert np.array_equal(y, ref["y"])
            assert flags_match(f, ref, s, g.lay)
            if site == "x":
                assert (f & 2).any() and not (f & 1).any()
            elif site == "w":
                assert (f & 1).any() and not (f & 2).any()
            else:
                assert np.array_equal(y, clean["y"]) and f.any()
            flip_dev(t, idx, bit)                       # restore
    y, f = g.run(g.x, compute_xchk=False)
    assert np.array_equal(y, clean["y"]) and not f.any()


@pytest.mark.parametrize("variant", [1, 2])
def test_stored_output_flip_seen_by_variants_that_reread(oracle, variant):
    from gpu_helpers import GpuConv, flags_match
    s = S1
    x, w = int8_tensors(s, 5454)
    g = GpuConv(s, variant); g.prepare(w)
    idx, bit = 4321, 17
    y, f = g.run(x, inject=(2, idx, bit))
    ref = oracle.abed_int8(x, w, s, stored_flip=(idx, bit), check_sees_stored=True)
    assert np.array_equal(y, ref["y"]) and flags_match(f, ref, s, g.lay) and (f & 3).any()


def test_stored_output_flip_after_fused_check_is_out_of_scope(oracle):
    """Corruption after the check completed is outside the method's coverage (Sec. 5.4)."""
    from gpu_helpers import GpuConv
    s = S1
    x, w = int8_tensors(s, 5454)
    g = GpuConv(s, 4); g.prepare(w)
    y, f = g.run(x, inject=(2, 4321, 17))
    ref = oracle.abed_int8(x, w, s, stored_flip=(4321, 17), check_sees_stored=False)
    assert np.array_equal(y, ref["y"]) and not f.any()


@pytest.mark.parametrize("variant", [3, 4])
def test_detection_rate_of_accumulator_flips(oracle, variant):
    """Every single-bit flip of an accumulator must be flagged (the target is 100 %), and a clean
    run must never be (0 false positives): 200 seeded flips on config 1."""
    from gpu_helpers import GpuConv
    s = CONFIG1[0]
    x, w = int8_tensors(s, 1000, -8, 7)
    g = GpuConv(s, variant); g.prepare(w)
    rng = np.random.default_rng(2024)
    detected = 0
    trials = 200
    for _ in range(trials):
        idx, bit = int(rng.integers(0, s.N * s.P * s.Q * s.K)), int(rng.integers(0, 32))
        _, f = g.run(x, inject=(1, idx, bit))
        pix = (idx // s.K) % (s.P * s.Q)
        fw = f.reshape(g.lay.grid_m, -1)
        hit = np.bitwise_or.reduce(fw, axis=1)
        if hit[pix // 16] & 3 == 3 and np.count_nonzero(hit) == 1:
            detected += 1
    assert detected == trials
    for seed in range(20):
        x2, w2 = int8_tensors(s, 7000 + seed, -8, 7)
        g.prepare(w2)
        _, f = g.run(x2)
        assert not f.any()
