"""Pins for the int8 oracle: each test checks it against something other than
itself (brute force in a different formulation, a library routine, a closed
form, an algebraic invariant the paper relies on, or a hand-worked fixture)."""
import os

import numpy as np
import pytest
import torch

from synth import ConvShape, CONFIG1, int8_tensors, ones_tensors

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

# shapes with every pair of like parameters different, so that a transposed
# operand or swapped index cannot go unnoticed
ASYM = [
    ConvShape(3, 6, 5, 4, 5, 3, 2, 1, 1, 1, 0, "asym_a"),
    ConvShape(2, 7, 9, 3, 4, 2, 3, 2, 1, 0, 2, "asym_b"),
    ConvShape(2, 8, 6, 2, 3, 3, 3, 2, 2, 1, 1, "stride2"),
    ConvShape(1, 5, 5, 4, 6, 1, 1, 1, 1, 0, 0, "1x1"),
    ConvShape(2, 9, 9, 2, 2, 7, 7, 2, 2, 3, 3, "7x7s2"),
    ConvShape(3, 4, 4, 1, 1, 3, 3, 1, 1, 2, 2, "pad2"),
]


def brute_force(x, w, s):
    """Sec. 2.2 in a different formulation from the oracle's C loops: pad the
    image explicitly, cut each window out and take its dot product in Python."""
    xp = np.zeros((s.N, s.H + 2 * s.pad_h, s.W + 2 * s.pad_w, s.C), dtype=np.int64)
    xp[:, s.pad_h:s.pad_h + s.H, s.pad_w:s.pad_w + s.W, :] = x
    y = np.zeros((s.N, s.P, s.Q, s.K), dtype=np.int64)
    for n in range(s.N):
        for p in range(s.P):
            for q in range(s.Q):
                win = xp[n, p * s.stride_h:p * s.stride_h + s.R, q * s.stride_w:q * s.stride_w + s.S, :]
                for k in range(s.K):
                    y[n, p, q, k] = int((win * w[k].astype(np.int64)).sum())
    return y


def torch_conv(x, w, s, dtype=torch.int64):
    xt = torch.from_numpy(np.ascontiguousarray(x)).to(dtype).permute(0, 3, 1, 2)
    wt = torch.from_numpy(np.ascontiguousarray(w)).to(dtype).permute(0, 3, 1, 2)
    yt = torch.nn.functional.conv2d(xt, wt, stride=(s.stride_h, s.stride_w), padding=(s.pad_h, s.pad_w))
    return yt.permute(0, 2, 3, 1).contiguous().numpy()


@pytest.mark.parametrize("s", ASYM, ids=lambda s: s.name)
def test_conv_brute_force(oracle, s):
    x, w = int8_tensors(s, 11)
    assert np.array_equal(oracle.conv_int(x, w, s), brute_force(x, w, s))


@pytest.mark.parametrize("s", ASYM + CONFIG1, ids=lambda s: s.name)
def test_conv_vs_torch_int64(oracle, s):
    x, w = int8_tensors(s, 12)
    assert np.array_equal(oracle.conv_int(x, w, s), torch_conv(x, w, s))


def test_conv_1x1_is_matmul(oracle):
    s = ConvShape(3, 5, 4, 7, 6, 1, 1, 1, 1, 0, 0)
    x, w = int8_tensors(s, 13)
    ref = x.reshape(-1, s.C).astype(np.int64) @ w.reshape(s.K, s.C).astype(np.int64).T
    assert np.array_equal(oracle.conv_int(x, w, s).reshape(-1, s.K), ref)


def test_conv_points_match_full(oracle):
    s = ASYM[1]
    x, w = int8_tensors(s, 14)
    y = oracle.conv_int(x, w, s)
    g = np.random.default_rng(0)
    pts = np.stack([g.integers(0, d, 50) for d in (s.N, s.P, s.Q, s.K)], axis=1)
    assert np.array_equal(oracle.conv_int_points(x, w, s, pts), y[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]])


def test_all_ones_closed_form(oracle):
    """Fixture worked by hand from Sec. 2.2 / 3.1 / 3.2 for all-ones tensors."""
    s = ConvShape(3, 4, 5, 2, 5, 3, 3, 1, 1, 1, 1)
    exp = np.loadtxt(os.path.join(GOLDEN, "ones_3x3_pad1.txt"), dtype=np.int64)
    x, w = ones_tensors(s)
    r = oracle.abed_int8(x, w, s)
    for n in range(s.N):
        for k in range(s.K):
            assert np.array_equal(r["y"][n, :, :, k], exp)
    assert np.array_equal(r["yf"], np.broadcast_to(s.K * exp, (s.N, s.P, s.Q)))
    assert np.array_equal(r["yi"], np.broadcast_to((s.N * exp)[:, :, None], (s.P, s.Q, s.K)))
    assert np.array_equal(r["yfi"], s.N * s.K * exp)
    assert not r["fc_bad"].any() and not r["ic_bad"].any() and not r["corner_bad"].any()


@pytest.mark.parametrize("s", ASYM + CONFIG1, ids=lambda s: s.name)
def test_linearity_invariants_clean(oracle, s):
    """sum_k y = conv(x, sum_k w) and sum_n y = conv(sum_n x, w)  (Sec. 3):
    the extra fmaps are computed here by the library routine, not by the oracle."""
    x, w = int8_tensors(s, 15)
    r = oracle.abed_int8(x, w, s)
    wsum = w.astype(np.int64).sum(0, keepdims=True)
    xsum = x.astype(np.int64).sum(0, keepdims=True)
    assert np.array_equal(r["yf"], torch_conv(x, wsum, s)[..., 0])
    assert np.array_equal(r["yi"], torch_conv(xsum, w, s)[0])
    assert np.array_equal(r["yfi"], torch_conv(xsum, wsum, s)[0, :, :, 0])
    assert np.array_equal(r["rs"], r["yf"]) and np.array_equal(r["cs"], r["yi"])
    assert not (r["fc_bad"].any() or r["ic_bad"].any() or r["corner_bad"].any())


def test_digits_round_trip_and_range(oracle):
    g = np.random.default_rng(3)
    for count, nd in [(1, 1), (2, 2), (32, 2), (256, 2), (257, 2), (258, 3), (2048, 3), (65536, 3), (70000, 4)]:
        assert oracle.num_digits_for_count(count) == nd, count
        lo, hi = -128 * count, 127 * count
        s = np.concatenate([g.integers(lo, hi + 1, 1000), np.clip([lo, hi, 0, -1, 1, 127, 128, -128, -129], lo, hi)])
        d = oracle.split_digits(s, nd)
        assert d.dtype == np.int8 and d.shape == (nd, len(s))
        # recombination written out independently of recombine_digits
        back = sum(int(256 ** i) * d[i].astype(object) for i in range(nd))
        assert all(int(a) == int(b) for a, b in zip(back, s))
        assert np.array_equal(oracle.recombine_digits(list(d)), s)
    with pytest.raises(OverflowError):
        oracle.split_digits(np.array([40000]), 2)


def test_bit_budget(oracle):
    """Sec. 4.1: an int8 convolution output needs at most 16 + log2(CRS) bits
    (int32 suffices for CRS <= 64K); the filter checksum 8 + log2(K) bits."""
    s = ConvShape(1, 3, 3, 64, 300, 3, 3, 1, 1, 1, 1)
    x = np.full((1, 3, 3, 64), -128, dtype=np.int8)
    w = np.full((300, 3, 3, 64), -128, dtype=np.int8)
    y = oracle.conv_int(x, w, s)
    crs = s.C * s.R * s.S
    assert y.max() == 128 * 128 * crs and y.max() < 2 ** (16 + int(np.ceil(np.log2(crs))))
    wsum = oracle.filter_checksum(w)
    assert wsum.min() == -128 * 300 and abs(wsum.min()) <= 2 ** (8 + int(np.ceil(np.log2(300))) - 1)


def test_wrap32_is_mod_2_32(oracle):
    v = np.array([0, 1, -1, 2 ** 31 - 1, 2 ** 31, 2 ** 32, 2 ** 32 + 5, -2 ** 31, -2 ** 31 - 1, 3 * 2 ** 40 + 7], dtype=np.int64)
    w = oracle.wrap32(v)
    assert w.dtype == np.int32
    for a, b in zip(v, w):
        assert (int(a) - int(b)) % (2 ** 32) == 0 and -2 ** 31 <= int(b) < 2 ** 31


def test_wrapped_checks_hold_when_sums_overflow_int32(oracle):
    """The reduced sums may exceed 32 bits; compared mod 2^32 the identities still hold
    (modular arithmetic, end of Sec. 4.1)."""
    s = ConvShape(4, 3, 3, 256, 64, 3, 3, 1, 1, 1, 1)
    x = np.full((s.N, s.H, s.W, s.C), 127, dtype=np.int8)
    w = np.full((s.K, s.R, s.S, s.C), 127, dtype=np.int8)
    r = oracle.abed_int8(x, w, s)
    assert r["y_exact"].sum(axis=3).max() > 2 ** 31          # the row sum really overflows int32
    assert not (r["fc_bad"].any() or r["ic_bad"].any() or r["corner_bad"].any())


def test_scalar_identity_of_fic(oracle):
    """Sec. 3.3: the sum of all outputs equals the dot product of the filter checksum
    with the input patch-sum checksum (Sec. 3.2, option 2)."""
    s = ASYM[2]
    x, w = int8_tensors(s, 16)
    y = oracle.conv_int(x, w, s)
    xp = np.zeros((s.N, s.H + 2 * s.pad_h, s.W + 2 * s.pad_w, s.C), dtype=np.int64)
    xp[:, s.pad_h:s.pad_h + s.H, s.pad_w:s.pad_w + s.W] = x
    patch = np.zeros((s.R, s.S, s.C), dtype=np.int64)
    for r in range(s.R):
        for c in range(s.S):
            patch[r, c] = xp[:, r:r + (s.P - 1) * s.stride_h + 1:s.stride_h,
                             c:c + (s.Q - 1) * s.stride_w + 1:s.stride_w].sum(axis=(0, 1, 2))
    assert int(y.sum()) == int((patch * oracle.filter_checksum(w)).sum())


def test_single_bit_flip_in_accumulator_is_localised(oracle):
    """An accumulator flip changes one row sum and one column sum by +-2^b != 0 mod 2^32."""
    s = CONFIG1[0]
    x, w = int8_tensors(s, 1000, -8, 7)
    g = np.random.default_rng(5)
    for _ in range(8):
        n, p, q, k = (int(g.integers(0, d)) for d in (s.N, s.P, s.Q, s.K))
        bit = int(g.integers(0, 32))
        idx = ((n * s.P + p) * s.Q + q) * s.K + k
        r = oracle.abed_int8(x, w, s, acc_flip=(idx, bit))
        clean = oracle.abed_int8(x, w, s)
        assert (r["y"] != clean["y"]).sum() == 1
        fc = np.zeros_like(r["fc_bad"]); fc[n, p, q] = True
        ic = np.zeros_like(r["ic_bad"]); ic[p, q, k] = True
        assert np.array_equal(r["fc_bad"], fc) and np.array_equal(r["ic_bad"], ic)
        assert not r["corner_bad"].any()


def test_stored_flip_seen_only_by_variants_that_reread(oracle):
    s = ASYM[0]
    x, w = int8_tensors(s, 17)
    r1 = oracle.abed_int8(x, w, s, stored_flip=(7, 3), check_sees_stored=True)
    r2 = oracle.abed_int8(x, w, s, stored_flip=(7, 3), check_sees_stored=False)
    assert np.array_equal(r1["y"], r2["y"])
    assert r1["fc_bad"].sum() == 1 and r1["ic_bad"].sum() == 1
    assert not r2["fc_bad"].any() and not r2["ic_bad"].any()


def test_coverage_matrix(oracle):
    """Table 1 / Sec. 5.4 error injections: FC alone is blind to input-fmap flips and
    catches filter flips; IC alone is blind to filter flips and catches input flips."""
    s = ConvShape(4, 6, 6, 4, 8, 3, 3, 1, 1, 1, 1)
    x, w = int8_tensors(s, 18, 1, 100)     # non-zero data so that every flip changes outputs
    clean = oracle.abed_int8(x, w, s)
    # input flip after both checksums were generated
    x2 = x.copy(); oracle.flip_bit(x2, 77, 6)
    r = oracle.abed_int8(x2, w, s, wchk=clean["wchk"], xchk=clean["xchk"])
    assert (r["y"] != clean["y"]).any()
    assert not r["fc_bad"].any() and r["ic_bad"].any()
    # filter flip after the filter checksum was generated
    w2 = w.copy(); oracle.flip_bit(w2, 50, 2)
    r = oracle.abed_int8(x, w2, s, wchk=clean["wchk"], xchk=clean["xchk"])
    assert (r["y"] != clean["y"]).any()
    assert r["fc_bad"].any() and not r["ic_bad"].any()
    # flips in the checksum data themselves: outputs stay clean, a check fires (Sec. 6.4:
    # errors detected with no output corruption point at the verification path)
    wc = clean["wchk"].copy(); oracle.flip_bit(wc, 5, 1)
    r = oracle.abed_int8(x, w, s, wchk=wc, xchk=clean["xchk"])
    assert np.array_equal(r["y"], clean["y"]) and r["fc_bad"].any() and not r["ic_bad"].any() and r["corner_bad"].any()
    xc = clean["xchk"].copy(); oracle.flip_bit(xc, 9, 0)
    r = oracle.abed_int8(x, w, s, wchk=clean["wchk"], xchk=xc)
    assert np.array_equal(r["y"], clean["y"]) and r["ic_bad"].any() and not r["fc_bad"].any() and r["corner_bad"].any()


def test_epilog_hand_cases(oracle):
    rows = np.loadtxt(os.path.join(GOLDEN, "epilog_cases.txt"))
    for acc, scale, bias, relu, exp in rows:
        got = oracle.epilog_int8(np.array([int(acc)], dtype=np.int32), np.array([scale], dtype=np.float32),
                                 np.array([bias], dtype=np.float32), bool(relu))
        assert got.dtype == np.int8 and int(got[0]) == int(exp), (acc, scale, bias, relu, got, exp)


def test_epilog_and_next_checksum(oracle):
    s = ConvShape(4, 5, 5, 16, 8, 3, 3, 1, 1, 1, 1)
    x, w = int8_tensors(s, 19)
    scale = np.linspace(1e-3, 3e-3, s.K).astype(np.float32)
    bias = np.linspace(-2, 2, s.K).astype(np.float32)
    r = oracle.abed_int8(x, w, s, epilog=(scale, bias, True))
    # independent evaluation in double precision: away from rounding ties the results agree
    t = r["y"].astype(np.float64) * scale.astype(np.float64) + bias.astype(np.float64)
    t = np.maximum(t, 0)
    near_tie = np.abs(t - np.floor(t) - 0.5) < 1e-3
    ref = np.clip(np.rint(t), -128, 127)
    assert np.array_equal(r["out8"][~near_tie], ref[~near_tie].astype(np.int8))
    assert r["out8"].min() >= 0 and r["out8"].max() > 20
    assert np.array_equal(r["xsum_next"], r["out8"].astype(np.int64).sum(0))
    assert np.array_equal(oracle.recombine_digits(list(r["xchk_next"])), r["xsum_next"])
