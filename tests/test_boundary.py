"""Host-side tests of the C-ABI boundary that need no GPU: the library loads,
exports every symbol include/abed.h declares, validates arguments and reports
tile layouts consistently."""
import os
import re

import pytest

import paper_2006_04984_amd as abed
from paper_2006_04984_amd import ConvDesc, Variant, AbedError
from synth import CONFIG1, CONFIG2, CONFIG3, resnet50_layers

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(abed.lib_path()):
        from paper_2006_04984_amd import build
        build.build()
    return abed.lib()


def test_exports_match_header(L):
    text = open(os.path.join(ROOT, "include", "abed.h")).read()
    declared = set(re.findall(r"\b(abed_[a-z0-9_]+)\s*\(", text))
    assert declared, "no declarations found"
    for name in declared:
        assert hasattr(L, name), name
    from paper_2006_04984_amd.binding import EXPORTS
    assert declared == set(EXPORTS)


def test_status_strings(L):
    for s in range(6):
        assert L.abed_status_string(s)


@pytest.mark.parametrize("bad", [dict(N=0), dict(C=-1), dict(stride_h=0), dict(pad_w=-1), dict(R=40)])
def test_invalid_descriptor(L, bad):
    d = abed.desc_from_shape(CONFIG1[0])
    for k, v in bad.items():
        setattr(d, k, v)
    with pytest.raises(AbedError) as e:
        abed.get_layout(d)
    assert e.value.status == 1


def test_unsupported_descriptor(L):
    d = abed.desc_from_shape(CONFIG1[0])
    d.C = 17
    with pytest.raises(AbedError) as e:
        abed.get_layout(d)
    assert e.value.status == 2
    d = abed.desc_from_shape(CONFIG1[0])
    d.C, d.R, d.S = 4096, 5, 5                      # C*R*S > 64K: int32 accumulation no longer exact
    with pytest.raises(AbedError) as e:
        abed.get_layout(d)
    assert e.value.status == 2


def _other_shapes():
    """Shapes outside the configured networks: filter counts that are no powers of two (also beyond 257: three digit
    filters), single images and small batches, batches beyond 257 (three digit images), strides, full-HD-sized planes."""
    from synth import ConvShape
    return [ConvShape(1, 17, 23, 48, 40, 3, 3, 1, 1, 1, 1, "n1_k40"),
            ConvShape(8, 135, 240, 32, 24, 3, 3, 2, 2, 1, 1, "n8_fullhd_eighth_stride2_k24"),
            ConvShape(8, 68, 120, 96, 200, 1, 1, 1, 1, 0, 0, "n8_1x1_k200"),
            ConvShape(3, 9, 9, 16, 272, 3, 3, 1, 1, 1, 1, "n3_k272_three_digit_filters"),
            ConvShape(300, 7, 7, 64, 64, 3, 3, 1, 1, 1, 1, "n300_three_digit_images"),
            ConvShape(2, 540, 960, 16, 16, 3, 3, 1, 1, 1, 1, "n2_quarter_fullhd_plane"),
            ConvShape(5, 31, 31, 80, 112, 5, 5, 2, 2, 2, 2, "n5_5x5_stride2_k112")]


def _digits(count):
    return 1 if count <= 1 else 2 if count <= 257 else 3


@pytest.mark.parametrize("s", CONFIG1 + CONFIG2 + CONFIG3 + resnet50_layers(128)[1:] + _other_shapes(), ids=lambda s: s.name)
def test_layout_consistency(L, s):
    d = abed.desc_from_shape(s)
    for v in Variant:
        lay = abed.get_layout(d, 0, v)
        checked = 1 <= v <= 5
        entries = s.N + (lay.d_i if checked else 0)
        fblocks = (s.K + 15) // 16 + (1 if checked else 0)
        assert lay.tile_pixels == 16 and lay.tile_n % 16 == 0 and lay.tile_batch % 4 == 0
        assert lay.grid_m == (s.P * s.Q + 15) // 16
        assert lay.grid_b * lay.tile_batch >= entries > (lay.grid_b - 1) * lay.tile_batch
        assert lay.grid_n * lay.tile_n >= fblocks * 16 > (lay.grid_n - 1) * lay.tile_n
        assert lay.n_flag_words == lay.grid_m * lay.grid_b * lay.grid_n
        assert lay.d_f == _digits(s.K) and lay.d_i == _digits(s.N)
        assert lay.wchk_bytes == lay.d_f * s.R * s.S * s.C
        assert lay.xchk_bytes == lay.d_i * s.H * s.W * s.C


@pytest.mark.parametrize("s", CONFIG1 + CONFIG2, ids=lambda s: s.name)
def test_layout_of_one_scheme_alone(L, s):
    """FC alone has no checksum images, IC alone no checksum filter block (Sec. 3.1 / 3.2, Table 1)."""
    d = abed.desc_from_shape(s)
    both = abed.get_layout(d, 0, 4)
    fc = abed.get_layout(d, 0, 4 | abed.ONLY_FC)
    ic = abed.get_layout(d, 0, 4 | abed.ONLY_IC)
    assert (fc.d_f, fc.d_i) == (both.d_f, 0) and fc.xchk_bytes == 0 and fc.wchk_bytes == both.wchk_bytes
    assert (ic.d_f, ic.d_i) == (0, both.d_i) and ic.wchk_bytes == 0 and ic.xchk_bytes == both.xchk_bytes
    assert fc.grid_b * fc.tile_batch >= s.N > (fc.grid_b - 1) * fc.tile_batch
    assert fc.grid_n * fc.tile_n >= ((s.K + 15) // 16 + 1) * 16 > (fc.grid_n - 1) * fc.tile_n
    assert ic.grid_b * ic.tile_batch >= s.N + ic.d_i > (ic.grid_b - 1) * ic.tile_batch
    assert ic.grid_n * ic.tile_n >= (s.K + 15) // 16 * 16 > (ic.grid_n - 1) * ic.tile_n


def test_scheme_selection_errors(L):
    d = abed.desc_from_shape(CONFIG1[0])
    for v in (0 | abed.ONLY_FC, 6 | abed.ONLY_IC, 4 | abed.ONLY_FC | abed.ONLY_IC, 5 | abed.ONLY_FC, 4 | 0x2000,
              4 | abed.PACKED_FC | abed.ONLY_IC, 3 | abed.PACKED_FC):
        with pytest.raises(AbedError) as e:
            abed.get_layout(d, 0, v)
        assert e.value.status == 1


def test_packed_checksum_filters_layout(L):
    """Checksum filters in the free rows of the last block of 16 filters (Sec. 6.2, reserved space):
    one filter block fewer than the plain layout when there is room, unsupported when there is not."""
    from synth import ConvShape
    for K, ok in ((60, True), (62, True), (63, False), (64, False), (13, True), (15, False), (77, True)):
        d = abed.desc_from_shape(ConvShape(8, 6, 6, 16, K, 3, 3, 1, 1, 1, 1))
        if not ok:
            with pytest.raises(AbedError) as e:
                abed.get_layout(d, 0, 4 | abed.PACKED_FC)
            assert e.value.status == 2
            continue
        plain = abed.get_layout(d, 0, 4)
        packed = abed.get_layout(d, 0, 4 | abed.PACKED_FC)
        assert packed.d_f == plain.d_f and packed.wchk_bytes == plain.wchk_bytes
        assert packed.grid_n * packed.tile_n >= (K + 15) // 16 * 16 > (packed.grid_n - 1) * packed.tile_n
        assert packed.grid_n * packed.tile_n <= plain.grid_n * plain.tile_n


def test_tensor_size_limits_are_in_bytes(L):
    """Offsets inside a tensor are 32-bit byte offsets: 2^30 fp16 elements are too many, 2^30 int8 elements are not."""
    from synth import ConvShape
    d = abed.desc_from_shape(ConvShape(1024, 64, 64, 256, 16, 1, 1, 1, 1, 0, 0))
    assert abed.get_layout(d, 0, 0).grid_m == 256
    with pytest.raises(AbedError) as e:
        abed.get_layout(d, 1, 0)
    assert e.value.status == 2


def test_fic_inloop_layout_and_limits(L):
    """Host logic of the in-loop FIC option: digit buffer size, workspace carving, range limits."""
    import dataclasses
    for s in list(CONFIG2) + [l for l in resnet50_layers(128) if l.C % 16 == 0][:20]:
        d = abed.desc_from_shape(s)
        lay = abed.fic_inloop_get_layout(d)
        crs = s.R * s.S * s.C
        assert lay.wdig_bytes == 3 * 64 * ((crs + 63) // 64)
        plain = abed.get_layout(d, 0, 0)
        tiles, rows = plain.grid_m * plain.grid_b * plain.grid_n, plain.grid_m * plain.grid_b
        align = lambda v: (v + 255) // 256 * 256
        assert lay.workspace_bytes == 256 + align(8 * tiles) + align(8 * rows)
    s = CONFIG2[0]
    with pytest.raises(AbedError) as e:      # the digits of a reduction axis of 9216 do not fit beside the tile
        abed.fic_inloop_get_layout(abed.desc_from_shape(dataclasses.replace(s, C=1024)))
    assert e.value.status == 2
    with pytest.raises(AbedError) as e:      # three digits hold the filter checksum up to K = 32768
        abed.fic_inloop_get_layout(abed.desc_from_shape(dataclasses.replace(s, K=32768 + 16)))
    assert e.value.status in (2, 5)      # the tile plan may refuse such a filter count first


def test_tile_plan_rules(L):
    """The tile plan for shapes the rules were measured on (entries per tile, filters per tile)."""
    from synth import ConvShape

    def tile(shape, variant):
        lay = abed.get_layout(abed.desc_from_shape(ConvShape(*shape, "plan")), 0, variant)
        return lay.tile_batch, lay.tile_n

    FC, IC = abed.ONLY_FC, abed.ONLY_IC
    # the benchmark's layers at N = 32: checked and unchecked
    assert [tile(tuple(getattr(s, f) for f in ("N", "H", "W", "C", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w")), 4)
            for s in CONFIG2] == [(12, 80), (8, 80), (12, 64), (8, 64)]
    assert [tile(tuple(getattr(s, f) for f in ("N", "H", "W", "C", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w")), 0)
            for s in CONFIG2] == [(8, 64), (8, 64), (8, 64), (4, 64)]
    # 256 filters + the digit block: 9-wide tiles for the filter checksum alone on a long reduction axis, not with both schemes
    s = (128, 14, 14, 256, 256, 3, 3, 1, 1, 1, 1)
    assert tile(s, 4 | FC) == (8, 144) and tile(s, 4) == (12, 64) and tile(s, 0) == (8, 128)
    # ... and not at N = 32 (too few tiles)
    assert tile((32, 14, 14, 256, 256, 3, 3, 1, 1, 1, 1), 4 | FC)[1] == 64
    # 128 filters + the digit block = 9 blocks: one filter tile for the filter checksum alone from 384 tiles on
    assert tile((64, 28, 28, 512, 128, 1, 1, 1, 1, 0, 0), 4 | FC) == (8, 144)
    assert tile((32, 28, 28, 128, 128, 3, 3, 1, 1, 1, 1), 4 | FC) == (8, 80)
    # 512 filters at 7x7 with 128 images: 8-wide tiles for the plain problem from 256 tiles on (long reduction axis),
    # 5-wide tiles (33 blocks in 7 tiles) with both schemes, 4-wide for the batch checksum alone
    s = (128, 7, 7, 512, 512, 3, 3, 1, 1, 1, 1)
    assert tile(s, 0) == (8, 128) and tile(s, 4) == (8, 80) and tile(s, 4 | IC) == (8, 64)
    # a plain problem on a small grid takes the largest tile that still gives every CU a workgroup
    assert tile((64, 7, 7, 2048, 512, 1, 1, 1, 1, 0, 0), 0) == (8, 64)


def test_static_scratch_entry_point_rejects_large_workspace(L):
    """abed_conv_int8_static refuses, before anything touches a GPU, a convolution whose layout needs more
    scratch than the library's array holds (the pointers are never used: the call must return first)."""
    from synth.shapes import ConvShape
    s = ConvShape(64, 56, 56, 64, 256, 1, 1, 1, 1, 0, 0, "too_big")
    desc = abed.desc_from_shape(s)
    lay = abed.get_layout(desc, 0, Variant.UNFUSED)
    assert lay.workspace_bytes > 16 << 20
    import ctypes
    st = L.abed_conv_int8_static(ctypes.byref(desc), None, None, None, None, 1, None, None, int(Variant.UNFUSED),
                                 None, None, None, None, None)
    assert st == 3


def test_abft_gemm_layout(L):
    """Host logic of the traditional ABFT-GEMM baseline: digits, padded sizes, limits."""
    lay = abed.abft_gemm_get_layout(100352, 64, 576)
    assert (lay.d_a, lay.d_b) == (4, 2) and lay.ld_c == 68 and lay.rows_padded == 100608
    assert lay.workspace_bytes >= 100608 * 576 + 68 * 576 + 100608 * 68 * 4
    lay = abed.abft_gemm_get_layout(70, 40, 32)
    assert (lay.d_a, lay.d_b, lay.ld_c, lay.rows_padded) == (2, 2, 44, 256)
    for bad, status in (((0, 4, 16), 1), ((4, 4, 24), 2), ((4, 4, 65536 + 16), 2)):
        with pytest.raises(AbedError) as e:
            abed.abft_gemm_get_layout(*bad)
        assert e.value.status == status
