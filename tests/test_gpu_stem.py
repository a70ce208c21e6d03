"""GPU parity for the channel-padding helper: the 3-channel first layer through the checked convolution."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_three_channel_stem_padded_by_the_library(oracle):
    """The 3-channel first layer (7x7, stride 2): channels padded to 16 with abed_pad_channels, outputs and flags
    those of the oracle on the unpadded layer (zero channels add nothing to the convolution or the checksums)."""
    import dataclasses
    import torch
    import paper_2006_04984_amd as abed
    from synth import ConvShape, int8_tensors
    from gpu_helpers import GpuConv, flags_match, to_dev
    s3 = ConvShape(6, 40, 36, 3, 64, 7, 7, 2, 2, 3, 3, "stem_small")
    s16 = dataclasses.replace(s3, C=16)
    x, w = int8_tensors(s3, 3131)
    xp = torch.full((s3.N, s3.H, s3.W, 16), 77, dtype=torch.int8, device="cuda:0")
    wp = torch.full((s3.K, s3.R, s3.S, 16), 77, dtype=torch.int8, device="cuda:0")
    abed.pad_channels(to_dev(x), xp, 3, 16)
    abed.pad_channels(to_dev(w), wp, 3, 16)
    assert torch.equal(xp[..., :3].cpu(), torch.from_numpy(x)) and not xp[..., 3:].any()
    assert torch.equal(wp[..., :3].cpu(), torch.from_numpy(w)) and not wp[..., 3:].any()
    for variant in (0, 4):
        g = GpuConv(s16, variant)
        g.prepare(wp)
        ref = oracle.abed_int8(x, w, s3)
        y, flags = g.run(xp)
        assert np.array_equal(y, ref["y"])
        if variant == 4:
            assert not flags.any()
            idx = 12345
            bad = oracle.abed_int8(x, w, s3, acc_flip=(idx, 30))
            y2, f2 = g.run(xp, inject=(1, idx, 30))
            assert np.array_equal(y2, bad["y"]) and flags_match(f2, bad, s16, g.lay)
