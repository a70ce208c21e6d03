"""The analytic operation / byte model (Sec. 5.1): closed forms on a layer whose counts can be done by hand,
and the orders of magnitude the paper reports for its networks (Sec. 6.1: FC adds a few percent of
operations, FIC under one or two percent; fused options move far fewer bytes than unfused ones)."""
from paper_2006_04984_amd import model
from synth import ConvShape, CONFIG2, resnet50_layers


def test_hand_counted_layer():
    s = ConvShape(2, 4, 4, 16, 8, 3, 3, 1, 1, 1, 1)        # P = Q = 4, 32 output pixels, C*R*S = 144
    o = model.ops(s)
    assert o["baseline"]["convolution"] == 2 * 16 * 8 * 144 and o["baseline"]["epilog"] == 5 * 2 * 16 * 8
    assert o["fc"]["convolution"] == 2 * 16 * (8 + 2) * 144            # two digit filters for K = 8
    assert o["fc"]["output_checksum"] == 32 * 7 + 32 * 2 and o["fc"]["verification"] == 32
    assert o["fic"]["input_checksum"] == 32 * 144 and o["fic"]["dot_product"] == 144 and o["fic"]["output_checksum"] == 32 * 8
    assert o["ic2"]["checksum_convolution"] == 144 * 8 and o["ic2"]["verification"] == 8
    b = model.moved_bytes(s)
    x, w, outs = 2 * 4 * 4 * 16, 8 * 144, 32 * 8
    assert b["baseline_fused"] == x + w + outs
    assert b["baseline_unfused"] == x + w + 4 * outs + 4 * outs + outs
    assert b["fic_fused"] == b["baseline_fused"] + x + 4 * 144 + 4 * 144 + 16


def test_orders_of_magnitude():
    layers = resnet50_layers(128)[1:]
    tot = {}
    for s in layers:
        for k, v in model.ops(s).items():
            tot[k] = tot.get(k, 0) + sum(v.values())
    inc = {k: v / tot["baseline"] - 1.0 for k, v in tot.items()}
    assert 0.0 < inc["fic"] < 0.02 and inc["fic"] < inc["fc"] < 0.07
    assert inc["fc"] < inc["fc_granule"]
    for s in CONFIG2:
        b = model.moved_bytes(s)
        assert b["fc_fused"] < b["fic_fused"] < b["baseline_unfused"] < b["fic_unfused"] and b["fc_unfused"] > b["baseline_unfused"]
