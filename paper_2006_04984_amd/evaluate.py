"""Evaluation runs on one GPU, beside bench.py (which covers the headline 3x3 configuration):

  python -m paper_2006_04984_amd.evaluate layers   --config 3      per-layer table of a configuration
  python -m paper_2006_04984_amd.evaluate abft                      the traditional ABFT-GEMM baseline, task by task (Sec. 5.3)
  python -m paper_2006_04984_amd.evaluate fp16                      false-positive / detection rates (fp16 layer)
  python -m paper_2006_04984_amd.evaluate detect                    int8 single-bit detection rates
  python -m paper_2006_04984_amd.evaluate resnet50 --batch 128      the 53 convolution layers back to back
  python -m paper_2006_04984_amd.evaluate ksweep                    filter-count sweep on one 3x3 layer

All inputs are seeded and synthetic (synth/).  Each command prints one JSON object.
Times are GPU times of HIP-graph replays measured with events on the launch stream.
"""
import argparse
import json
import sys

import numpy as np
import torch

from . import binding as abed
from .binding import Variant

DEV = "cuda:0"
PEAK_HBM_GBS = 8000.0


def _graph_time(fn, stream, reps=20, replays=10):
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(stream):
        fn()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            for _ in range(reps):
                fn()
        g.replay()
        torch.cuda.synchronize()
        e0.record(stream)
        for _ in range(replays):
            g.replay()
        e1.record(stream)
        torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / (reps * replays)


class Int8Layer:
    """Device buffers of one int8 convolution and a call closure per variant."""

    def __init__(self, s, seed, variant, epilogue=False, x=None):
        from synth import int8_tensors, requant_params
        self.s, self.variant = s, int(variant)           # may carry abed.ONLY_FC / abed.ONLY_IC
        self.desc = abed.desc_from_shape(s)
        self.lay = abed.get_layout(self.desc, 0, self.variant)
        xh, wh = int8_tensors(s, seed)
        self.x = torch.from_numpy(xh).to(DEV) if x is None else x
        self.w = torch.from_numpy(wh).to(DEV)
        self.y = torch.empty((s.N, s.P, s.Q, s.K), dtype=torch.int8 if epilogue else torch.int32, device=DEV)
        self.y2 = torch.empty_like(self.y) if self.variant == int(Variant.DUPLICATE) else None
        self.flags = torch.zeros((max(1, self.lay.n_flag_words),), dtype=torch.int32, device=DEV)
        self.ws = torch.zeros((max(256, self.lay.workspace_bytes),), dtype=torch.uint8, device=DEV)
        local = bool(self.lay.local_checksums)                # checksum filters per filter tile, no checksum images
        self.wchk = torch.empty((self.lay.d_f * (self.lay.grid_n if local else 1), s.R, s.S, s.C), dtype=torch.int8, device=DEV)
        self.xchk = torch.empty((0 if local else self.lay.d_i, s.H, s.W, s.C), dtype=torch.int8, device=DEV)
        self.xchk_next = torch.empty((self.lay.d_i, s.P, s.Q, s.K), dtype=torch.int8, device=DEV) if epilogue else None
        self.epi = None
        if epilogue:
            sc, bi = requant_params(s, seed)
            self.scale, self.bias = torch.from_numpy(sc).to(DEV), torch.from_numpy(bi).to(DEV)
            self.epi = (self.scale, self.bias, True)
        abed.workspace_init(self.ws)
        if self.variant & abed.PACKED_FC:                 # filters and checksum filters in one buffer
            both = torch.empty((s.K + self.lay.d_f, s.R, s.S, s.C), dtype=torch.int8, device=DEV)
            both[: s.K].copy_(self.w)
            self.w, self.wchk = both[: s.K], both[s.K:]
        if self.lay.d_f:
            abed.filter_prepare_local_int8(self.desc, self.variant, self.w, self.wchk)

    def run(self, compute_xchk=True, inject=None):
        abed.conv_int8(self.desc, self.x, self.w, self.wchk, self.xchk, compute_xchk, self.y, self.variant,
                       flags=self.flags, epilogue=self.epi, xchk_next=self.xchk_next, workspace=self.ws,
                       inject=inject, y2=self.y2)


class FicLayer:
    """Device buffers of one int8 convolution checked by the FIC scheme (Sec. 3.3)."""

    def __init__(self, s, seed, variant, epilogue=False, x=None):
        from synth import int8_tensors, requant_params
        self.s, self.variant = s, Variant(variant)
        self.desc = abed.desc_from_shape(s)
        lay = abed.fic_get_layout(self.desc, self.variant)
        xh, wh = int8_tensors(s, seed)
        self.x = torch.from_numpy(xh).to(DEV) if x is None else x
        self.xsum_in = self.xsum_next = None
        self.w = torch.from_numpy(wh).to(DEV)
        self.y = torch.empty((s.N, s.P, s.Q, s.K), dtype=torch.int8 if epilogue else torch.int32, device=DEV)
        self.wsum = torch.empty((s.R, s.S, s.C), dtype=torch.int32, device=DEV)
        self.xrows = torch.empty((lay.xrows_parts, s.H, s.S, s.C), dtype=torch.int32, device=DEV)
        self.result = torch.zeros((2,), dtype=torch.int64, device=DEV)
        self.flag = torch.zeros((1,), dtype=torch.int32, device=DEV)
        self.ws = torch.zeros((max(256, lay.workspace_bytes),), dtype=torch.uint8, device=DEV)
        self.epi = None
        if epilogue:
            sc, bi = requant_params(s, seed)
            self.scale, self.bias = torch.from_numpy(sc).to(DEV), torch.from_numpy(bi).to(DEV)
            self.epi = (self.scale, self.bias, True)
        abed.fic_filter_prepare_int8(self.desc, self.w, self.wsum)

    def run(self):
        abed.fic_conv_int8(self.desc, self.x, self.w, self.wsum, self.xrows, True, self.y, self.variant, self.result,
                           self.flag, epilogue=self.epi, workspace=self.ws, xsum_in=self.xsum_in, xsum_next=self.xsum_next)


class FicInloopLayer:
    """Device buffers of one int8 convolution checked by FIC with the input side formed in the main loop."""

    def __init__(self, s, seed, epilogue=False, x=None):
        from synth import int8_tensors, requant_params
        self.s, self.variant = s, abed.FIC_INLOOP
        self.desc = abed.desc_from_shape(s)
        lay = abed.fic_inloop_get_layout(self.desc)
        xh, wh = int8_tensors(s, seed)
        self.x = torch.from_numpy(xh).to(DEV) if x is None else x
        self.w = torch.from_numpy(wh).to(DEV)
        self.y = torch.empty((s.N, s.P, s.Q, s.K), dtype=torch.int8 if epilogue else torch.int32, device=DEV)
        self.wdig = torch.empty((lay.wdig_bytes,), dtype=torch.int8, device=DEV)
        self.result = torch.zeros((2,), dtype=torch.int64, device=DEV)
        self.flag = torch.zeros((1,), dtype=torch.int32, device=DEV)
        self.ws = torch.zeros((max(256, lay.workspace_bytes),), dtype=torch.uint8, device=DEV)
        self.epi = None
        if epilogue:
            sc, bi = requant_params(s, seed)
            self.scale, self.bias = torch.from_numpy(sc).to(DEV), torch.from_numpy(bi).to(DEV)
            self.epi = (self.scale, self.bias, True)
        abed.fic_inloop_filter_prepare_int8(self.desc, self.w, self.wdig)

    def run(self, deferred=False, inject=None):
        abed.fic_inloop_conv_int8(self.desc, self.x, self.w, self.wdig, self.y, None if deferred else self.result,
                                  None if deferred else self.flag, epilogue=self.epi, workspace=self.ws, inject=inject)


class Ic2Layer:
    """Device buffers of one int8 convolution checked by IC option 2 (Sec. 3.2)."""

    def __init__(self, s, seed, variant, epilogue=False):
        from synth import int8_tensors, requant_params
        self.s, self.variant = s, Variant(variant)
        self.desc = abed.desc_from_shape(s)
        lay = abed.ic2_get_layout(self.desc, self.variant)
        xh, wh = int8_tensors(s, seed)
        self.x, self.w = torch.from_numpy(xh).to(DEV), torch.from_numpy(wh).to(DEV)
        self.y = torch.empty((s.N, s.P, s.Q, s.K), dtype=torch.int8 if epilogue else torch.int32, device=DEV)
        self.xrows = torch.empty((lay.xrows_parts, s.H, s.S, s.C), dtype=torch.int32, device=DEV)
        self.result = torch.zeros((2, s.K), dtype=torch.int64, device=DEV)
        self.flags = torch.zeros((s.K,), dtype=torch.int32, device=DEV)
        self.ws = torch.zeros((max(256, lay.workspace_bytes),), dtype=torch.uint8, device=DEV)
        self.epi = None
        if epilogue:
            sc, bi = requant_params(s, seed)
            self.scale, self.bias = torch.from_numpy(sc).to(DEV), torch.from_numpy(bi).to(DEV)
            self.epi = (self.scale, self.bias, True)

    def run(self):
        abed.ic2_conv_int8(self.desc, self.x, self.w, self.xrows, True, self.y, self.variant, self.result, self.flags,
                           epilogue=self.epi, workspace=self.ws)


def cmd_layers(args):
    from synth import CONFIG2, CONFIG3, seed_for
    layers = {2: CONFIG2, 3: CONFIG3}[args.config]
    if args.batch:        # the same layers at another batch size (the asymptote of a configuration's small layers)
        import dataclasses
        layers = [dataclasses.replace(s, N=args.batch) for s in layers]
    stream = torch.cuda.Stream()
    rows = []
    for i, s in enumerate(layers):
        row = dict(layer=s.name, gop=s.ops / 1e9)
        for epi in (False, True):
            tag = "i8out" if epi else "i32out"
            t = {}
            FC_ONLY, IC_ONLY = Variant.FUSED_OCG | abed.ONLY_FC, Variant.FUSED_OCG | abed.ONLY_IC
            for v in (Variant.NONE, Variant.FUSED_OCG, Variant.DUPLICATE, FC_ONLY, IC_ONLY):
                L = Int8Layer(s, seed_for(args.config, i), v, epilogue=epi)
                L.run()
                t[v] = _graph_time(lambda: L.run(), stream)
                if v not in (Variant.NONE, Variant.DUPLICATE):
                    assert int(L.flags.abs().max().item()) == 0
                if v == Variant.NONE and args.config == 3:
                    # HBM figure: rotate through buffer sets that together exceed the 256 MB last-level
                    # cache twice over, so that no launch finds its operands cached
                    sets = [L]
                    while sum(o.x.numel() + 4 * o.y.numel() // (4 if epi else 1) for o in sets) < (600 << 20) and len(sets) < 12:
                        sets.append(Int8Layer(s, seed_for(args.config, i) + len(sets), v, epilogue=epi))
                    t_rot = _graph_time(lambda: [o.run() for o in sets], stream, reps=4, replays=5) / len(sets)
                    rot = dict(buffer_sets=len(sets), unchecked_us=t_rot * 1e6)
                    del sets
            F = FicLayer(s, seed_for(args.config, i), Variant.FUSED_OCG, epilogue=epi)
            F.run()
            t_fic = _graph_time(lambda: F.run(), stream)
            assert int(F.flag.item()) == 0
            FL = FicInloopLayer(s, seed_for(args.config, i), epilogue=epi)
            FL.run()
            t_ficl = _graph_time(lambda: FL.run(), stream)
            t_ficl_def = _graph_time(lambda: FL.run(deferred=True), stream)    # the convolution's launch alone
            assert int(FL.flag.item()) == 0
            I2 = Ic2Layer(s, seed_for(args.config, i), Variant.FUSED_OCG, epilogue=epi)
            I2.run()
            t_ic2 = _graph_time(lambda: I2.run(), stream)
            assert int(I2.flags.abs().max().item()) == 0
            nbytes = s.min_bytes(1, 1, 1 if epi else 4)
            row[tag] = dict(unchecked_us=t[Variant.NONE] * 1e6, checked_us=t[Variant.FUSED_OCG] * 1e6,
                            fic_fused_us=t_fic * 1e6, fic_fused_overhead_pct=100.0 * (t_fic / t[Variant.NONE] - 1.0),
                            fic_inloop_us=t_ficl * 1e6, fic_inloop_overhead_pct=100.0 * (t_ficl / t[Variant.NONE] - 1.0),
                            fic_inloop_conv_only_us=t_ficl_def * 1e6, fic_inloop_conv_only_overhead_pct=100.0 * (t_ficl_def / t[Variant.NONE] - 1.0),
                            duplicate_us=t[Variant.DUPLICATE] * 1e6,
                            ic2_fused_us=t_ic2 * 1e6, ic2_fused_overhead_pct=100.0 * (t_ic2 / t[Variant.NONE] - 1.0),
                            fc_only_us=t[FC_ONLY] * 1e6, fc_only_overhead_pct=100.0 * (t[FC_ONLY] / t[Variant.NONE] - 1.0),
                            ic_only_us=t[IC_ONLY] * 1e6, ic_only_overhead_pct=100.0 * (t[IC_ONLY] / t[Variant.NONE] - 1.0),
                            unchecked_tops=s.ops / t[Variant.NONE] / 1e12, checked_tops=s.ops / t[Variant.FUSED_OCG] / 1e12,
                            overhead_pct=100.0 * (t[Variant.FUSED_OCG] / t[Variant.NONE] - 1.0),
                            min_bytes=nbytes, unchecked_hbm_gbs=nbytes / t[Variant.NONE] / 1e9,
                            checked_hbm_gbs=nbytes / t[Variant.FUSED_OCG] / 1e9,
                            unchecked_frac_of_hbm_peak=nbytes / t[Variant.NONE] / 1e9 / PEAK_HBM_GBS)
            if args.config == 3:
                rot.update(unchecked_hbm_gbs=nbytes / (rot["unchecked_us"] * 1e-6) / 1e9,
                           frac_of_hbm_peak=nbytes / (rot["unchecked_us"] * 1e-6) / 1e9 / PEAK_HBM_GBS)
                row[tag]["rotating_buffers"] = rot
        rows.append(row)
    print(json.dumps(dict(config=args.config, batch=layers[0].N, note="checked = FC + batch-checksum IC, FusedOCG incl. the ICG kernel; fc_only / ic_only = one of the two alone (FusedOCG; ic_only incl. the ICG kernel); fic_fused = the FIC scheme of Sec. 3.3, fused option; fic_inloop = FIC with the input side formed in the convolution's main loop (conv_only: without the comparison launch); ic2_fused = IC option 2 of Sec. 3.2 (K values), fused option; GB/s = algorithmic minimum bytes / time",
                          layers=rows)))


def cmd_detect(args):
    """Single-bit flips in accumulators, filters, inputs of an int8 layer (Sec. 5.4 campaigns), for every
    scheme: FC + IC, FC alone, IC alone (abed_conv_int8), FIC (abed_fic_conv_int8, abed_fic_inloop_conv_int8), IC option 2
    (abed_ic2_conv_int8).  Filter and input flips are made after the checksums were generated; only
    flips that change an output count ("corrupting").  The rates are Table 1 of Sec. 3.4, measured."""
    from synth import ConvShape
    s = ConvShape(32, 14, 14, 64, 64, 3, 3, 1, 1, 1, 1, "3x3_c64_14_n32")
    out = {}

    def campaign(name, run, flagged, y, w, x):
        """run(inject, regenerate) enqueues the scheme; regenerate = make the online checksums again."""
        rng = np.random.default_rng(args.seed)
        run(None, True)
        torch.cuda.synchronize()
        assert not flagged(), name + ": flag on a clean run"
        clean = y.clone()
        res = {}
        det = 0
        for _ in range(args.trials):
            idx, bit = int(rng.integers(0, clean.numel())), int(rng.integers(0, 32))
            run((1, idx, bit), False)
            det += int(flagged())
        res["accumulator"] = dict(trials=args.trials, detected=det)
        for site, t in (("filter", w), ("input", x)):
            det = corrupting = 0
            u = t.view(torch.uint8).view(-1)
            for _ in range(args.trials):
                idx, bit = int(rng.integers(0, u.numel())), int(rng.integers(0, 8))
                u[idx] ^= (1 << bit)
                run(None, False)
                changed = not torch.equal(y, clean)
                corrupting += int(changed)
                det += int(changed and flagged())
                u[idx] ^= (1 << bit)
            res[site] = dict(trials=args.trials, corrupting=corrupting, detected_of_corrupting=det)
        out[name] = res

    for name, v in (("fc_ic", Variant.FUSED_OCG), ("fc_only", Variant.FUSED_OCG | abed.ONLY_FC), ("ic_only", Variant.FUSED_OCG | abed.ONLY_IC)):
        L = Int8Layer(s, 7001, v)
        campaign(name, lambda inject, regen, L=L: L.run(compute_xchk=regen, inject=inject),
                 lambda L=L: int(L.flags.abs().max().item()) != 0, L.y, L.w, L.x)
    F = FicLayer(s, 7001, Variant.FUSED_OCG)
    campaign("fic", lambda inject, regen: abed.fic_conv_int8(F.desc, F.x, F.w, F.wsum, F.xrows, regen, F.y, F.variant, F.result, F.flag,
                                                             workspace=F.ws, inject=inject),
             lambda: int(F.flag.item()) != 0, F.y, F.w, F.x)
    # FIC with the input side formed in the main loop: it has no input checksum made ahead of the convolution,
    # so a corrupted input is what both sides of the comparison see (expected: none of those flips caught)
    FL = FicInloopLayer(s, 7001)
    campaign("fic_inloop", lambda inject, regen: FL.run(inject=inject), lambda: int(FL.flag.item()) != 0, FL.y, FL.w, FL.x)
    I2 = Ic2Layer(s, 7001, Variant.FUSED_OCG)
    campaign("ic2", lambda inject, regen: abed.ic2_conv_int8(I2.desc, I2.x, I2.w, I2.xrows, regen, I2.y, I2.variant, I2.result, I2.flags,
                                                             workspace=I2.ws, inject=inject),
             lambda: int(I2.flags.abs().max().item()) != 0, I2.y, I2.w, I2.x)
    fp = 0
    for r in range(args.clean):
        L2 = Int8Layer(s, 8000 + r, Variant.FUSED_OCG)
        L2.run()
        fp += int(L2.flags.abs().max().item() != 0)
    out["clean_runs"] = dict(runs=args.clean, false_positives=fp)
    print(json.dumps(out))


def cmd_fp16(args):
    from synth import CONFIG4, fp16_tensors, seed_for
    s = CONFIG4[0]
    desc = abed.desc_from_shape(s)
    lay = abed.get_layout(desc, 1, Variant.FUSED_OCG)
    y = torch.empty((s.N, s.P, s.Q, s.K), dtype=torch.float16, device=DEV)
    flags = torch.zeros((lay.n_flag_words,), dtype=torch.int32, device=DEV)
    ws = torch.zeros((max(256, lay.workspace_bytes),), dtype=torch.uint8, device=DEV)
    wchk = torch.empty((2, s.R, s.S, s.C), dtype=torch.float16, device=DEV)
    xchk = torch.empty((2, s.H, s.W, s.C), dtype=torch.float16, device=DEV)
    abed.workspace_init(ws)
    res = dict(layer=s.name, runs=args.trials, thresholds=[],
               note="a flip counts as detected only when the flag word that covers the flipped element (its pixel group and "
                    "batch tile for FC, its pixel group and filter tile for IC) has the scheme's bit set and had it clear "
                    "in the clean run of the same input; l1: threshold = rtol * sum|y| over the reduced elements + atol, "
                    "otherwise rtol * max(|s|, |c|) + atol")
    L1 = abed.L1_THRESHOLD
    # (rtol, atol, threshold relative to the sum of magnitudes)
    settings = [(1e-3, 0.0, False), (1e-3, 1e-3, False), (1e-3, 1e-2, False), (1e-3, 3e-2, False),
                (1e-3, 0.0, True), (1e-4, 0.0, True), (1e-5, 0.0, True), (1e-6, 0.0, True)]
    variant_of = lambda st: int(Variant.FUSED_OCG) | (L1 if st[2] else 0)
    clean_fp = {st: 0 for st in settings}
    tiles_fp = {st: 0 for st in settings}
    clean_flags = {}
    for r in range(args.trials):
        xh, wh = fp16_tensors(s, seed_for(4, 0, r))
        x, w = torch.from_numpy(xh).to(DEV), torch.from_numpy(wh).to(DEV)
        abed.filter_prepare_fp16(desc, w, wchk)
        for i, st in enumerate(settings):
            abed.conv_fp16(desc, x, w, wchk, xchk, i == 0, y, variant_of(st), st[0], st[1], flags=flags, workspace=ws)
            n = int((flags != 0).sum().item())
            clean_fp[st] += int(n > 0)
            tiles_fp[st] += n
            clean_flags[st] = flags.cpu().numpy().reshape(lay.grid_m, lay.grid_b, lay.grid_n).copy()
    # detection: flips of one bit of one fp16 output value, on the last input
    rng = np.random.default_rng(args.seed)
    det = {st: [0] * 16 for st in settings}
    masked = {st: 0 for st in settings}        # flips whose covering words were already flagged in the clean run
    cnt = [0] * 16
    PQK = s.P * s.Q * s.K
    for _ in range(args.trials):
        idx, bit = int(rng.integers(0, y.numel())), int(rng.integers(0, 16))
        cnt[bit] += 1
        n, rem = divmod(idx, PQK)
        pix, k = divmod(rem, s.K)
        fcw, icw = (pix // 16, n // lay.tile_batch, 0), (pix // 16, 0, k // lay.tile_n)
        for st in settings:
            abed.conv_fp16(desc, x, w, wchk, xchk, False, y, variant_of(st), st[0], st[1], flags=flags, workspace=ws,
                           inject=(1, idx, bit))
            f = flags.cpu().numpy().reshape(lay.grid_m, lay.grid_b, lay.grid_n)
            c = clean_flags[st]
            fc_hit = bool(f[fcw] & 1) and not (c[fcw] & 1)
            ic_hit = bool(f[icw] & 2) and not (c[icw] & 2)
            det[st][bit] += int(fc_hit or ic_hit)
            masked[st] += int(bool(c[fcw] & 1) and bool(c[icw] & 2))
    # throughput of the same layer: unchecked, checked (ICG + augmented convolution), duplicated
    stream = torch.cuda.Stream()
    y2 = torch.empty_like(y)
    t_plain = _graph_time(lambda: abed.conv_fp16(desc, x, w, None, None, False, y, Variant.NONE, 1e-3, 1e-3), stream)
    t_chk = _graph_time(lambda: abed.conv_fp16(desc, x, w, wchk, xchk, True, y, Variant.FUSED_OCG, 1e-3, 1e-3, flags=flags, workspace=ws), stream)
    t_dup = _graph_time(lambda: abed.conv_fp16(desc, x, w, None, None, False, y, Variant.DUPLICATE, 1e-3, 1e-3, flags=flags, workspace=ws, y2=y2), stream)
    t_l1 = _graph_time(lambda: abed.conv_fp16(desc, x, w, wchk, xchk, True, y, int(Variant.FUSED_OCG) | L1, 1e-3, 0.0, flags=flags, workspace=ws), stream)
    res["timing"] = dict(gflop=s.ops / 1e9, unchecked_us=t_plain * 1e6, checked_us=t_chk * 1e6, duplicate_us=t_dup * 1e6, checked_l1_threshold_us=t_l1 * 1e6,
                         unchecked_tflops=s.ops / t_plain / 1e12, checked_tflops=s.ops / t_chk / 1e12,
                         overhead_pct=100.0 * (t_chk / t_plain - 1.0), frac_of_fp16_peak=s.ops / t_plain / 1e12 / 2500.0)
    for st in settings:
        res["thresholds"].append(dict(rtol=st[0], atol=st[1], l1=st[2], clean_runs_with_a_flag=clean_fp[st],
                                      flagged_tiles_per_clean_run=tiles_fp[st] / args.trials,
                                      tiles_per_run=int(lay.n_flag_words),
                                      flips_detected=sum(det[st]), flips=args.trials, flips_on_already_flagged_words=masked[st],
                                      detected_by_bit=det[st], flips_by_bit=cnt))
    print(json.dumps(res))


def cmd_resnet50(args):
    """The 53 convolution layers of a ResNet-50-shaped network, int8 with a fused requantize + ReLU
    epilog, back to back on one stream: unchecked, FC + IC checked (FusedOCG on every layer, and
    FusedIOCG where inside a bottleneck the second and third convolutions take their batch checksum
    from the previous kernel; the better of the two is reported as `checked`), duplicated, FC alone,
    and the FIC scheme."""
    from synth import ConvShape, resnet50_layers
    layers = resnet50_layers(args.batch)
    stream = torch.cuda.Stream()
    total_ops = sum(s.ops for s in layers)
    result = dict(batch=args.batch, layers=len(layers), gop=total_ops / 1e9)
    def preferred(s, only):
        """FusedOCG in the form the library's timing rule prefers for the layer: checksums local to a workgroup
        (ABED_LOCAL) where the shape is covered and abed_layout_t.local_preferred says so, else layer-wide."""
        v = int(Variant.FUSED_OCG) | only
        try:
            return v | abed.LOCAL if abed.get_layout(abed.desc_from_shape(s), 0, v | abed.LOCAL).local_preferred else v
        except abed.AbedError:
            return v

    n_local = {}
    for mode, variant in (("unchecked", Variant.NONE), ("checked_iocg", Variant.FUSED_IOCG), ("checked_ocg", Variant.FUSED_OCG),
                          ("duplicate", Variant.DUPLICATE), ("fc_only", Variant.FUSED_OCG | abed.ONLY_FC),
                          ("checked_ocg_preferred_form", None), ("fc_only_preferred_form", None)):
        objs, chained = [], []
        prev = None
        per_layer = variant is None
        for i, s in enumerate(layers):
            if s.C % 16:      # the 3-channel stem: channels padded with zeros to 16 by the caller
                s = ConvShape(s.N, s.H, s.W, 16, s.K, s.R, s.S, s.stride_h, s.stride_w, s.pad_h, s.pad_w, s.name)
            chain = prev is not None and s.name.split(".")[-1] in ("c2", "c3") and prev.s.name.split(".")[0] == s.name.split(".")[0]
            if per_layer:
                variant = preferred(s, abed.ONLY_FC if mode.startswith("fc_only") else 0)
                n_local[mode] = n_local.get(mode, 0) + (1 if variant & abed.LOCAL else 0)
            L = Int8Layer(s, 5000 + i, variant, epilogue=True, x=prev.y if chain else None)
            objs.append(L)
            chained.append(chain)
            prev = L

        def step():
            for j, L in enumerate(objs):
                L.run(compute_xchk=not (variant == Variant.FUSED_IOCG and chained[j]))
        if variant == Variant.FUSED_IOCG:
            # chained layers read the previous layer's emitted checksum directly
            for j, L in enumerate(objs):
                if chained[j]:
                    L.xchk = objs[j - 1].xchk_next
        step()
        torch.cuda.synchronize()
        if variant not in (Variant.NONE, Variant.DUPLICATE):
            bad = [L.s.name for L in objs if int(L.flags.abs().max().item()) != 0]
            assert not bad, "flags set on a clean run: %s" % bad
        t = _graph_time(step, stream, reps=2, replays=5)
        result[mode] = dict(ms=t * 1e3, tops=total_ops / t / 1e12)
        if per_layer:
            result[mode]["local_layers"] = n_local[mode]
            result[mode + "_overhead_pct"] = 100.0 * (result[mode]["ms"] / result["unchecked"]["ms"] - 1.0)
            variant = None
        del objs
        torch.cuda.empty_cache()
    # the FIC scheme (Sec. 3.3), fused option, every layer with its own input checksum generation
    objs = []
    for i, s in enumerate(layers):
        if s.C % 16:
            s = ConvShape(s.N, s.H, s.W, 16, s.K, s.R, s.S, s.stride_h, s.stride_w, s.pad_h, s.pad_w, s.name)
        objs.append(FicLayer(s, 5000 + i, Variant.FUSED_OCG, epilogue=True))

    def fic_step():
        for L in objs:
            L.run()
    fic_step()
    torch.cuda.synchronize()
    bad = [L.s.name for L in objs if int(L.flag.item()) != 0]
    assert not bad, "FIC flag set on a clean run: %s" % bad
    t = _graph_time(fic_step, stream, reps=2, replays=5)
    result["fic_fused"] = dict(ms=t * 1e3, tops=total_ops / t / 1e12)
    result["fic_fused_overhead_pct"] = 100.0 * (result["fic_fused"]["ms"] / result["unchecked"]["ms"] - 1.0)
    # the same with the comparisons deferred: every layer leaves its partial sums, two launches verify all 53
    res_all = torch.zeros((len(objs), 2), dtype=torch.int64, device=DEV)
    flag_all = torch.zeros((len(objs),), dtype=torch.int32, device=DEV)

    def fic_deferred_step():
        for L in objs:
            abed.fic_conv_int8(L.desc, L.x, L.w, L.wsum, L.xrows, True, L.y, L.variant, None, None, epilogue=L.epi, workspace=L.ws)
        abed.fic_verify([L.desc for L in objs], [L.variant for L in objs], [L.ws for L in objs], res_all, flag_all)
    fic_deferred_step()
    torch.cuda.synchronize()
    assert int(flag_all.abs().max().item()) == 0 and bool((res_all[:, 0] == res_all[:, 1]).all().item())
    t = _graph_time(fic_deferred_step, stream, reps=2, replays=5)
    result["fic_fused_deferred"] = dict(ms=t * 1e3, tops=total_ops / t / 1e12)
    result["fic_fused_deferred_overhead_pct"] = 100.0 * (result["fic_fused_deferred"]["ms"] / result["unchecked"]["ms"] - 1.0)
    del objs
    torch.cuda.empty_cache()
    # FIC with the input side formed in the main loop: one launch per layer plus the comparison, or deferred
    objs = []
    for i, s in enumerate(layers):
        if s.C % 16:
            s = ConvShape(s.N, s.H, s.W, 16, s.K, s.R, s.S, s.stride_h, s.stride_w, s.pad_h, s.pad_w, s.name)
        objs.append(FicInloopLayer(s, 5000 + i, epilogue=True))

    def inloop_step():
        for L in objs:
            L.run()
    inloop_step()
    torch.cuda.synchronize()
    bad = [L.s.name for L in objs if int(L.flag.item()) != 0]
    assert not bad, "FIC (in-loop) flag set on a clean run: %s" % bad
    t = _graph_time(inloop_step, stream, reps=2, replays=5)
    result["fic_inloop"] = dict(ms=t * 1e3, tops=total_ops / t / 1e12)
    result["fic_inloop_overhead_pct"] = 100.0 * (result["fic_inloop"]["ms"] / result["unchecked"]["ms"] - 1.0)

    def inloop_deferred_step():
        for L in objs:
            L.run(deferred=True)
        abed.fic_verify([L.desc for L in objs], [L.variant for L in objs], [L.ws for L in objs], res_all, flag_all)
    inloop_deferred_step()
    torch.cuda.synchronize()
    assert int(flag_all.abs().max().item()) == 0 and bool((res_all[:, 0] == res_all[:, 1]).all().item())
    t = _graph_time(inloop_deferred_step, stream, reps=2, replays=5)
    result["fic_inloop_deferred"] = dict(ms=t * 1e3, tops=total_ops / t / 1e12)
    result["fic_inloop_deferred_overhead_pct"] = 100.0 * (result["fic_inloop_deferred"]["ms"] / result["unchecked"]["ms"] - 1.0)
    # per layer the faster of the two (timed once per distinct shape, as a deployment would tune it), comparisons deferred
    rows_objs, pick, seen = [], [], {}
    for i, L in enumerate(objs):
        s = L.s
        R = FicLayer(s, 5000 + i, Variant.FUSED_OCG, epilogue=True, x=L.x)
        rows_objs.append(R)
        key = (s.H, s.W, s.C, s.K, s.R, s.S, s.stride_h)
        if key not in seen:
            t_in = _graph_time(lambda: L.run(deferred=True), stream, reps=5, replays=3)
            t_rows = _graph_time(lambda: abed.fic_conv_int8(R.desc, R.x, R.w, R.wsum, R.xrows, True, R.y, R.variant, None, None,
                                                            epilogue=R.epi, workspace=R.ws), stream, reps=5, replays=3)
            seen[key] = t_in <= t_rows
        pick.append(L if seen[key] else R)

    def best_step():
        for L in pick:
            if isinstance(L, FicInloopLayer):
                L.run(deferred=True)
            else:
                abed.fic_conv_int8(L.desc, L.x, L.w, L.wsum, L.xrows, True, L.y, L.variant, None, None, epilogue=L.epi, workspace=L.ws)
        abed.fic_verify([L.desc for L in pick], [L.variant for L in pick], [L.ws for L in pick], res_all, flag_all)
    best_step()
    torch.cuda.synchronize()
    assert int(flag_all.abs().max().item()) == 0 and bool((res_all[:, 0] == res_all[:, 1]).all().item())
    t = _graph_time(best_step, stream, reps=2, replays=5)
    result["fic_faster_of_two_deferred"] = dict(ms=t * 1e3, tops=total_ops / t / 1e12,
                                                inloop_layers=sum(1 for L in pick if isinstance(L, FicInloopLayer)))
    result["fic_faster_of_two_deferred_overhead_pct"] = 100.0 * (result["fic_faster_of_two_deferred"]["ms"] / result["unchecked"]["ms"] - 1.0)
    del objs, rows_objs, pick
    torch.cuda.empty_cache()
    # FIC with the next layer's input checksum generation fused in (Sec. 4.3): inside a bottleneck the
    # second and third convolutions take the batch sum of their input from the previous kernel
    objs, prev = [], None
    for i, s in enumerate(layers):
        if s.C % 16:
            s = ConvShape(s.N, s.H, s.W, 16, s.K, s.R, s.S, s.stride_h, s.stride_w, s.pad_h, s.pad_w, s.name)
        chain = prev is not None and s.name.split(".")[-1] in ("c2", "c3") and prev.s.name.split(".")[0] == s.name.split(".")[0]
        L = FicLayer(s, 5000 + i, Variant.FUSED_IOCG, epilogue=True, x=prev.y if chain else None)
        if chain:
            prev.xsum_next = torch.zeros((prev.s.P, prev.s.Q, prev.s.K), dtype=torch.int32, device=DEV)
            L.xsum_in = prev.xsum_next
        objs.append(L)
        prev = L

    def fic_chain_step():
        for L in objs:
            L.run()
    fic_chain_step()
    torch.cuda.synchronize()
    bad = [L.s.name for L in objs if int(L.flag.item()) != 0]
    assert not bad, "FIC (chained) flag set on a clean run: %s" % bad
    t = _graph_time(fic_chain_step, stream, reps=2, replays=5)
    result["fic_iocg"] = dict(ms=t * 1e3, tops=total_ops / t / 1e12, chained_layers=sum(1 for L in objs if L.xsum_in is not None))
    result["fic_iocg_overhead_pct"] = 100.0 * (result["fic_iocg"]["ms"] / result["unchecked"]["ms"] - 1.0)
    del objs
    torch.cuda.empty_cache()
    # FC + IC: with every layer running its own input checksum kernel (FusedOCG), or with the second and
    # third convolution of a bottleneck taking the batch checksum the previous kernel emitted (FusedIOCG)
    best = min(("checked_ocg", "checked_iocg"), key=lambda k: result[k]["ms"])
    result["checked"] = dict(result[best], variant=best)
    for k in ("checked_ocg", "checked_iocg"):
        result[k + "_overhead_pct"] = 100.0 * (result[k]["ms"] / result["unchecked"]["ms"] - 1.0)
    result["overhead_pct"] = 100.0 * (result["checked"]["ms"] / result["unchecked"]["ms"] - 1.0)
    result["duplicate_overhead_pct"] = 100.0 * (result["duplicate"]["ms"] / result["unchecked"]["ms"] - 1.0)
    result["fc_only_overhead_pct"] = 100.0 * (result["fc_only"]["ms"] / result["unchecked"]["ms"] - 1.0)
    print(json.dumps(result))


def cmd_abft(args):
    """The traditional ABFT technique at the GEMM level (Sec. 5.3 / 6.3): run time of its tasks (copy into the larger
    operands, checksum generation, the larger GEMM, verification by rows and by columns, copy back) against the plain
    GEMM, on the GEMM shapes of the configured layers (M = N*P*Q, Kg = C*R*S, Ng = K; the operand of a 3x3 layer's
    GEMM is a synthetic matrix of the lowered shape), next to the FC + IC and FIC overheads of the same layers."""
    from synth import CONFIG2, CONFIG3
    stream = torch.cuda.Stream()
    rows = []
    for cfg, layers in ((3, CONFIG3), (2, CONFIG2)):
        for li, s in enumerate(layers):
            M, Kg, Ng = s.N * s.P * s.Q, s.C * s.R * s.S, s.K
            g = torch.Generator(device="cpu").manual_seed(900 + 10 * cfg + li)
            A = torch.randint(-128, 128, (M, Kg), dtype=torch.int8, generator=g).to(DEV)
            B = torch.randint(-128, 128, (Ng, Kg), dtype=torch.int8, generator=g).to(DEV)
            lay = abed.abft_gemm_get_layout(M, Ng, Kg)
            ws = torch.zeros((lay.workspace_bytes,), dtype=torch.uint8, device=DEV)
            C = torch.empty((M, Ng), dtype=torch.int32, device=DEV)
            flags = torch.zeros((8,), dtype=torch.int32, device=DEV)
            run = lambda tasks=0: abed.abft_gemm_int8(M, Ng, Kg, A, B, C, flags, ws, tasks=tasks)
            run(); torch.cuda.synchronize()
            assert int(flags[0].item()) == 0
            # the plain GEMM: the same product without checksums, as a 1x1 convolution over 16x16 planes
            from synth import ConvShape
            mp = (M + 255) // 256 * 256
            Ap = torch.zeros((mp, Kg), dtype=torch.int8, device=DEV); Ap[:M].copy_(A)
            gd = abed.desc_from_shape(ConvShape(mp // 256, 16, 16, Kg, Ng, 1, 1, 1, 1, 0, 0, "gemm"))
            Cg = torch.empty((mp, Ng), dtype=torch.int32, device=DEV)
            t_plain = _graph_time(lambda: abed.conv_int8(gd, Ap, B, None, None, False, Cg, Variant.NONE), stream)
            assert torch.equal(Cg[:M], C)
            t = {name: _graph_time(lambda bit=bit: run(bit), stream) for name, bit in abed.ABFT_TASKS.items()}
            t_all = _graph_time(lambda: run(0), stream)
            row = dict(config=cfg, layer=s.name, M=M, Kg=Kg, Ng=Ng, gemm_us=t_plain * 1e6, abft_total_us=t_all * 1e6,
                       abft_overhead_pct=100.0 * (t_all / t_plain - 1.0),
                       tasks_us={k: v * 1e6 for k, v in t.items()},
                       larger_gemm_overhead_pct=100.0 * (t["gemm"] / t_plain - 1.0))
            # the paper's schemes on the same layer, same protocol
            t_conv = {}
            for name, variant in (("unchecked", Variant.NONE), ("fc_ic", Variant.FUSED_OCG), ("fc_only", Variant.FUSED_OCG | abed.ONLY_FC)):
                L = Int8Layer(s, seed_for_layer(cfg, li), variant)
                t_conv[name] = _graph_time(L.run, stream)
                del L
            F = FicLayer(s, seed_for_layer(cfg, li), Variant.FUSED_OCG)
            t_conv["fic"] = _graph_time(F.run, stream)
            del F
            row.update(conv_unchecked_us=t_conv["unchecked"] * 1e6,
                       fc_ic_overhead_pct=100.0 * (t_conv["fc_ic"] / t_conv["unchecked"] - 1.0),
                       fc_only_overhead_pct=100.0 * (t_conv["fc_only"] / t_conv["unchecked"] - 1.0),
                       fic_overhead_pct=100.0 * (t_conv["fic"] / t_conv["unchecked"] - 1.0))
            rows.append(row)
            print(json.dumps(row), flush=True)
            del ws, A, B, C, Ap, Cg
            torch.cuda.empty_cache()
    print(json.dumps(dict(abft_gemm=rows)))


def seed_for_layer(cfg, li):
    from synth import seed_for
    return seed_for(cfg, li)


def cmd_ksweep(args):
    """Filter-count sweep on one layer (Sec. 6.2's tile-boundary study): 3x3, C=64, stride 1, pad 1 on a
    112x112 input, K from 8 upwards in steps of 8; unchecked, the filter checksum scheme alone (its extra
    block of checksum filters is what a tile boundary makes expensive), and FC + IC.  int32 ConvOut."""
    from synth import ConvShape
    stream = torch.cuda.Stream()
    rows = []
    for K in range(8, args.kmax + 1, 8):
        s = ConvShape(args.batch, 112, 112, 64, K, 3, 3, 1, 1, 1, 1, "3x3_c64_112_k%d" % K)
        t, tile = {}, {}
        runs = [("unchecked", Variant.NONE), ("fc_only", Variant.FUSED_OCG | abed.ONLY_FC), ("fc_ic", Variant.FUSED_OCG)]
        if K % 16 and K % 16 + 2 <= 16:      # room for the two checksum filters in the last block of 16
            runs.append(("fc_only_packed", Variant.FUSED_OCG | abed.ONLY_FC | abed.PACKED_FC))
        for name, v in runs:
            L = Int8Layer(s, 9000 + K, v)
            L.run()
            t[name] = _graph_time(lambda: L.run(), stream, reps=5, replays=4)
            tile[name] = "%dx%d, grid %dx%dx%d" % (L.lay.tile_batch, L.lay.tile_n, L.lay.grid_m, L.lay.grid_b, L.lay.grid_n)
            if v != Variant.NONE:
                assert int(L.flags.abs().max().item()) == 0
            del L
        rows.append(dict(K=K, gop=s.ops / 1e9, unchecked_us=t["unchecked"] * 1e6, fc_only_us=t["fc_only"] * 1e6, fc_ic_us=t["fc_ic"] * 1e6,
                         fc_only_overhead_pct=100.0 * (t["fc_only"] / t["unchecked"] - 1.0),
                         fc_ic_overhead_pct=100.0 * (t["fc_ic"] / t["unchecked"] - 1.0),
                         unchecked_tops=s.ops / t["unchecked"] / 1e12, tile_unchecked=tile["unchecked"], tile_fc_only=tile["fc_only"]))
        if "fc_only_packed" in t:
            rows[-1].update(fc_only_packed_us=t["fc_only_packed"] * 1e6, fc_only_packed_overhead_pct=100.0 * (t["fc_only_packed"] / t["unchecked"] - 1.0))
        print("K", K, "done", file=sys.stderr, flush=True)
    print(json.dumps(dict(layer="3x3 C=64 112x112 s1 p1", batch=args.batch, rows=rows)))


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    a = sub.add_parser("layers"); a.add_argument("--config", type=int, default=3, choices=[2, 3]); a.add_argument("--batch", type=int, default=0)
    a = sub.add_parser("detect"); a.add_argument("--trials", type=int, default=1000); a.add_argument("--clean", type=int, default=100); a.add_argument("--seed", type=int, default=1)
    sub.add_parser("abft")
    a = sub.add_parser("fp16"); a.add_argument("--trials", type=int, default=1000); a.add_argument("--seed", type=int, default=1)
    a = sub.add_parser("resnet50"); a.add_argument("--batch", type=int, default=128)
    a = sub.add_parser("ksweep"); a.add_argument("--batch", type=int, default=16); a.add_argument("--kmax", type=int, default=144)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        sys.exit(1)
    abed.lib()
    {"layers": cmd_layers, "detect": cmd_detect, "fp16": cmd_fp16, "resnet50": cmd_resnet50, "ksweep": cmd_ksweep, "abft": cmd_abft}[args.cmd](args)


if __name__ == "__main__":
    main()
