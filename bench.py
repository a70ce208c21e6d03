#!/usr/bin/env python3
"""Benchmark of the ABED convolution hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input:
the four ResNet-50-shaped int8 3x3 layers (batch 32, stride 1, pad 1; C=K=64 at
56x56, 128 at 28x28, 256 at 14x14, 512 at 7x7), each through abed_conv_int8 with
the fully fused variant (FusedOCG: checksum generation, reduction, comparison and
flagging inside the convolution's launch), int32 ConvOut as output.  A layer takes
the form of FusedOCG that the library's own rule prefers for its shape: checksums
local to a workgroup (ABED_LOCAL: one launch, batch checksum formed inside the
kernel) where the box kernel fills the chip, else the layer-wide checksums (input
checksum kernel + augmented convolution).  Inputs are resident in HBM before the
timed region.  TOPS count the real convolution work only (2*N*P*Q*K*C*R*S);
checksum work is overhead and is never credited.

Prints ONE JSON line.  Extra keys report the unchecked kernel, the duplication
baseline, every variant's overhead, per-layer times, the same layers at batch 256,
the memory-bound 1x1 layers and the machine's measured ceilings.
"""
import argparse
import dataclasses
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0     # MI355X dense int8 MFMA peak, TOP/s
PEAK_HBM_GBS = 8000.0
# HBM bytes per launch of the checked convolution kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# scaled by a copy of known size (profiles/), keyed by (layer, batch, variant form, tile plan as the layout
# reports it); anything not listed was not measured and is reported as null.
MEASURED_TRAFFIC_BYTES = {
    ("3x3_c512_7", 32, "layer", (16, 8, 64, 4, 5, 9)): 16.2e6 + 7.9e6,
    ("3x3_c256_14", 32, "layer", (16, 12, 64, 13, 3, 5)): 12.7e6 + 9.9e6,
    ("3x3_c128_28", 32, "layer", (16, 8, 80, 49, 5, 2)): 12.8e6 + 20.9e6,
    ("3x3_c64_56", 32, "local", (64, 8, 64, 49, 4, 1)): 9.7e6 + 34.3e6,
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--variants", default="all", help="'all' or 'main' (only unchecked, fused, duplicate)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path has no multi-GPU part); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2006_04984_amd as abed
    from paper_2006_04984_amd import Variant
    from paper_2006_04984_amd.evaluate import Int8Layer, FicLayer, FicInloopLayer
    from synth import CONFIG2, CONFIG3, int8_tensors, seed_for

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    abed.lib()  # fails loudly if libabed.so is not built
    dev = "cuda:0"
    layers = CONFIG2
    total_ops = sum(s.ops for s in layers)
    stream = torch.cuda.Stream()
    V_OCG, V_LOCAL = int(Variant.FUSED_OCG), int(Variant.FUSED_OCG) | abed.LOCAL

    def fused_form(s, only=0):
        """The form of FusedOCG a layer takes: ABED_LOCAL where the shape is covered and the library's own
        timing rule prefers it (abed_layout_t.local_preferred), else the layer-wide checksums.  only: ABED_ONLY_FC
        or ABED_ONLY_IC (one scheme alone; the rule looks at the scheme)."""
        try:
            lay = abed.get_layout(abed.desc_from_shape(s), 0, V_LOCAL | only)
        except abed.AbedError:
            return V_OCG | only
        return (V_LOCAL if lay.local_preferred else V_OCG) | only

    def graph_of(fn, per_graph):
        with torch.cuda.stream(stream):
            fn()
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for _ in range(per_graph):
                    fn()
            graph.replay()
            torch.cuda.synchronize()
        return graph

    def time_steps(fn, steps, warmup, per_graph=10, samples=5):
        """`samples` timed runs of `steps` steps each, launched as replays of a HIP graph that holds `per_graph`
        steps (the launches of a step are tiny next to the host's cost of issuing them one by one), bracketed by
        device synchronisation.  Returns (median seconds per step, all samples)."""
        if steps % per_graph:
            per_graph = 1
        graph = graph_of(fn, per_graph)
        with torch.cuda.stream(stream):
            for _ in range(max(1, warmup // per_graph)):
                graph.replay()
            torch.cuda.synchronize()
            ts = []
            for _ in range(samples):
                t0 = time.perf_counter()
                for _ in range(steps // per_graph):
                    graph.replay()
                torch.cuda.synchronize()
                ts.append((time.perf_counter() - t0) / steps)
        return statistics.median(ts), ts

    def time_eager(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    def event_time(fn, reps=20, replays=10, samples=3):
        """Median duration of one call of fn (its kernel launches), from HIP events on the stream the library
        launches on, around replays of a graph of `reps` calls."""
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        graph = graph_of(fn, reps)
        ts = []
        with torch.cuda.stream(stream):
            for _ in range(samples):
                e0.record(stream)
                for _ in range(replays):
                    graph.replay()
                e1.record(stream)
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1) * 1e-3 / (reps * replays))
        return statistics.median(ts)

    def make_set(shapes, variant_of, cfg=2):
        return [Int8Layer(s, seed_for(cfg, i), variant_of(s)) for i, s in enumerate(shapes)]

    def step_of(Ls):
        return lambda: [L.run() for L in Ls]

    def assert_clean(Ls, what):
        for L in Ls:
            assert int(L.flags.abs().max().item()) == 0, "error flag set on a fault-free run (%s, %s)" % (what, L.s.name)

    sets = {"FUSED_OCG": make_set(layers, fused_form), "NONE": make_set(layers, lambda s: int(Variant.NONE)),
            "DUPLICATE": make_set(layers, lambda s: int(Variant.DUPLICATE))}
    forms = ["local" if L.variant & abed.LOCAL else "layer" for L in sets["FUSED_OCG"]]
    other = {"FUSED_OCG_LAYERWIDE": lambda s: V_OCG}
    if args.variants == "all":
        other.update(UNFUSED=lambda s: int(Variant.UNFUSED), FUSED_WRITE=lambda s: int(Variant.FUSED_WRITE),
                     FUSED_PARTIAL_REDUCTION=lambda s: int(Variant.FUSED_PARTIAL_REDUCTION), FUSED_IOCG=lambda s: int(Variant.FUSED_IOCG))

    # ---- the timed region: K steps of the fully fused checked path ----
    t_checked, checked_samples = time_steps(step_of(sets["FUSED_OCG"]), args.steps, args.warmup)
    assert_clean(sets["FUSED_OCG"], "FusedOCG")     # clean run => no flag may be set
    sub_steps, sub_warm = max(20, args.steps // 2 // 10 * 10), max(10, args.warmup // 2)
    t_var = {"FUSED_OCG": t_checked}
    for name in ("NONE", "DUPLICATE"):
        t_var[name] = time_steps(step_of(sets[name]), sub_steps, sub_warm)[0]
    for name, vo in other.items():
        Ls = make_set(layers, vo)
        t_var[name] = time_steps(step_of(Ls), sub_steps, sub_warm)[0]
        assert_clean(Ls, name)
        del Ls
    t_unchecked, t_dup = t_var["NONE"], t_var["DUPLICATE"]
    # each of the two checksum schemes of the headline path alone (Table 1 of Sec. 3.4), same form per layer
    t_single = {}
    for name, bit in (("fc_only", abed.ONLY_FC), ("ic_only", abed.ONLY_IC)):
        Ls = make_set(layers, lambda s: fused_form(s, bit))
        t_single[name] = time_steps(step_of(Ls), sub_steps, sub_warm)[0]
        assert_clean(Ls, name)
        del Ls
    # the paper's own FIC scheme (one scalar check per layer): fused / unfused options, deferred comparisons
    fic_sets = {v: [FicLayer(s, seed_for(2, i), v) for i, s in enumerate(layers)] for v in (Variant.FUSED_OCG, Variant.UNFUSED)}
    t_fic = {}
    for v, Ls in fic_sets.items():
        t_fic[v] = time_steps(step_of(Ls), sub_steps, sub_warm)[0]
        for L in Ls:
            r = L.result.cpu().numpy()
            assert int(L.flag.item()) == 0 and r[0] == r[1], "FIC mismatch on a fault-free run"
    Ls = fic_sets[Variant.FUSED_OCG]
    res_all = torch.zeros((len(Ls), 2), dtype=torch.int64, device=dev)
    flag_all = torch.zeros((len(Ls),), dtype=torch.int32, device=dev)

    def fic_deferred_step():
        for L in Ls:
            abed.fic_conv_int8(L.desc, L.x, L.w, L.wsum, L.xrows, True, L.y, L.variant, None, None, workspace=L.ws)
        abed.fic_verify([L.desc for L in Ls], [L.variant for L in Ls], [L.ws for L in Ls], res_all, flag_all)
    t_fic_deferred = time_steps(fic_deferred_step, sub_steps, sub_warm)[0]
    assert int(flag_all.abs().max().item()) == 0 and bool((res_all[:, 0] == res_all[:, 1]).all().item()), "FIC mismatch on a fault-free run"
    Li = [FicInloopLayer(s, seed_for(2, i)) for i, s in enumerate(layers)]

    def fic_inloop_step():
        for L in Li:
            L.run(deferred=True)
        abed.fic_verify([L.desc for L in Li], [abed.FIC_INLOOP for L in Li], [L.ws for L in Li], res_all, flag_all)
    t_fic_inloop = time_steps(fic_inloop_step, sub_steps, sub_warm)[0]
    assert int(flag_all.abs().max().item()) == 0 and bool((res_all[:, 0] == res_all[:, 1]).all().item()), "FIC (in-loop) mismatch on a fault-free run"
    del Li, fic_sets, Ls
    t_checked_eager = time_eager(step_of(sets["FUSED_OCG"]), max(20, args.steps // 4), 5)

    # ---- per-layer kernel durations with events on the launch stream ----
    def attainable(s):
        """Roofline of the layer itself: min(matrix peak, arithmetic intensity x HBM peak), as a fraction of the matrix peak."""
        ai = s.ops / s.min_bytes(1, 1, 4)
        return min(PEAK_INT8_TOPS, ai * PEAK_HBM_GBS / 1e3) / PEAK_INT8_TOPS

    def layer_rows(shapes, cfg, Lcs, Lns):
        rows = []
        for s, Lc, Ln in zip(shapes, Lcs, Lns):
            local = bool(Lc.variant & abed.LOCAL)
            t_all = event_time(Lc.run)                                   # everything the checked call launches
            t_conv = t_all if local else event_time(lambda: Lc.run(compute_xchk=False))   # its convolution kernel alone
            t_plain = event_time(Ln.run)
            lay = Lc.lay
            rows.append(dict(layer=s.name, batch=s.N, gop=s.ops / 1e9, form="local" if local else "layer",
                             unchecked_us=t_plain * 1e6, checked_conv_us=t_conv * 1e6, checked_total_us=t_all * 1e6,
                             unchecked_tops=s.ops / t_plain / 1e12, checked_tops=s.ops / t_all / 1e12,
                             overhead_pct=100.0 * (t_all / t_plain - 1.0), min_bytes_i32=s.min_bytes(1, 1, 4),
                             attainable_frac_of_peak=attainable(s),
                             unchecked_frac_of_attainable=s.ops / t_plain / 1e12 / PEAK_INT8_TOPS / attainable(s),
                             checked_frac_of_attainable=s.ops / t_all / 1e12 / PEAK_INT8_TOPS / attainable(s),
                             tile=[lay.tile_pixels, lay.tile_batch, lay.tile_n], grid=[lay.grid_m, lay.grid_b, lay.grid_n]))
        return rows

    per_layer = layer_rows(layers, 2, sets["FUSED_OCG"], sets["NONE"])
    dom = max(per_layer, key=lambda r: r["checked_conv_us"])
    dom_shape = layers[[r["layer"] for r in per_layer].index(dom["layer"])]
    achieved = dom_shape.ops / (dom["checked_conv_us"] * 1e-6) / 1e12
    traffic = MEASURED_TRAFFIC_BYTES.get((dom["layer"], dom["batch"], dom["form"], tuple(dom["tile"] + dom["grid"])))
    roofline = dict(bound="mfma", kernel=("box_conv_kernel" if dom["form"] == "local" else "conv_kernel (augmented)") + " on " + dom["layer"],
                    achieved=achieved, peak=PEAK_INT8_TOPS, unit="TFLOP/s", op="int8 multiply-add counted as 2 ops",
                    frac=achieved / PEAK_INT8_TOPS, traffic=traffic, algorithmic_bytes=dom["min_bytes_i32"],
                    ops_per_launch=dom_shape.ops, avg_launch_us=dom["checked_conv_us"],
                    attainable_frac_of_peak=dom["attainable_frac_of_peak"])
    for name in ("FUSED_OCG", "NONE", "DUPLICATE"):
        del sets[name][:]
    torch.cuda.empty_cache()

    # ---- the same four layers at 256 images: where the fixed costs of a launch no longer dominate ----
    big = [dataclasses.replace(s, N=256) for s in layers]
    Lc, Ln = make_set(big, fused_form), make_set(big, lambda s: int(Variant.NONE))
    n256_rows = layer_rows(big, 2, Lc, Ln)
    assert_clean(Lc, "FusedOCG, 256 images")
    # the same unchecked layers through the library's second 3x3 main loop (one wave per SIMD; opt-in, ABED_IMG=1)
    os.environ["ABED_IMG"] = "1"
    for row, L in zip(n256_rows, Ln):
        t_img = event_time(L.run)
        row["unchecked_img_kernel_us"] = t_img * 1e6
        row["unchecked_img_kernel_tops"] = L.s.ops / t_img / 1e12
    os.environ.pop("ABED_IMG")
    del Lc, Ln
    torch.cuda.empty_cache()
    # the other schemes at 256 images: FC alone (Sec. 3.1; the library's form per layer) and FIC (Sec. 3.3; fused
    # option, its one-workgroup comparison launch included)
    for i, (row, s) in enumerate(zip(n256_rows, big)):
        Lf = Int8Layer(s, seed_for(2, i), fused_form(s, abed.ONLY_FC))
        t_fc = event_time(Lf.run)
        assert int(Lf.flags.abs().max().item()) == 0, "error flag set on a fault-free run (FC alone, 256 images, %s)" % s.name
        del Lf
        Lq = FicLayer(s, seed_for(2, i), Variant.FUSED_OCG)
        t_q = event_time(Lq.run)
        r = Lq.result.cpu().numpy()
        assert int(Lq.flag.item()) == 0 and r[0] == r[1], "FIC mismatch on a fault-free run (256 images)"
        del Lq
        row.update(fc_only_us=t_fc * 1e6, fc_only_overhead_pct=100.0 * (t_fc * 1e6 / row["unchecked_us"] - 1.0),
                   fic_fused_us=t_q * 1e6, fic_fused_overhead_pct=100.0 * (t_q * 1e6 / row["unchecked_us"] - 1.0))
        torch.cuda.empty_cache()
    t_plain_256 = sum(r["unchecked_us"] for r in n256_rows)
    n256 = dict(note="the four layers at 256 images (8x the work per launch), same protocol; overhead_pct is FC + IC FusedOCG (the north-star scheme), fc_only / fic_fused the other schemes of Sec. 3",
                layers=n256_rows,
                unchecked_tops=sum(s.ops for s in big) / t_plain_256 / 1e6,
                checked_tops=sum(s.ops for s in big) / sum(r["checked_total_us"] for r in n256_rows) / 1e6,
                overhead_pct=100.0 * (sum(r["checked_total_us"] for r in n256_rows) / t_plain_256 - 1.0),
                fc_only_overhead_pct=100.0 * (sum(r["fc_only_us"] for r in n256_rows) / t_plain_256 - 1.0),
                fic_fused_overhead_pct=100.0 * (sum(r["fic_fused_us"] for r in n256_rows) / t_plain_256 - 1.0))
    torch.cuda.empty_cache()

    # ---- supplement: the same layers with the fused requantize + ReLU epilog (Sec. 4.3), int8 output: a quarter of the
    # output bytes, so the first two layers are no longer bound by their stores ----
    def i8_rows(shapes):
        rows = []
        for i, s in enumerate(shapes):
            Lc = Int8Layer(s, seed_for(2, i), fused_form(s), epilogue=True)
            Ln = Int8Layer(s, seed_for(2, i), int(Variant.NONE), epilogue=True)
            t_c, t_n = event_time(Lc.run), event_time(Ln.run)
            assert int(Lc.flags.abs().max().item()) == 0, "error flag set on a fault-free run (int8 output, %s)" % s.name
            att = min(PEAK_INT8_TOPS, s.ops / s.min_bytes(1, 1, 1) * PEAK_HBM_GBS / 1e3) / PEAK_INT8_TOPS
            rows.append(dict(layer=s.name, batch=s.N, form="local" if Lc.variant & abed.LOCAL else "layer",
                             unchecked_us=t_n * 1e6, checked_total_us=t_c * 1e6, unchecked_tops=s.ops / t_n / 1e12,
                             checked_tops=s.ops / t_c / 1e12, overhead_pct=100.0 * (t_c / t_n - 1.0),
                             min_bytes_i8=s.min_bytes(1, 1, 1), attainable_frac_of_peak=att,
                             unchecked_frac_of_attainable=s.ops / t_n / 1e12 / PEAK_INT8_TOPS / att))
            del Lc, Ln
        return rows
    int8_out = dict(note="config-2 layers with the fused int8 epilog (int8 ConvOut), unchecked and FusedOCG in the library's form per layer",
                    n32=i8_rows(layers), n256=i8_rows(big))
    torch.cuda.empty_cache()

    # ---- the memory-bound 1x1 layers (64 images), unchecked, int32 ConvOut: achieved HBM rate on buffer sets
    # that together exceed twice the 256 MB last-level cache, so that no launch finds its operands cached ----
    c3 = []
    for i, s in enumerate(CONFIG3):
        sets3 = [Int8Layer(s, seed_for(3, i), int(Variant.NONE))]
        per = sets3[0].x.numel() + 4 * sets3[0].y.numel()
        while per * len(sets3) < (600 << 20) and len(sets3) < 12:
            sets3.append(Int8Layer(s, seed_for(3, i) + len(sets3), int(Variant.NONE)))
        t_rot = event_time(lambda: [o.run() for o in sets3], reps=4, replays=5) / len(sets3)
        t_hot = event_time(sets3[0].run)
        nbytes = s.min_bytes(1, 1, 4)
        c3.append(dict(layer=s.name, gop=s.ops / 1e9, min_bytes_i32=nbytes, buffer_sets=len(sets3), unchecked_us=t_rot * 1e6,
                       hbm_gbs=nbytes / t_rot / 1e9, frac_of_hbm_peak=nbytes / t_rot / 1e9 / PEAK_HBM_GBS,
                       cache_resident_us=t_hot * 1e6, tops=s.ops / t_rot / 1e12))
        del sets3
        torch.cuda.empty_cache()

    # ---- the machine's own ceilings (library probes): matrix instruction loop, fill, copy ----
    scratch = torch.empty((1 << 30,), dtype=torch.uint8, device=dev)
    half = scratch[: 1 << 29], scratch[1 << 29:]
    iters = 4000
    t_mfma = event_time(lambda: abed.probe(0, scratch, iters=iters), reps=2, replays=3)
    t_fill = event_time(lambda: abed.probe(1, scratch), reps=2, replays=3)
    t_copy = event_time(lambda: abed.probe(2, half[0], half[1]), reps=2, replays=3)
    peaks = dict(mfma_int8_tops=256 * 8 * iters * 16 * 32768 / t_mfma / 1e12, fill_gbs=(1 << 30) / t_fill / 1e9,
                 copy_gbs_read_plus_write=2 * (1 << 29) / t_copy / 1e9,
                 note="measured here with the library's probes: register-resident v_mfma_i32_16x16x64_i8 loop on all CUs; 1 GiB fill; 512 MiB copy (read + write bytes)")
    del scratch, half

    ovh = lambda t: 100.0 * (t / t_unchecked - 1.0)
    out = dict(metric="checked conv TOPS (int8) and ABED overhead % vs unchecked and vs duplication",
               value=total_ops / t_checked / 1e12, unit="TOPS", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=t_checked * 1e3, ms_per_step_samples=[t * 1e3 for t in checked_samples],
               ms_per_step_eager_launch=t_checked_eager * 1e3,
               launch="HIP graph replay of 10 steps; median of 5 timed runs of `steps` steps", higher_is_better=True, scaling="weak", vs_baseline=None,
               dtype="int8 (int32 accumulate)", data="synthetic",
               config=dict(workload="configs[1]: four ResNet-50-shaped int8 3x3 layers, N=32, s1 p1, C=K=64@56, 128@28, 256@14, 512@7; "
                                    "variant FusedOCG, int32 ConvOut; per layer the form the library's tile rule prefers",
                           fused_form_per_layer=dict(zip([s.name for s in layers], forms)), gop_per_step=total_ops / 1e9),
               unchecked_tops=total_ops / t_unchecked / 1e12, duplicate_tops=total_ops / t_dup / 1e12,
               overhead_pct_vs_unchecked=ovh(t_checked), duplicate_overhead_pct=ovh(t_dup), speedup_vs_duplicate=t_dup / t_checked,
               variant_overhead_pct={k: ovh(t) for k, t in t_var.items() if k != "NONE"},
               fic=dict(note="FIC scheme of Sec. 3.3 (input patch checksum . filter checksum == sum of ConvOut, int64): fused option = the input checksum workgroups ride in the convolution's launch, then a one-workgroup kernel adds up the partial sums and compares; fused_deferred = one such launch for the four layers at the end of the step; inloop_deferred = the input side formed in the convolution's main loop (the input fmaps are then not covered), comparisons deferred",
                        fused_tops=total_ops / t_fic[Variant.FUSED_OCG] / 1e12, fused_overhead_pct=ovh(t_fic[Variant.FUSED_OCG]),
                        fused_deferred_tops=total_ops / t_fic_deferred / 1e12, fused_deferred_overhead_pct=ovh(t_fic_deferred),
                        inloop_deferred_tops=total_ops / t_fic_inloop / 1e12, inloop_deferred_overhead_pct=ovh(t_fic_inloop),
                        unfused_tops=total_ops / t_fic[Variant.UNFUSED] / 1e12, unfused_overhead_pct=ovh(t_fic[Variant.UNFUSED])),
               single_scheme=dict(note="the headline path carries FC (Sec. 3.1) and the batch-checksum IC (Sec. 3.2 option 1) together; here each alone, FusedOCG, same form per layer",
                                  fc_only_tops=total_ops / t_single["fc_only"] / 1e12, fc_only_overhead_pct=ovh(t_single["fc_only"]),
                                  ic_only_tops=total_ops / t_single["ic_only"] / 1e12, ic_only_overhead_pct=ovh(t_single["ic_only"])),
               per_layer=per_layer, n256=n256, int8_out=int8_out, config3=dict(note="configs[2]: 1x1 layers, 64 images, unchecked, int32 ConvOut, rotating buffer sets", layers=c3),
               measured_peaks=peaks, roofline=roofline)

    if not args.no_cpu_baseline:
        from oracle import abed_oracle
        abed_oracle.build()
        ins = [int8_tensors(s, seed_for(2, i)) for i, s in enumerate(layers)]
        reps, t0 = 0, time.perf_counter()
        while True:                       # repeat whole steps until about 10 s of CPU work
            for s, (x, w) in zip(layers, ins):
                abed_oracle.abed_int8(x, w, s)
            reps += 1
            if time.perf_counter() - t0 > 10.0 or reps >= 200:
                break
        dt = (time.perf_counter() - t0) / reps
        out["cpu_baseline"] = dict(value=total_ops / dt / 1e12, unit="TOPS", cores=abed_oracle.num_threads(),
                                   kind="oracle", seconds=dt,
                                   sample="whole steps (all four layers: convolution + checksum convolutions + checks), repeated %d times" % reps)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
