#!/usr/bin/env python3
"""Benchmark of the ABED convolution hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input:
the four ResNet-50-shaped int8 3x3 layers (batch 32, stride 1, pad 1; C=K=64 at
56x56, 128 at 28x28, 256 at 14x14, 512 at 7x7), each through abed_conv_int8 with
the fully fused variant (input checksum generation + augmented convolution that
reduces, compares and flags in its epilogue), int32 ConvOut as output.  Inputs
are resident in HBM before the timed region.  TOPS count the real convolution
work only (2*N*P*Q*K*C*R*S); checksum work is overhead and is never credited.

Prints ONE JSON line (see the keys below).  Extra keys report the unchecked
kernel, the duplication baseline, every variant's overhead and per-layer times.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0     # MI355X dense int8 MFMA peak, TOP/s
PEAK_HBM_GBS = 8000.0
# HBM bytes per launch of the checked convolution kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs scaled by a copy of known size (profiles/conv_int8_checked_config2.md); None where not measured.
MEASURED_TRAFFIC_BYTES = {"3x3_c64_56": 16.7e6 + 38.3e6, "3x3_c128_28": 12.8e6 + 20.9e6,
                          "3x3_c256_14": 12.7e6 + 9.9e6, "3x3_c512_7": 16.2e6 + 7.9e6}


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
    from synth import CONFIG2, int8_tensors, seed_for

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    abed.lib()  # fails loudly if libabed.so is not built
    dev = "cuda:0"
    layers = CONFIG2
    total_ops = sum(s.ops for s in layers)

    class Layer:
        pass

    def setup(s, idx, variant, int8_out=False):
        L = Layer()
        L.s, L.variant = s, int(variant)                  # may carry abed.ONLY_FC / abed.ONLY_IC
        L.desc = abed.desc_from_shape(s)
        L.lay = abed.get_layout(L.desc, 0, L.variant)
        x, w = int8_tensors(s, seed_for(2, idx))
        L.x = torch.from_numpy(x).to(dev)
        L.w = torch.from_numpy(w).to(dev)
        L.y = torch.empty((s.N, s.P, s.Q, s.K), dtype=torch.int32, device=dev)
        L.y2 = torch.empty_like(L.y) if L.variant == int(Variant.DUPLICATE) else None
        L.flags = torch.zeros((max(1, L.lay.n_flag_words),), dtype=torch.int32, device=dev)
        L.ws = torch.zeros((max(256, L.lay.workspace_bytes),), dtype=torch.uint8, device=dev)
        abed.workspace_init(L.ws)
        L.wchk = torch.empty((L.lay.d_f, s.R, s.S, s.C), dtype=torch.int8, device=dev)
        L.xchk = torch.empty((L.lay.d_i, s.H, s.W, s.C), dtype=torch.int8, device=dev)
        if L.lay.d_f:
            abed.filter_prepare_int8(L.desc, L.w, L.wchk)  # offline step, not timed (Sec. 3.4: filter checksums are made offline)
        return L

    def setup_fic(s, idx, variant):
        """Buffers for the FIC scheme (Sec. 3.3) on the same layer and data."""
        L = Layer()
        L.s, L.variant = s, Variant(variant)
        L.desc = abed.desc_from_shape(s)
        lay = abed.fic_get_layout(L.desc, L.variant)
        x, w = int8_tensors(s, seed_for(2, idx))
        L.x = torch.from_numpy(x).to(dev)
        L.w = torch.from_numpy(w).to(dev)
        L.y = torch.empty((s.N, s.P, s.Q, s.K), dtype=torch.int32, device=dev)
        L.wsum = torch.empty((s.R, s.S, s.C), dtype=torch.int32, device=dev)
        L.xrows = torch.empty((lay.xrows_parts, s.H, s.S, s.C), dtype=torch.int32, device=dev)
        L.result = torch.zeros((2,), dtype=torch.int64, device=dev)
        L.flag = torch.zeros((1,), dtype=torch.int32, device=dev)
        L.ws = torch.zeros((max(256, lay.workspace_bytes),), dtype=torch.uint8, device=dev)
        abed.workspace_init(L.ws)
        abed.fic_filter_prepare_int8(L.desc, L.w, L.wsum)   # offline step, not timed
        return L

    def setup_fic_inloop(s, idx):
        """Buffers for FIC with the input side formed in the convolution's main loop, same layer and data."""
        L = Layer()
        L.s, L.variant = s, abed.FIC_INLOOP
        L.desc = abed.desc_from_shape(s)
        lay = abed.fic_inloop_get_layout(L.desc)
        x, w = int8_tensors(s, seed_for(2, idx))
        L.x = torch.from_numpy(x).to(dev)
        L.w = torch.from_numpy(w).to(dev)
        L.y = torch.empty((s.N, s.P, s.Q, s.K), dtype=torch.int32, device=dev)
        L.wdig = torch.empty((lay.wdig_bytes,), dtype=torch.int8, device=dev)
        L.ws = torch.zeros((max(256, lay.workspace_bytes),), dtype=torch.uint8, device=dev)
        abed.workspace_init(L.ws)
        abed.fic_inloop_filter_prepare_int8(L.desc, L.w, L.wdig)   # offline step, not timed
        return L

    def run_fic(L):
        abed.fic_conv_int8(L.desc, L.x, L.w, L.wsum, L.xrows, True, L.y, L.variant, L.result, L.flag, workspace=L.ws)

    def run_layer(L, compute_xchk=True):
        abed.conv_int8(L.desc, L.x, L.w, L.wchk, L.xchk, compute_xchk, L.y, L.variant, flags=L.flags,
                       workspace=L.ws, y2=L.y2)

    stream = torch.cuda.Stream()

    def time_steps(fn, steps, warmup, per_graph=10):
        """K steps, launched as replays of a HIP graph that holds `per_graph` steps (the launches of a
        step are tiny next to the host's cost of issuing them one by one).  Returns seconds per step."""
        if steps % per_graph:
            per_graph = 1
        with torch.cuda.stream(stream):
            for _ in range(max(1, warmup // 2)):
                fn()                                  # eager warm-up (also one-time function attributes)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for _ in range(per_graph):
                    fn()
            for _ in range(max(1, warmup // per_graph)):
                graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps // per_graph):
                graph.replay()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / steps

    def time_eager(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    def event_time(fn, reps=20, replays=10):
        """Average duration of one call of fn (its kernel launches), from HIP events on the stream the
        library launches on, around replays of a graph of `reps` calls."""
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(stream):
            fn()
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for _ in range(reps):
                    fn()
            graph.replay()
            torch.cuda.synchronize()
            e0.record(stream)
            for _ in range(replays):
                graph.replay()
            e1.record(stream)
            torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / (reps * replays)

    sets = {}
    wanted = [Variant.FUSED_OCG, Variant.NONE, Variant.DUPLICATE]
    if args.variants == "all":
        wanted += [Variant.UNFUSED, Variant.FUSED_WRITE, Variant.FUSED_PARTIAL_REDUCTION, Variant.FUSED_IOCG]
    for v in wanted:
        sets[v] = [setup(s, i, v) for i, s in enumerate(layers)]

    def step_of(v):
        Ls = sets[v]
        return lambda: [run_layer(L) for L in Ls]

    # ---- the timed region: K steps of the fully fused checked path ----
    t_checked = time_steps(step_of(Variant.FUSED_OCG), args.steps, args.warmup)
    # clean run => no flag may be set
    for L in sets[Variant.FUSED_OCG]:
        assert int(L.flags.abs().max().item()) == 0, "error flag set on a fault-free run"
    # the other variants: same protocol, fewer steps for the slow ones
    t_var = {Variant.FUSED_OCG: t_checked}
    for v in wanted[1:]:
        t_var[v] = time_steps(step_of(v), max(20, args.steps // 2 // 10 * 10), max(10, args.warmup // 2))
    t_unchecked = t_var[Variant.NONE]
    # the paper's own FIC scheme (one scalar check per layer), fused and unfused options
    fic_sets = {v: [setup_fic(s, i, v) for i, s in enumerate(layers)] for v in (Variant.FUSED_OCG, Variant.UNFUSED)}
    t_fic = {}
    for v, Ls in fic_sets.items():
        t_fic[v] = time_steps(lambda: [run_fic(L) for L in Ls], max(20, args.steps // 2 // 10 * 10), max(10, args.warmup // 2))
        for L in Ls:
            r = L.result.cpu().numpy()
            assert int(L.flag.item()) == 0 and r[0] == r[1], "FIC mismatch on a fault-free run"
    # each of the two checksum schemes of the headline path alone (Table 1 of Sec. 3.4), FusedOCG
    t_single = {}
    for name, bit in (("fc_only", abed.ONLY_FC), ("ic_only", abed.ONLY_IC)):
        Ls = [setup(s, i, int(Variant.FUSED_OCG) | bit) for i, s in enumerate(layers)]
        t_single[name] = time_steps(lambda: [run_layer(L) for L in Ls], max(20, args.steps // 2 // 10 * 10), max(10, args.warmup // 2))
        for L in Ls:
            assert int(L.flags.abs().max().item()) == 0, "error flag set on a fault-free run"
        del Ls
    # FIC fused with the comparisons of the four layers deferred to one launch at the end of the step
    Ls = fic_sets[Variant.FUSED_OCG]
    res_all = torch.zeros((len(Ls), 2), dtype=torch.int64, device=dev)
    flag_all = torch.zeros((len(Ls),), dtype=torch.int32, device=dev)

    def fic_deferred_step():
        for L in Ls:
            abed.fic_conv_int8(L.desc, L.x, L.w, L.wsum, L.xrows, True, L.y, L.variant, None, None, workspace=L.ws)
        abed.fic_verify([L.desc for L in Ls], [L.variant for L in Ls], [L.ws for L in Ls], res_all, flag_all)
    t_fic_deferred = time_steps(fic_deferred_step, max(20, args.steps // 2 // 10 * 10), max(10, args.warmup // 2))
    assert int(flag_all.abs().max().item()) == 0 and bool((res_all[:, 0] == res_all[:, 1]).all().item()), "FIC mismatch on a fault-free run"
    # FIC with the input side formed in the main loop (no second pass over x), comparisons deferred the same way
    Li = [setup_fic_inloop(s, i) for i, s in enumerate(layers)]

    def fic_inloop_step():
        for L in Li:
            abed.fic_inloop_conv_int8(L.desc, L.x, L.w, L.wdig, L.y, None, None, workspace=L.ws)
        abed.fic_verify([L.desc for L in Li], [L.variant for L in Li], [L.ws for L in Li], res_all, flag_all)
    t_fic_inloop = time_steps(fic_inloop_step, max(20, args.steps // 2 // 10 * 10), max(10, args.warmup // 2))
    assert int(flag_all.abs().max().item()) == 0 and bool((res_all[:, 0] == res_all[:, 1]).all().item()), "FIC (in-loop) mismatch on a fault-free run"
    del Li
    t_checked_eager = time_eager(step_of(Variant.FUSED_OCG), max(20, args.steps // 4), 5)
    t_dup = t_var[Variant.DUPLICATE]

    # ---- per-layer kernel durations with events on the launch stream ----
    per_layer = []
    for i, s in enumerate(layers):
        Lc, Ln = sets[Variant.FUSED_OCG][i], sets[Variant.NONE][i]
        run_layer(Lc, True)
        t_conv_chk = event_time(lambda: run_layer(Lc, False))       # augmented conv kernel alone
        t_all_chk = event_time(lambda: run_layer(Lc, True))         # ICG + augmented conv
        t_conv_plain = event_time(lambda: run_layer(Ln, False))
        per_layer.append(dict(layer=s.name, gop=s.ops / 1e9, unchecked_us=t_conv_plain * 1e6,
                              checked_conv_us=t_conv_chk * 1e6, checked_total_us=t_all_chk * 1e6,
                              unchecked_tops=s.ops / t_conv_plain / 1e12, checked_tops=s.ops / t_all_chk / 1e12,
                              overhead_pct=100.0 * (t_all_chk / t_conv_plain - 1.0),
                              min_bytes_i32=s.min_bytes(1, 1, 4),
                              tile=[Lc.lay.tile_pixels, Lc.lay.tile_batch, Lc.lay.tile_n],
                              grid=[Lc.lay.grid_m, Lc.lay.grid_b, Lc.lay.grid_n]))
    dom = max(per_layer, key=lambda r: r["checked_conv_us"])
    dom_shape = layers[[r["layer"] for r in per_layer].index(dom["layer"])]
    achieved = dom_shape.ops / (dom["checked_conv_us"] * 1e-6) / 1e12
    roofline = dict(bound="mfma", kernel="conv_i8_kernel (augmented) on " + dom["layer"], achieved=achieved,
                    peak=PEAK_INT8_TOPS, unit="TFLOP/s", op="int8 multiply-add counted as 2 ops",
                    frac=achieved / PEAK_INT8_TOPS, traffic=MEASURED_TRAFFIC_BYTES.get(dom["layer"]),
                    algorithmic_bytes=dom["min_bytes_i32"],
                    ops_per_launch=dom_shape.ops, avg_launch_us=dom["checked_conv_us"])

    out = dict(metric="checked conv TOPS (int8) and ABED overhead % vs unchecked and vs duplication",
               value=total_ops / t_checked / 1e12, unit="TOPS", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=t_checked * 1e3, ms_per_step_eager_launch=t_checked_eager * 1e3,
               launch="HIP graph replay of 10 steps (8 kernel launches per step)", higher_is_better=True, scaling="weak", vs_baseline=None,
               dtype="int8 (int32 accumulate)", data="synthetic",
               config=dict(workload="configs[1]: four ResNet-50-shaped int8 3x3 layers, N=32, s1 p1, "
                                    "C=K=64@56, 128@28, 256@14, 512@7; variant FusedOCG (ICG + augmented conv), int32 ConvOut",
                           gop_per_step=total_ops / 1e9),
               unchecked_tops=total_ops / t_unchecked / 1e12,
               duplicate_tops=total_ops / t_dup / 1e12,
               overhead_pct_vs_unchecked=100.0 * (t_checked / t_unchecked - 1.0),
               duplicate_overhead_pct=100.0 * (t_dup / t_unchecked - 1.0),
               speedup_vs_duplicate=t_dup / t_checked,
               variant_overhead_pct={v.name: 100.0 * (t / t_unchecked - 1.0) for v, t in t_var.items() if v != Variant.NONE},
               fic=dict(note="FIC scheme of Sec. 3.3 (input patch checksum . filter checksum == sum of ConvOut, int64): "
                             "fused option = the input checksum workgroups ride in the convolution's launch, then a one-workgroup kernel adds up the partial sums and compares; fused_deferred = one such launch for the four layers at the end of the step; inloop_deferred = the input side formed in the convolution's main loop from the tiles it loads (no second pass over x; the input fmaps are then not covered), comparisons deferred",
                        fused_tops=total_ops / t_fic[Variant.FUSED_OCG] / 1e12,
                        fused_overhead_pct=100.0 * (t_fic[Variant.FUSED_OCG] / t_unchecked - 1.0),
                        fused_deferred_tops=total_ops / t_fic_deferred / 1e12,
                        fused_deferred_overhead_pct=100.0 * (t_fic_deferred / t_unchecked - 1.0),
                        inloop_deferred_tops=total_ops / t_fic_inloop / 1e12,
                        inloop_deferred_overhead_pct=100.0 * (t_fic_inloop / t_unchecked - 1.0),
                        unfused_tops=total_ops / t_fic[Variant.UNFUSED] / 1e12,
                        unfused_overhead_pct=100.0 * (t_fic[Variant.UNFUSED] / t_unchecked - 1.0)),
               single_scheme=dict(note="the headline path carries FC (Sec. 3.1) and the batch-checksum IC (Sec. 3.2 option 1) together; here each alone, FusedOCG",
                                  fc_only_tops=total_ops / t_single["fc_only"] / 1e12,
                                  fc_only_overhead_pct=100.0 * (t_single["fc_only"] / t_unchecked - 1.0),
                                  ic_only_tops=total_ops / t_single["ic_only"] / 1e12,
                                  ic_only_overhead_pct=100.0 * (t_single["ic_only"] / t_unchecked - 1.0)),
               per_layer=per_layer, roofline=roofline)

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
