"""Small driver for rocprofv3 runs (kernel trace or counters):

  rocprofv3 --kernel-trace --stats ... -- python3 -m paper_2006_04984_amd.profile_run --config 2 --layer 3 --variant 4
  rocprofv3 --pmc FETCH_SIZE ...      -- python3 -m paper_2006_04984_amd.profile_run ... --copy-mb 256

Launches the chosen int8 layer `--reps` times through abed_conv_int8 (or the entry point of another scheme, --scheme) (eager launches, so that every
dispatch is seen by the profiler) and, with --copy-mb, one device-to-device copy of that many MiB,
whose known size calibrates the FETCH_SIZE / WRITE_SIZE counters.
"""
import argparse

import torch

from .binding import Variant
from .evaluate import Int8Layer


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=2, choices=[2, 3])
    ap.add_argument("--layer", type=int, default=3)
    ap.add_argument("--variant", type=int, default=4)
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--int8-out", action="store_true")
    ap.add_argument("--copy-mb", type=int, default=0)
    ap.add_argument("--scheme", default="fcic", choices=["fcic", "fc", "ic", "fic", "fic_inloop", "ic2"],
                    help="fcic: filter + batch checksums (abed_conv_int8); fc / ic: one of the two alone; "
                         "fic: the scalar scheme (abed_fic_conv_int8); fic_inloop: the same with its input side formed in the main loop (abed_fic_inloop_conv_int8); ic2: IC option 2, K values (abed_ic2_conv_int8)")
    ap.add_argument("--batch", type=int, default=0, help="override the configuration's batch size")
    ap.add_argument("--local", action="store_true", help="checksums local to a workgroup (ABED_LOCAL, with --variant 4)")
    ap.add_argument("--img", action="store_true", help="unchecked 3x3 layers through the one-wave-per-SIMD kernel (sets ABED_IMG=1)")
    ap.add_argument("--img-clock", type=int, default=-1, metavar="DBG",
                    help="library built with ABED_ENABLE_DBG=1 only: run the --img kernel with ABED_DBG=<DBG> (0: as is, 1: the loop's "
                         "activation loads fetch nothing, 2: its filter loads, 3: both) and print the main loop's length in shader-clock "
                         "ticks and in real time, i.e. the shader clock under that load")
    args = ap.parse_args()
    if args.img or args.img_clock >= 0:
        import os
        os.environ["ABED_IMG"] = "1"
    clk = None
    if args.img_clock >= 0:
        clk = torch.zeros((2,), dtype=torch.int64, device="cuda:0")
        os.environ["ABED_DBG"] = str(args.img_clock)
        os.environ["ABED_DBG_PTR"] = str(clk.data_ptr())
    from synth import CONFIG2, CONFIG3, seed_for
    s = {2: CONFIG2, 3: CONFIG3}[args.config][args.layer]
    if args.batch:
        import dataclasses
        s = dataclasses.replace(s, N=args.batch)
    if args.scheme == "fic":
        from .evaluate import FicLayer
        L = FicLayer(s, seed_for(args.config, args.layer), Variant(args.variant), epilogue=args.int8_out)
    elif args.scheme == "fic_inloop":
        from .evaluate import FicInloopLayer
        L = FicInloopLayer(s, seed_for(args.config, args.layer), epilogue=args.int8_out)
    elif args.scheme == "ic2":
        from .evaluate import Ic2Layer
        L = Ic2Layer(s, seed_for(args.config, args.layer), Variant(args.variant), epilogue=args.int8_out)
    else:
        from . import binding as abed
        only = {"fcic": 0, "fc": abed.ONLY_FC, "ic": abed.ONLY_IC}[args.scheme] if args.variant in (1, 2, 3, 4, 5) else 0
        L = Int8Layer(s, seed_for(args.config, args.layer), args.variant | only | (abed.LOCAL if args.local else 0), epilogue=args.int8_out)
    for _ in range(args.reps):
        L.run()
    torch.cuda.synchronize()
    if clk is not None:
        t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0.record()
        for _ in range(args.reps):
            L.run()
        t1.record()
        torch.cuda.synchronize()
        ticks, rt = (int(v) for v in clk.cpu())
        print("main loop of workgroup 0: %d shader-clock ticks in %.2f us -> %.3f GHz; %.1f us per launch (events, eager launches)"
              % (ticks, rt / 100.0, ticks / (rt * 10.0), t0.elapsed_time(t1) * 1e3 / args.reps))
    if args.copy_mb:
        a = torch.empty((args.copy_mb << 20,), dtype=torch.uint8, device="cuda:0")
        b = torch.empty_like(a)
        a.fill_(1)
        torch.cuda.synchronize()
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
    if args.scheme == "fic_inloop":
        print("profiled", s.name, "FIC, input side in the main loop, flag", int(L.flag.item()))
    elif args.scheme == "fic":
        print("profiled", s.name, "FIC variant", args.variant, "flag", int(L.flag.item()))
    elif args.scheme == "ic2":
        print("profiled", s.name, "IC option 2 variant", args.variant, "flags", int(L.flags.abs().max().item()))
    else:
        print("profiled", s.name, "variant", args.variant, "grid", L.lay.grid_m, L.lay.grid_b, L.lay.grid_n,
              "flags", int(L.flags.abs().max().item()))


if __name__ == "__main__":
    main()
