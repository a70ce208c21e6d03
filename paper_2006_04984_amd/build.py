"""Builds libabed.so (HIP, gfx950 only) in-tree: python -m paper_2006_04984_amd.build"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(os.path.dirname(HERE), "_build")
LIB = os.path.join(HERE, "libabed.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# ABED_STAGES=<n> and ABED_ENABLE_DBG=1 in the environment build experiment variants (pipeline depth; the
# ABED_DBG run-time switch that cuts the kernel short for timing breakdowns, absent from normal builds)
FLAGS = (["-DABED_STAGES=" + os.environ["ABED_STAGES"]] if "ABED_STAGES" in os.environ else []) + \
        (["-DABED_ENABLE_DBG"] if os.environ.get("ABED_ENABLE_DBG") else []) + ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]

UNITS = [("abed_api.hip", [], "abed_api.o"),
         ("conv_dispatch.hip", [], "conv_dispatch.o")] + \
        [("conv_inst.hip", ["-DINST_WK=%d" % wk, "-DINST_KG=%d" % kg], "conv_wk%d_kg%d.o" % (wk, kg))
         for kg in (1, 2, 4) for wk in (9, 8, 5, 4, 1)] + \
        [("conv_box_inst.hip", ["-DBOX_XCH=%d" % x], "conv_box_x%d.o" % x) for x in (8, 4, 2, 1, 0)] + \
        [("conv_img_inst.hip", [], "conv_img.o")]


def _compile(unit):
    src, defs, obj = unit
    cmd = [HIPCC] + FLAGS + defs + ["-c", os.path.join(CSRC, src), "-o", os.path.join(BUILD, obj)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), err))
    return err


def build(jobs=8, verbose=False):
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        for msg in ex.map(_compile, UNITS):
            if verbose and msg.strip():
                print(msg, file=sys.stderr)
    objs = [os.path.join(BUILD, u[2]) for u in UNITS]
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
