"""Builds the HIP library in-tree: csrc/*.hip -> liboz_mi355x.so (gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liboz_mi355x.so")
PROBE_LIB = os.path.join(HERE, "liboz_probe.so")      # measurement probes: separate from the product library
PROBE_SOURCES = ["oz_probe.hip"]
SOURCES = ["oz_api.hip", "oz_scan.hip", "oz_esc.hip", "oz_slice.hip", "oz_gemm_i8.hip",
           "oz_recompose.hip", "oz_dgemm_f64.hip", "oz_complex.hip"]
# packed FP32 instructions are switched off for all device code (known-bad on the test machines)
# -ffp-contract=off: the FP64 epilogues round every product and sum separately, as the header specifies;
# hipcc's default would fuse a*b + c into one rounding.
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-command-line-argument",
         "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]
# per-source additions.  oz_esc.hip: MFMA results are consumed by the vector ALU right away, so they
# are kept in ordinary VGPRs (the default puts them in accumulation registers and copies them out).
SOURCE_FLAGS = {"oz_esc.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


def _compile(src: str, extra=()) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, *SOURCE_FLAGS.get(src, []), *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
    noise = ("packed-fp32-ops", "is not a recognized feature")
    for line in r.stderr.splitlines():
        if line.strip() and not any(n in line for n in noise):
            print(line, file=sys.stderr)
    return obj


def _link(lib: str, objs) -> None:
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))


def build_library(verbose: bool = True, extra=()) -> str:
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + len(PROBE_SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, extra), SOURCES + PROBE_SOURCES))
    _link(LIB, objs[:len(SOURCES)])
    _link(PROBE_LIB, objs[len(SOURCES):])
    if verbose:
        print("built", LIB)
        print("built", PROBE_LIB)
    return LIB


if __name__ == "__main__":
    build_library(extra=sys.argv[1:])
