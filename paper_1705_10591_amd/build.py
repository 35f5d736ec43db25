"""Build libdconv.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
LIB = PKG / "libdconv.so"
# standalone microbenchmarks, no part of the library: LDS access widths (the paper's bank-width
# experiment) and the hardware rates that shaped the kernels
LDS_BENCH = PKG / "lds_width_bench"
HW_BENCH = PKG / "hw_bench"
BUILD = PKG / "_build"
# (source, extra flags, object name); the general-case kernels are compiled once per filter side
SOURCES = [("api.hip", [], "api"), ("simple.hip", [], "simple"), ("single.hip", [], "single"), ("single_fewfilters.hip", [], "single_fewfilters"),
           *[("single_multi_inst.hip", [f"-DDCONV_C={c}"], f"single_c{c}") for c in (2, 3, 4)],
           ("general.hip", [], "general"), ("general_fewfilters.hip", [], "general_fewfilters")] + \
          [("general_few_inst.hip", [f"-DDCONV_F={f}"], f"general_few_f{f}") for f in range(1, 8)] + \
          [("general_inst.hip", [f"-DDCONV_F={f}"], f"general_f{f}") for f in range(1, 33)] + \
          [("half.hip", [], "half")] + \
          [("half_inst.hip", [f"-DDCONV_F={f}"], f"half_f{f}") for f in range(1, 33)]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# Packed fp32 VALU forms are switched off for all device code (the host pass
# prints a harmless "not a recognized feature" note for the same flag).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # matrix-core results stay in ordinary VGPRs: no copies out of the
         # accumulator file before they are stored
         "-mllvm", "-amdgpu-mfma-vgpr-form",
         "-Wall", "-Wno-unused-command-line-argument"]


def _compile(item) -> Path:
    src, extra, name = item
    obj = BUILD / (name + ".o")
    cmd = [HIPCC, *FLAGS, *extra, "-c", str(CSRC / src), "-o", str(obj)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stderr[-4000:]}")
    return obj


def build(verbose: bool = False) -> Path:
    """Compile every HIP source and link libdconv.so; always recompiles."""
    BUILD.mkdir(exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = PKG / f"libdconv.tmp{os.getpid()}.so"
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(tmp), *map(str, objs)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr[-4000:]}")
    os.replace(tmp, LIB)
    # The microbenchmarks are no part of the library: bench.py quotes hw_bench's rates as measured
    # peaks when it is there, and the tests that run them skip when they are not.  A failure to
    # build one is reported and does not fail the library's build.
    built = []
    for exe in (LDS_BENCH, HW_BENCH):
        cmd = [HIPCC, *[f for f in FLAGS if f != "-fPIC"], str(CSRC / (exe.name + ".hip")), "-o", str(exe)]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            exe.unlink(missing_ok=True)
            print(f"warning: hipcc failed for {exe.name}.hip (the library is built):\n{r.stderr[-2000:]}",
                  file=sys.stderr)
        else:
            built.append(exe.name)
    if verbose:
        print(f"built {LIB}" + "".join(f", {n}" for n in built))
    return LIB


if __name__ == "__main__":  # python -m paper_1705_10591_amd.build
    build(verbose=True)
    sys.exit(0)
