"""Builds libanchor_attention.so, and bench.py's measurement aid libanchor_probe.so (HIP, gfx950 only),
next to the sources' package."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libanchor_attention.so")
PROBE_LIB = os.path.join(HERE, "libanchor_probe.so")
PROBE_SOURCE = os.path.join("probe", "mfma_probe.hip")
SOURCES = ["aa_api.hip", "aa_engine_bf16.hip", "aa_engine_bf16_pp.hip", "aa_engine_fp32.hip", "aa_select.hip"]
# The bf16 engines never produce a NaN that is used (masked scores are -inf, the guards around
# exp(-inf - -inf) select the other arm), so their row-max chains may drop NaN canonicalisation.
EXTRA = {"aa_engine_bf16.hip": ["-fno-honor-nans"], "aa_engine_bf16_pp.hip": ["-fno-honor-nans"]}
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wno-unused-command-line-argument",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = False) -> str:
    """Compile every kernel source and link the shared library; always recompiles."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(objdir, os.path.basename(src).replace(".hip", ".o"))
        cmd = ["hipcc", *FLAGS, *EXTRA.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s" % (src, r.stderr))
        if verbose:
            sys.stderr.write(r.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(compile_one, SOURCES + [PROBE_SOURCE]))
    for lib, parts in ((LIB, objs[:-1]), (PROBE_LIB, objs[-1:])):
        r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *parts],
                           capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
