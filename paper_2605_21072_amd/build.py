"""Builds ``libqarvd.so`` (the gfx950 HIP library behind the C ABI) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
LIB = PKG / "libqarvd.so"
SOURCES = ["quant_act.hip", "quantize_weight.hip", "gemm_api.hip", "gemm_staged.hip", "gemm_dma.hip", "gemm_dma128.hip", "gemm_mfma16.hip", "probe.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# QARVD_PROF=1 in the environment compiles the GEMM kernels with their per-wave tick counters
FLAGS = (["-DQARVD_PROF=" + os.environ["QARVD_PROF"]] if os.environ.get("QARVD_PROF") else []) + [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",                      # the epilogue and the detector spell out every fma
    "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
]


def _compile(src: str, verbose: bool) -> Path:
    obj = CSRC / (Path(src).stem + ".o")
    cmd = [HIPCC, *FLAGS, "-c", str(CSRC / src), "-o", str(obj)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0 or verbose:
        sys.stderr.write(r.stdout + r.stderr)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s" % src)
    return obj


def build(verbose: bool = False) -> Path:
    """Compile every HIP source for gfx950 and link the shared library (always rebuilds)."""
    with ThreadPoolExecutor(max_workers=min(len(SOURCES), 8)) as ex:
        objs = list(ex.map(lambda s: _compile(s, verbose), SOURCES))
    tmp = LIB.with_suffix(".so.tmp%d" % os.getpid())
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *map(str, objs), "-o", str(tmp)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("link failed")
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
