"""Build the HIP library for gfx950 in-tree: ``python -m paper_2407_11062_amd.build``."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.environ.get("EQAT_OBJ_DIR", os.path.join(HERE, "_build"))
LIB = os.environ.get("EQAT_LIB_OUT", os.path.join(HERE, "libeqat.so"))
SOURCES = ["api.hip", "quant.hip", "gemm_f32.hip", "gemm_mfma.hip", "gemv.hip", "train_step.hip"]
# measurement aids of bench.py (a bare MFMA loop, a plain copy): a library of their own, not part of the product
PEAKS_SOURCE = "bench_peaks.hip"
PEAKS_LIB = os.environ.get("EQAT_PEAKS_LIB_OUT", os.path.join(HERE, "libeqat_peaks.so"))
FLAGS = [*os.environ.get("EQAT_EXTRA_FLAGS", "").split(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(_compile, SOURCES + [PEAKS_SOURCE]))
    for out, parts in ((LIB, objs[:-1]), (PEAKS_LIB, objs[-1:])):
        r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *os.environ.get("EQAT_EXTRA_LINK_FLAGS", "").split(),
                            *parts, "-o", out],
                           capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
        if verbose:
            print(f"built {out}")
    return LIB


if __name__ == "__main__":
    build()
