"""Build libflashblock.so (hand-written HIP for gfx950) and libfbcalib.so (the benchmark's calibration
kernels: read and MFMA ceilings, a plain copy) in-tree with hipcc.

    python -m paper_2602_05305_amd.build [--force]

The libraries are written next to this file so that they travel with the source tree; nothing is
installed.  Objects go to paper_2602_05305_amd/_build/ (ignored by git).
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libflashblock.so")
CALIB_LIB = os.path.join(HERE, "libfbcalib.so")
CALIB_SOURCES = ["fb_calib.hip"]
SOURCES = ["fb_api.hip", "fb_attn_f32.hip", "fb_attn_bf16.hip", "fb_stream_bf16.hip", "fb_aux.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # the direct-to-LDS loads set M0 from inline assembly and say so in the clobber list
         "-Wno-inline-asm",
         # keep the compiler from forming packed fp32 VALU ops
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l).strip()
    if err:
        sys.stderr.write(err + "\n")
    return obj


def build(force: bool = True) -> str:
    """Compile every HIP source for gfx950 and link the shared library.  Returns its path."""
    os.makedirs(OBJ, exist_ok=True)
    if not force and os.path.exists(LIB) and os.path.exists(CALIB_LIB):
        newest = max(os.path.getmtime(os.path.join(CSRC, f)) for f in os.listdir(CSRC))
        newest = max(newest, os.path.getmtime(os.path.join(HERE, "..", "include", "flashblock.h")))
        if min(os.path.getmtime(LIB), os.path.getmtime(CALIB_LIB)) >= newest:
            return LIB
    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(_compile, SOURCES + CALIB_SOURCES))
    for lib, lobjs in ((LIB, objs[:len(SOURCES)]), (CALIB_LIB, objs[len(SOURCES):])):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *lobjs]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    return LIB


if __name__ == "__main__":
    print(build(force=True))
