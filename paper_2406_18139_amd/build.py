"""Builds liblookm.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2406_18139_amd.build

hipcc cross-compiles without a GPU present.  Packed-fp32 instruction selection is switched off
for device code on purpose (hand-checked scalar fp32 arithmetic only).
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
OBJ = PKG / "_build"
LIB = PKG / "liblookm.so"

SOURCES = ["api.hip", "score_generic.hip", "score_mfma.hip", "select.hip", "nearest_generic.hip", "nearest_mfma.hip",
           "merge.hip", "decode.hip", "probe.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]


def _compile(src: str) -> Path:
    obj = OBJ / (src + ".o")
    cmd = [HIPCC, *FLAGS, *os.environ.get("LOOKM_EXTRA_FLAGS", "").split(), "-c", str(CSRC / src), "-o", str(obj)]
    p = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in p.stderr.splitlines() if "not a recognized feature" not in l)
    if p.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> Path:
    OBJ.mkdir(exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB.with_suffix(f".so.tmp{os.getpid()}")
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *map(str, objs), "-o", str(tmp)])
    os.replace(tmp, LIB)
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build()
