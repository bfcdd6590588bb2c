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


SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
             "-fno-sanitize-recover=undefined"]


def build_host_sanitized() -> Path:
    """The same library with AddressSanitizer and UndefinedBehaviorSanitizer on its HOST code only (argument
    validation, workspace layout, launch sequencing; device code is compiled as usual), for the CPU-side tests:
    paper_2406_18139_amd/_build/liblookm_san.so.  Load it with the clang runtime preloaded (see asan_runtime)."""
    OBJ.mkdir(exist_ok=True)
    objs = []
    for src in SOURCES:
        obj = OBJ / (src + ".san.o")
        flags = [f for f in FLAGS if f != "-O3"] + ["-O1", "-g"]
        p = subprocess.run([HIPCC, *flags, *SAN_FLAGS, "-c", str(CSRC / src), "-o", str(obj)], capture_output=True, text=True)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc (sanitized) failed for {src}:\n{p.stderr}")
        objs.append(obj)
    out = OBJ / "liblookm_san.so"
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *SAN_FLAGS, *map(str, objs), "-o", str(out)])
    return out


def asan_runtime() -> Path:
    """The shared AddressSanitizer runtime of the clang that hipcc drives (to be preloaded into the Python process)."""
    p = subprocess.run([HIPCC, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    path = Path(p.stdout.strip())
    if not path.is_absolute() or not path.exists():
        cands = sorted(Path("/opt/rocm/lib/llvm/lib/clang").glob("*/lib/linux/libclang_rt.asan-x86_64.so"))
        if not cands:
            raise FileNotFoundError("libclang_rt.asan-x86_64.so not found")
        path = cands[-1]
    return path


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
