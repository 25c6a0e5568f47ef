"""Builds the gfx950 shared library (csrc/*.hip -> libla_hip.so) with hipcc.

hipcc cross-compiles without a GPU, so this runs anywhere the ROCm toolchain is
installed.  The library is kept in-tree next to this file.
"""
from __future__ import annotations

import concurrent.futures
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libla_hip.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _deps_mtime():
    files = sources() + glob.glob(os.path.join(CSRC, "*.h")) + \
        glob.glob(os.path.join(HERE, "..", "include", "*.h"))
    return max(os.path.getmtime(f) for f in files)


def is_current() -> bool:
    return os.path.exists(LIB) and os.path.getmtime(LIB) >= _deps_mtime()


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.basename(src)[:-4] + ".o")
    subprocess.run([HIPCC, *FLAGS, "-c", src, "-o", obj], check=True, cwd=CSRC,
                   stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    return obj


def build_library(force: bool = True, jobs: int = 6) -> str:
    """Compile every HIP source for gfx950 and link libla_hip.so.  With
    force=False an up-to-date library is left alone."""
    if not force and is_current():
        return LIB
    os.makedirs(OBJ, exist_ok=True)
    try:
        with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
            objs = list(ex.map(_compile, sources()))
        subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    except subprocess.CalledProcessError as e:  # show the compiler's message
        raise RuntimeError(f"hipcc failed:\n{e.stdout.decode(errors='replace')}") from e
    return LIB


if __name__ == "__main__":
    print(build_library(force=True))
