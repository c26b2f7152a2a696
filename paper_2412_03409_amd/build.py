"""Builds libprefixkv.so (hand-written HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

HERE = Path(__file__).resolve().parent
CSRC = HERE / "csrc"
LIB = HERE / "libprefixkv.so"
SOURCES = ["api.hip", "importance.hip", "select.hip", "compact.hip", "decode.hip", "prefill.hip", "merge_feature.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=on",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]


def _compile(src: str) -> Path:
    obj = CSRC / (src + ".o")
    subprocess.check_call([HIPCC, *FLAGS, "-c", str(CSRC / src), "-o", str(obj)])
    return obj


def build(verbose: bool = True) -> Path:
    """Compile every source (always) and link the shared library."""
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB.with_suffix(".so.tmp%d" % os.getpid())
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(tmp),
                           *map(str, objs)])
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    build()
