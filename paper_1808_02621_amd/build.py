"""Builds libpx.so (the HIP library behind include/px.h) for gfx950, in-tree.

    python -m paper_1808_02621_amd.build

Every source is compiled with hipcc into an object next to it and linked into
``paper_1808_02621_amd/libpx.so``.  There is no other backend and no fallback.
"""

from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys
from typing import List, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIBRARY = os.path.join(HERE, "libpx.so")
SOURCES = ["px_core.hip", "px_coalesce.hip", "px_partition.hip", "px_apply.hip", "px_dense.hip", "px_lookup.hip", "px_costmodel.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    # packed-FP32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", INCLUDE, "-I", CSRC,
]


def _compile(src: str, extra: Sequence[str]) -> str:
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, err))
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_library(extra_flags: Sequence[str] = (), output: str = LIBRARY) -> str:
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs: List[str] = list(pool.map(lambda s: _compile(s, extra_flags), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", output, *objs]
    subprocess.run(cmd, check=True)
    return output


if __name__ == "__main__":
    print(build_library())
