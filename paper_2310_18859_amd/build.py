"""Build the HIP library in-tree: paper_2310_18859_amd/libsida_moe.so (gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsida_moe.so")
SOURCES = ["api.cpp", "plan.cpp", "sort_gather.hip", "grouped_ffn.hip", "combine.hip", "prefetch.hip", "hash_fn.hip", "debug.hip"]
HEADERS = ["ctx.h", "kernels.h", "tile_order.h"]


def _newest_source() -> float:
    files = [os.path.join(CSRC, f) for f in SOURCES + HEADERS] + [os.path.join(ROOT, "include", "sida_moe.h")]
    return max(os.path.getmtime(f) for f in files)


def is_current() -> bool:
    return os.path.exists(LIB) and os.path.getmtime(LIB) >= _newest_source()


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and is_current():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-x", "hip",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-command-line-argument",
           "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
           "-o", LIB] + os.environ.get("SIDA_EXTRA_HIPCC_FLAGS", "").split() + [os.path.join(CSRC, s) for s in SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the gfx feature name and says so once per file: drop that line
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if verbose or res.returncode != 0:
        sys.stderr.write(err + "\n")
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libsida_moe.so")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
