"""Builds libtt_emb.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
SOURCES = ["tt_emb_index.hip", "tt_emb_compute.hip", "tt_emb_mfma.hip", "tt_emb_calib.hip",
           "tt_emb_api.hip"]
LIB = os.path.join(HERE, "libtt_emb.so")


def lib_path() -> str:
    return LIB


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile every HIP source into one shared library, in-tree."""
    cmd = ["hipcc", *extra_flags, "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
           "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
           # packed fp32 instructions are kept out of the generated code
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    log = "\n".join(l for l in (res.stdout + res.stderr).splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + log)
    if verbose and log.strip():
        print(log)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(verbose=True, extra_flags=tuple(sys.argv[1:])))
