"""Builds ``csrc/libhelix_attn.so`` for gfx950 with hipcc (in-tree, no JIT cache)."""
from __future__ import annotations

import pathlib
import subprocess
import sys

CSRC = pathlib.Path(__file__).resolve().parent / "csrc"
LIB = CSRC / "libhelix_attn.so"
SOURCES = ["api.hip", "fwd.hip", "bwd.hip", "bwd_dkdv.hip", "bwd_dq.hip"]
# Packed fp32 VALU ops are switched off for the device pass; the host pass does not know
# the feature and says so in a harmless warning.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = False) -> pathlib.Path:
    cmd = ["hipcc", *FLAGS, *[str(CSRC / s) for s in SOURCES], "-o", str(LIB)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
