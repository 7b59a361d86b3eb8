"""Builds ``csrc/libhelix_attn.so`` for gfx950 with hipcc (in-tree, no JIT cache)."""
from __future__ import annotations

import pathlib
import re
import subprocess
import sys

CSRC = pathlib.Path(__file__).resolve().parent / "csrc"
LIB = CSRC / "libhelix_attn.so"
SOURCES = ["api.hip", "fwd.hip", "bwd.hip", "bwd_dkdv.hip", "bwd_dkdv_pair.hip", "bwd_dq.hip", "linear.hip", "mfma_probe.hip"]
# Packed fp32 VALU ops are switched off for the device pass; the host pass does not know
# the feature and says so in a harmless warning.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def kernel_resources(remarks: str) -> dict:
    """{kernel: {"vgpr", "agpr", "scratch", "occupancy"}} from -Rpass-analysis=kernel-resource-usage output."""
    out, cur = {}, None
    keys = {"VGPRs": "vgpr", "AGPRs": "agpr", r"ScratchSize \[bytes/lane\]": "scratch", r"Occupancy \[waves/SIMD\]": "occupancy"}
    for line in remarks.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        for pat, key in keys.items():
            m = re.search(r" " + pat + r": (\d+)", line)
            if m and cur is not None:
                cur[key] = int(m.group(1))
    return out


def build(verbose: bool = False) -> pathlib.Path:
    """Compiles the library and refuses a build in which any kernel spills to scratch memory:
    the kernels are written to fit the register file (a non-inlined helper that takes the
    accumulators by reference once put them in scratch without any warning)."""
    cmd = ["hipcc", *FLAGS, "-Rpass-analysis=kernel-resource-usage", *[str(CSRC / s) for s in SOURCES], "-o", str(LIB)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    remark = re.compile(r"kernel-resource-usage|^\s*$|^\s*\d*\s*\|")   # remarks and the source lines they quote
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l and not remark.search(l))
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    usage = kernel_resources(res.stderr)
    spilled = {k: v for k, v in usage.items() if v.get("scratch", 0) > 0}
    if spilled:
        LIB.unlink(missing_ok=True)
        raise RuntimeError(f"kernels use scratch memory: {spilled}")
    if verbose:
        if err.strip():
            print(err, file=sys.stderr)
        for k, v in sorted(usage.items()):
            print(f"{k[:72]:72s} vgpr {v.get('vgpr', 0):3d} agpr {v.get('agpr', 0):3d} waves/SIMD {v.get('occupancy', 0)}", file=sys.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
