"""HIP streams restricted to a subset of the compute units (plumbing for the overlap measurements).

The two-fold FILO schedule (Section 4.3) hides the stage-to-stage transfer of one micro batch
behind the attention of another, and Section 5.3 argues that the communication kernels occupy
only a few compute units.  A stream created with ``hipExtStreamCreateWithCUMask`` lets one GPU
show the attention side of that: the path runs while N compute units are withheld from it.
"""
from __future__ import annotations

import ctypes

import torch


def cu_masked_stream(n_cu: int, masked: int) -> torch.cuda.ExternalStream:
    """A torch stream (default priority) on which kernels may use all but ``masked`` compute units.
    The withheld units are mask bits 33*i mod n_cu, which spreads them over the XCDs whether
    consecutive bits go round the XCDs or fill one XCD after the other."""
    if not 0 <= masked < n_cu:
        raise ValueError("masked must lie in [0, n_cu)")
    hip = ctypes.CDLL("libamdhip64.so")
    words = (n_cu + 31) // 32
    bits = [1] * n_cu
    for i in range(masked):
        bits[(33 * i) % n_cu] = 0
    mask = (ctypes.c_uint32 * words)(*[sum(bits[32 * w + b] << b for b in range(32) if 32 * w + b < n_cu) for w in range(words)])
    stream = ctypes.c_void_p()
    err = hip.hipExtStreamCreateWithCUMask(ctypes.byref(stream), ctypes.c_uint32(words), mask)
    if err != 0:
        raise RuntimeError(f"hipExtStreamCreateWithCUMask failed with {err}")
    return torch.cuda.ExternalStream(stream.value)
