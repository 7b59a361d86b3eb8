"""Plain fp64 reference of the QKV linear layer and its two backward products.

TEST INFRASTRUCTURE ONLY -- see the package docstring.

What is computed.  HelixPipe runs the QKV linear layer on the attention stage (Section 4.2:
the layer's input A and its weights travel instead of Q, K, V).  Table 1 lists it with 6bsh^2
FLOPs forward and the same for each of "Backward B" (gradient of the input) and "Backward W"
(gradient of the weights), biases neglected:

    qkv_mn = sum_k a_mk w_kn
    da_mk  = sum_n dqkv_mn w_kn
    dw_kn  = sum_m a_mk dqkv_mn

``numpy.matmul`` in fp64 is the contraction step; nothing is blocked or reordered.

Parity pins (tests marked "not gpu"): scalar triple loops on tiny shapes, the identity
weight matrix, linearity, and central finite differences of L = sum(g * qkv) for every
element of da and dw.
"""
from __future__ import annotations

import numpy as np


def linear_fwd_ref(a, w):
    return np.matmul(np.asarray(a, dtype=np.float64), np.asarray(w, dtype=np.float64))


def linear_bwd_ref(a, w, dqkv):
    a, w, g = (np.asarray(x, dtype=np.float64) for x in (a, w, dqkv))
    return {"da": np.matmul(g, w.T), "dw": np.matmul(a.T, g)}


def linear_flops(M: int, K: int, N: int) -> int:
    """2MKN per product: Table 1's 6bsh^2 with M = b*s, K = h, N = 3h."""
    return 2 * M * K * N
