"""Seeded synthetic inputs for causal multi-head attention (forward + backward).

This module holds no attention arithmetic.  It only draws the random tensors that
both the CPU oracle and the HIP path consume, rounds them to bfloat16 (the storage
type of the path) and converts bfloat16 bit patterns back to floating point.

The paper trains on synthetic full-length batches (Section 5.1, experiment setup) and
evaluates on no public data set, so seeded iid normal tensors at the layer shapes of
its model table (Table 3: 16 or 32 heads, hidden 2048 / 4096, head dim 128) are the
workload itself rather than a stand-in.

Recipe: for tensor t in {q:0, k:1, v:2, dO:3} of head (b, h) of config c, draw
``standard_normal((S, D), float32)`` from ``Philox(key=[SEED<<32 | c, t<<32 | b*H+h])``,
multiply k by ``k_mult`` (a power of two, so exact), then round to nearest-even bfloat16.
Every head can be regenerated alone, which the sampled parity checks rely on.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

SEED = 250700394
TENSOR_IDS = {"q": 0, "k": 1, "v": 2, "dO": 3}


@dataclass(frozen=True)
class AttnConfig:
    """One synthetic workload: shape, softmax scale and the multiplier applied to K."""

    cfg_id: int
    name: str
    B: int
    H: int
    S: int
    D: int
    k_mult: float = 1.0
    causal: bool = True

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.D))

    @property
    def pairs_per_head(self) -> int:
        """Unmasked (query, key) pairs of one head."""
        return self.S * (self.S + 1) // 2 if self.causal else self.S * self.S


CONFIGS = {
    1: AttnConfig(1, "tiny B1 H2 S512 D64", 1, 2, 512, 64),
    2: AttnConfig(2, "1.3B layer B1 H16 S16384 D128", 1, 16, 16384, 128),
    3: AttnConfig(3, "7B layer B1 H32 S32768 D128", 1, 32, 32768, 128),
    4: AttnConfig(4, "7B layer B1 H32 S131072 D128", 1, 32, 131072, 128),
    5: AttnConfig(5, "13B-like B2 H40 S65536 D128, K x2", 2, 40, 65536, 128, k_mult=2.0),
}


def float_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (round to nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    u = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_float(bits: np.ndarray, dtype=np.float64) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) exactly to float32 or float64."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(dtype)


def head_tensor_bits(cfg_id: int, tensor: str, bh: int, S: int, D: int, k_mult: float = 1.0) -> np.ndarray:
    """bfloat16 bits, shape [S, D], of one tensor of one (batch, head) slice."""
    t = TENSOR_IDS[tensor]
    key = np.array([(SEED << 32) | (cfg_id & 0xFFFFFFFF), (t << 32) | (bh & 0xFFFFFFFF)], dtype=np.uint64)
    gen = np.random.Generator(np.random.Philox(key=key))
    x = gen.standard_normal((S, D), dtype=np.float32)
    if tensor == "k" and k_mult != 1.0:
        x *= np.float32(k_mult)
    return float_to_bf16_bits(x)


def head_inputs(cfg: AttnConfig, bh: int, dtype=np.float64, tensors=("q", "k", "v", "dO"), S: int | None = None):
    """Dict of [S, D] floating-point tensors (exact bfloat16 values) for one head."""
    S = cfg.S if S is None else S
    return {t: bf16_bits_to_float(head_tensor_bits(cfg.cfg_id, t, bh, S, cfg.D, cfg.k_mult), dtype) for t in tensors}


def all_inputs_bits(cfg: AttnConfig, tensors=("q", "k", "v", "dO"), threads: int = 8):
    """Dict of uint16 [B, H, S, D] arrays holding bfloat16 bits of the whole workload."""
    out = {t: np.empty((cfg.B, cfg.H, cfg.S, cfg.D), dtype=np.uint16) for t in tensors}

    def fill(job):
        t, bh = job
        out[t].reshape(cfg.B * cfg.H, cfg.S, cfg.D)[bh] = head_tensor_bits(cfg.cfg_id, t, bh, cfg.S, cfg.D, cfg.k_mult)

    jobs = [(t, bh) for t in tensors for bh in range(cfg.B * cfg.H)]
    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        list(ex.map(fill, jobs))
    return out


def random_case_bits(seed: int, B: int, H: int, S: int, D: int, k_mult: float = 1.0):
    """Ad-hoc seeded case (odd shapes for edge tests): same recipe, config id 1000+seed."""
    cfg = AttnConfig(1000 + seed, f"adhoc{seed}", B, H, S, D, k_mult)
    return cfg, all_inputs_bits(cfg, threads=1)


def sample_rows(cfg: AttnConfig, n: int = 256, seed: int = 7):
    """Stratified sample of (bh, i) query rows: tile edges forced, rest uniform."""
    S, BH = cfg.S, cfg.B * cfg.H
    forced = [0, 1, 31, 32, 63, 64, 127, 128, 255, 256, S // 2 - 1, S // 2, S - 129, S - 128, S - 2, S - 1]
    forced = sorted({i for i in forced if 0 <= i < S})
    rng = np.random.Generator(np.random.Philox(key=np.array([SEED, (seed << 32) | cfg.cfg_id], dtype=np.uint64)))
    picks = [((7 * n_ + 3) % BH, i) for n_, i in enumerate(forced)]
    while len(picks) < n:
        picks.append((int(rng.integers(BH)), int(rng.integers(S))))
    return picks[:n]


TAIL_WINDOW = 4096   # the tail stratum of the key-column sample lies in the last TAIL_WINDOW positions


def sample_cols(cfg: AttnConfig, n_full: int = 64, n_tail: int = 128, n_mid: int = 16, tail: int = TAIL_WINDOW, seed: int = 11):
    """Key-column sample in three strata, each a dict {bh: [j...]}:

    ``full``  whole key range of the first and the last (batch, head) slice, tile edges forced
              (a column needs the statistics of every later row: a whole forward of the head);
    ``mid``   columns of the second half of the sequence, before the tail window, in the middle
              slice (needs the rows from S/2 on);
    ``tail``  ``n_tail`` draws in the last ``tail`` positions dealt round-robin over ALL other
              slices, so that every head's last tiles are compared (needs the last rows only).
    """
    S, BH = cfg.S, cfg.B * cfg.H
    rng = np.random.Generator(np.random.Philox(key=np.array([SEED, (seed << 32) | cfg.cfg_id], dtype=np.uint64)))
    forced = sorted({j for j in [0, 1, 127, 128, 255, 256, S // 2, S - 128, S - 1] if 0 <= j < S})
    full = {}
    for bh in sorted({0, BH - 1}):
        cols = list(forced)
        while len(cols) < n_full:
            cols.append(int(rng.integers(S)))
        full[bh] = sorted(set(cols))
    lo = max(0, S - tail)
    mid = {}
    if S // 2 < lo and BH > 2:
        cols = {S // 2, S // 2 + 127, (S // 2 + lo) // 2, lo - 1}
        while len(cols) < n_mid:
            cols.add(int(rng.integers(S // 2, lo)))
        mid[BH // 2] = sorted(cols)
    others = [bh for bh in range(BH) if bh not in full] or list(full)
    tail_cols = {bh: set() for bh in others}
    for n in range(max(n_tail, len(others))):
        tail_cols[others[n % len(others)]].add(int(rng.integers(lo, S)))
    return full, mid, {bh: sorted(c) for bh, c in tail_cols.items() if c}


def linear_case_bits(seed: int, M: int, K: int, N: int, w_std: float = 0.02):
    """bf16 bit patterns of a linear-layer case: a [M,K] ~ N(0,1) (a LayerNorm output),
    w [K,N] ~ N(0, w_std^2) (GPT-style initialisation), dqkv [M,N] ~ N(0,1)."""
    out = {}
    for t, (name, shape, mult) in enumerate((("a", (M, K), 1.0), ("w", (K, N), w_std), ("dqkv", (M, N), 1.0))):
        g = np.random.Generator(np.random.Philox(key=[(SEED << 32) | (0xFFFF0000 + (seed & 0xFFFF)), 64 + t]))
        out[name] = float_to_bf16_bits(g.standard_normal(shape, dtype=np.float32) * np.float32(mult))
    return out
