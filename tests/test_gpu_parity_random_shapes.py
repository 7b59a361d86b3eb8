"""Seeded sweep over random valid shapes: batch, heads, sequence length (any value, not only
multiples of a tile), head dimension, causal or full attention, contiguous or sequence-major
strided tensors - each against the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import attention_ref as A
from paper_2507_00394_amd import inputs as I

pytestmark = pytest.mark.gpu


def _cases(n=36, seed=20250700394 % (2 ** 32)):
    r = np.random.default_rng(seed)
    out = []
    for i in range(n):
        S = int(r.choice([r.integers(1, 64), r.integers(64, 400), r.integers(400, 1600)]))
        out.append((i, int(r.integers(1, 4)), int(r.integers(1, 10)), S, int(r.choice([64, 128])), bool(r.integers(0, 2)),
                    bool(r.integers(0, 2))))
    return out


@pytest.mark.parametrize("idx,B,H,S,D,causal,strided", _cases())
def test_random_shape(idx, B, H, S, D, causal, strided):
    from paper_2507_00394_amd import binding as hx
    from tests import gpu_util as G

    cfg, bits = I.random_case_bits(3000 + idx, B, H, S, D)
    f = {t: I.bf16_bits_to_float(bits[t]) for t in bits}
    ref = A.attn_bwd_ref(f["q"], f["k"], f["v"], f["dO"], cfg.scale, causal)
    if not strided:
        out = G.run_fwd_bwd(bits, cfg.scale, causal)
        got = {n: G.to_f64(out[n]) for n in ("o", "dq", "dk", "dv", "lse")}
    else:
        buf = torch.full((S, B, H, 8, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        names = ("q", "k", "v", "dO", "o", "dq", "dk", "dv")
        v = {n: buf[:, :, :, i].permute(1, 2, 0, 3) for i, n in enumerate(names)}
        for t in ("q", "k", "v", "dO"):
            v[t].copy_(G.to_dev(bits[t]))
        lse = torch.full((B, H, S), float("nan"), dtype=torch.float32, device="cuda")
        ws = torch.empty(hx.helix_attn_bwd_workspace_bytes(B, H, S, D), dtype=torch.uint8, device="cuda")
        hx.helix_attn_fwd_strided(v["q"], v["k"], v["v"], v["o"], lse, cfg.scale, causal)
        hx.helix_attn_bwd_strided(v["q"], v["k"], v["v"], v["o"], lse, v["dO"], v["dq"], v["dk"], v["dv"], ws, cfg.scale, causal)
        torch.cuda.synchronize()
        got = {n: G.to_f64(v[n].contiguous()) for n in ("o", "dq", "dk", "dv")}
        got["lse"] = G.to_f64(lse)
    for n in ("o", "dq", "dk", "dv"):
        G.check(n, got[n], ref[n])
    assert np.abs(got["lse"] - ref["lse"]).max() <= G.TOL_LSE
