"""helix_attn_bwd_static (statistics in the library's built-in device array, no workspace argument)
against helix_attn_bwd, through the C ABI: two calls in a row, the second on a smaller input, so
that whatever the first call left in the shared array must not matter.  Same kernels, same
arithmetic: the results have to agree bit for bit; the first is also checked against the oracle."""
import numpy as np
import pytest
import torch

from oracle import attention_ref as A
from paper_2507_00394_amd import binding as hx
from paper_2507_00394_amd import inputs as I

pytestmark = pytest.mark.gpu


def _run(seed, B, H, S, D, causal):
    from tests import gpu_util as G

    cfg, bits = I.random_case_bits(seed, B, H, S, D)
    q, k, v, g = (G.to_dev(bits[t]) for t in ("q", "k", "v", "dO"))
    o = torch.empty_like(q); lse = torch.empty((B, H, S), dtype=torch.float32, device="cuda")
    hx.helix_attn_fwd(q, k, v, o, lse, cfg.scale, causal)
    nan = float("nan")
    ref = [torch.full_like(q, nan) for _ in range(3)]
    ws = torch.empty(hx.helix_attn_bwd_workspace_bytes(B, H, S, D), dtype=torch.uint8, device="cuda")
    hx.helix_attn_bwd(q, k, v, o, lse, g, *ref, ws, cfg.scale, causal)
    got = [torch.full_like(q, nan) for _ in range(3)]
    hx.helix_attn_bwd_static(q, k, v, o, lse, g, *got, cfg.scale, causal)
    torch.cuda.synchronize()
    for name, a, b in zip(("dq", "dk", "dv"), got, ref):
        assert torch.equal(a, b), f"{name}: helix_attn_bwd_static differs from helix_attn_bwd at B={B} H={H} S={S} D={D}"
    return cfg, bits, got


def test_static_scratch_backward_twice_second_smaller():
    from tests import gpu_util as G

    cfg, bits, got = _run(611, 2, 3, 1500, 128, True)
    f = {t: I.bf16_bits_to_float(bits[t]) for t in bits}
    ref = A.attn_bwd_ref(f["q"], f["k"], f["v"], f["dO"], cfg.scale, True)
    for name, t in zip(("dq", "dk", "dv"), got):
        G.check(name, G.to_f64(t), ref[name])
    _run(612, 1, 2, 333, 64, True)       # smaller, other head dimension, right after
    _run(613, 1, 1, 200, 128, False)     # and the non-causal path (no refinement of the first rows)
