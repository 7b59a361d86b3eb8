"""The path next to a concurrent disturbance (Section 4.3: transfers hidden behind attention; Section 5.3:
communication kernels take few compute units).  At the 7B / 32k size the forward and the backward run
(a) on a stream from which 16 of the compute units are withheld and (b) while a second stream of default
priority copies device memory back and forth: both must reproduce the undisturbed result bit for bit,
which is itself checked against the oracle on sampled query rows."""
import numpy as np
import pytest
import torch

from paper_2507_00394_amd import binding as hx
from paper_2507_00394_amd import inputs as I
from paper_2507_00394_amd.streams import cu_masked_stream

pytestmark = pytest.mark.gpu


def _run(t, cfg, stream=None):
    q, k, v, g = t["q"], t["k"], t["v"], t["dO"]
    B, H, S, D = q.shape
    with torch.cuda.stream(stream if stream is not None else torch.cuda.current_stream()):
        o = torch.empty_like(q); lse = torch.empty((B, H, S), dtype=torch.float32, device="cuda")
        dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
        ws = torch.empty(hx.helix_attn_bwd_workspace_bytes(B, H, S, D), dtype=torch.uint8, device="cuda")
        torch.cuda.current_stream().synchronize()
        hx.helix_attn_fwd(q, k, v, o, lse, cfg.scale, True)
        hx.helix_attn_bwd(q, k, v, o, lse, g, dq, dk, dv, ws, cfg.scale, True)
        torch.cuda.current_stream().synchronize()
    return {"o": o, "lse": lse, "dq": dq, "dk": dk, "dv": dv}


def test_masked_compute_units_and_concurrent_copy_leave_results_unchanged():
    from tests import gpu_util as G
    from tests.test_gpu_parity_sampled import _rows_check

    cfg = I.CONFIGS[3]
    bits = I.all_inputs_bits(cfg, threads=16)
    t = {n: G.to_dev(bits[n]) for n in bits}
    torch.cuda.synchronize()
    base = _run(t, cfg)
    errs = _rows_check(cfg, bits, base, G)
    assert errs["lse"].max() <= G.TOL_LSE
    for n in ("o", "dq"):
        assert errs[n].max() <= G.TOL_MAX and errs[n].mean() <= G.TOL_MEAN, n

    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    masked = _run(t, cfg, cu_masked_stream(n_cu, 16))
    for n in base:
        assert torch.equal(masked[n], base[n]), f"{n} differs with 16 compute units withheld"

    side = torch.cuda.Stream()                      # default priority
    src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda"); dst = torch.empty_like(src)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        for _ in range(48):                         # about 25 GB each way: outlasts the 35 ms of the path several times over
            dst.copy_(src, non_blocking=True)
    beside = _run(t, cfg)
    side.synchronize()
    for n in base:
        assert torch.equal(beside[n], base[n]), f"{n} differs beside a concurrent copy"
