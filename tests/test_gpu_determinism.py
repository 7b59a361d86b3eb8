"""Run-to-run bit equality under repetition.  No kernel uses atomics, so every output is a
pure function of the inputs; a tile that is read before its asynchronous copy has landed
shows up here as a run that differs from the others (it did once: the forward read the
first V operands of the next tile one iteration before that tile was guaranteed)."""
import numpy as np
import pytest
import torch

from paper_2507_00394_amd import inputs as I

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("BH,S,D,causal", [(3, 1500, 128, True), (8, 1500, 128, True), (5, 2100, 64, True),
                                           (4, 1100, 128, False)])
def test_repeated_runs_are_bit_identical(BH, S, D, causal):
    from tests import gpu_util as G

    cfg, bits = I.random_case_bits(6100 + BH + S, 1, BH, S, D)
    first = None
    for rep in range(30):
        out = G.run_fwd_bwd(bits, cfg.scale, causal)
        cur = {n: (out[n].view(torch.int16) if out[n].dtype == torch.bfloat16 else out[n]).clone()
               for n in ("o", "lse", "dq", "dk", "dv")}
        if first is None:
            first = cur
            continue
        for n in cur:
            assert torch.equal(cur[n], first[n]), f"{n} differs from the first run in repetition {rep}"


def test_repeated_runs_at_the_7b_32k_size():
    """Three runs of config 3 (B=1, H=32, S=32768, D=128): every wave goes round the four-stage tile
    pipelines some hundreds of times, the length at which a mis-counted copy wait would show."""
    from tests import gpu_util as G

    cfg = I.CONFIGS[3]
    bits = I.all_inputs_bits(cfg, threads=16)
    first = None
    for rep in range(3):
        out = G.run_fwd_bwd(bits, cfg.scale, True)
        cur = {n: (out[n].view(torch.int16) if out[n].dtype == torch.bfloat16 else out[n]).clone()
               for n in ("o", "lse", "dq", "dk", "dv")}
        del out
        if first is None:
            first = cur
            continue
        for n in cur:
            assert torch.equal(cur[n], first[n]), f"{n} differs from the first run in repetition {rep}"
