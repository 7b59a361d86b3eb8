"""HIP path against the fp64 oracle, element by element, on shapes the oracle finishes in
seconds: config 1 in full, ragged and tiny sequence lengths that cross tile edges,
both head dimensions, causal and full attention, several (batch, head) slices."""
import numpy as np
import pytest
import torch

from oracle import attention_ref as A
from paper_2507_00394_amd import inputs as I

pytestmark = pytest.mark.gpu


def _compare(bits, scale, causal, fused_bwd=True):
    from tests import gpu_util as G

    out = G.run_fwd_bwd(bits, scale, causal, fused_bwd)
    f = {t: I.bf16_bits_to_float(bits[t]) for t in bits}
    ref = A.attn_bwd_ref(f["q"], f["k"], f["v"], f["dO"], scale, causal)
    res = {}
    for n in ("o", "dq", "dk", "dv"):
        res[n] = G.check(n, G.to_f64(out[n]), ref[n])
    dl = np.abs(G.to_f64(out["lse"]) - ref["lse"]).max()
    assert dl <= G.TOL_LSE, f"lse: max abs {dl}"
    return out, ref, res


def test_config1_full():
    cfg = I.CONFIGS[1]
    bits = I.all_inputs_bits(cfg)
    _compare(bits, cfg.scale, True)


@pytest.mark.parametrize("S", [1, 2, 31, 33, 64, 65, 127, 255, 257, 300, 513, 777])
@pytest.mark.parametrize("D", [64, 128])
def test_ragged_lengths_causal(S, D):
    cfg, bits = I.random_case_bits(S * 2 + D, 1, 3, S, D)
    _compare(bits, cfg.scale, True)


@pytest.mark.parametrize("S,D", [(1, 64), (65, 128), (300, 64), (513, 128)])
def test_full_attention(S, D):
    cfg, bits = I.random_case_bits(5000 + S + D, 1, 2, S, D)
    _compare(bits, cfg.scale, False)


def test_many_heads_and_batches_separate_stage_calls():
    cfg, bits = I.random_case_bits(77, 2, 9, 320, 128)      # 18 slices: more than one per XCD slot
    _compare(bits, cfg.scale, True, fused_bwd=False)


def test_sharper_softmax_k_times_two():
    cfg, bits = I.random_case_bits(78, 1, 2, 1024, 128, k_mult=2.0)
    _compare(bits, cfg.scale, True)


def test_other_scale_values():
    cfg, bits = I.random_case_bits(79, 1, 2, 200, 64)
    _compare(bits, 0.05, True)
    _compare(bits, 0.18, True)


@pytest.mark.parametrize("k_mult", [8.0, 32.0])
def test_very_sharp_softmax_stays_finite_and_relatively_accurate(k_mult):
    """Logit standard deviation 8 and 32 (the benchmark workloads have 1 and 2): rows where one key
    takes all the weight, |dQ| up to ~100.  The absolute tolerances of the workloads no longer apply
    to bf16 outputs of that size; what must hold is finiteness, the LSE tolerance, and an error that
    is a bf16 rounding (2^-8 with a factor 2 of margin) relative to the largest magnitude."""
    from tests import gpu_util as G

    cfg, bits = I.random_case_bits(88, 1, 2, 2048, 128, k_mult=k_mult)
    out = G.run_fwd_bwd(bits, cfg.scale, True)
    f = {t: I.bf16_bits_to_float(bits[t]) for t in bits}
    ref = A.attn_bwd_ref(f["q"], f["k"], f["v"], f["dO"], cfg.scale, True)
    for n in ("o", "dq", "dk", "dv"):
        got = G.to_f64(out[n])
        assert np.isfinite(got).all(), n
        err = np.abs(got - ref[n]).max()
        assert err <= G.TOL_MAX + 2.0 ** -7 * np.abs(ref[n]).max(), (n, err, np.abs(ref[n]).max())
    assert np.abs(G.to_f64(out["lse"]) - ref["lse"]).max() <= G.TOL_LSE
