"""The pure MFMA loop the benchmark times beside the attention kernels: it reports the number of
FLOPs it performs (8 waves per workgroup, 16 MFMAs of 32 x 32 x 16 per iteration and wave), leaves
its sink untouched, runs on the caller's stream, and its rate with constant operands is at least
that with random ones (the chip is power limited on toggling data) and below the nominal peak."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_flop_count_rate_and_sink():
    from paper_2507_00394_amd import binding as hx

    cus, khz = hx.helix_attn_device_info()
    sink = torch.full((1,), 7.0, dtype=torch.float32, device="cuda")
    wgs, iters = 2 * cus, 20000
    rate = {}
    for rnd in (False, True):
        hx.helix_mfma_probe(sink, wgs, 500, rnd)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flops = hx.helix_mfma_probe(sink, wgs, iters, rnd)
        e1.record()
        torch.cuda.synchronize()
        assert flops == wgs * 8 * iters * 16 * 2 * 32 * 32 * 16
        rate[rnd] = flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
    peak = cus * 4096 * khz * 1e3 / 1e12
    print(f"sustained MFMA rate: constant {rate[False]:.0f}, random {rate[True]:.0f} TFLOP/s; nominal peak {peak:.0f}", flush=True)
    assert float(sink.item()) == 7.0
    assert 0.4 * peak < rate[True] <= rate[False] * 1.02 and rate[False] < 1.01 * peak

    # the loop with one LDS operand read and vector work per MFMA: same FLOP count, lower rate, the
    # forward's mix (more vector work) below the backward's
    mix = {}
    for fwd_mix in (False, True):
        hx.helix_mfma_mix_probe(sink, cus, 500, fwd_mix)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flops = hx.helix_mfma_mix_probe(sink, cus, iters, fwd_mix)
        e1.record()
        torch.cuda.synchronize()
        assert flops == cus * 8 * iters * 16 * 2 * 32 * 32 * 16
        mix[fwd_mix] = flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
    print(f"with the kernels' instruction mix: backward-like {mix[False]:.0f}, forward-like {mix[True]:.0f} TFLOP/s", flush=True)
    assert float(sink.item()) == 7.0
    assert 0.3 * peak < mix[True] < mix[False] * 1.02 and mix[False] < rate[True] * 1.02

    s2 = torch.cuda.Stream()
    with torch.cuda.stream(s2):
        hx.helix_mfma_probe(sink, 8, 100, True, stream=s2)
    s2.synchronize()
    assert float(sink.item()) == 7.0
