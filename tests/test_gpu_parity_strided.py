"""Strided entry points and small head counts: views into sequence-major buffers, as the
paper's layers produce them (activations [s, b, h], Section 2.1; fused QKV output, Section
4.2), must give bit-for-bit what the contiguous entry points give on the same values, and
that result must match the oracle.  Head counts that are not multiples of 8 exercise the
spreading of one head over several XCDs (one GPU's share of the heads, Section 2.2)."""
import numpy as np
import pytest
import torch

from oracle import attention_ref as A
from paper_2507_00394_amd import inputs as I

pytestmark = pytest.mark.gpu


def _contiguous_reference(bits, scale, causal):
    from tests import gpu_util as G

    out = G.run_fwd_bwd(bits, scale, causal)
    f = {t: I.bf16_bits_to_float(bits[t]) for t in bits}
    ref = A.attn_bwd_ref(f["q"], f["k"], f["v"], f["dO"], scale, causal)
    for n in ("o", "dq", "dk", "dv"):
        G.check(n, G.to_f64(out[n]), ref[n])
    assert np.abs(G.to_f64(out["lse"]) - ref["lse"]).max() <= G.TOL_LSE
    return out


def _run_strided(views, lse_shape, scale, causal):
    from paper_2507_00394_amd import binding as hx

    B, H, S, D = views["q"].shape
    lse = torch.empty(lse_shape, dtype=torch.float32, device="cuda")
    hx.helix_attn_fwd_strided(views["q"], views["k"], views["v"], views["o"], lse, scale, causal)
    ws = torch.empty(hx.helix_attn_bwd_workspace_bytes(B, H, S, D), dtype=torch.uint8, device="cuda")
    hx.helix_attn_bwd_strided(views["q"], views["k"], views["v"], views["o"], lse, views["dO"], views["dq"],
                              views["dk"], views["dv"], ws, scale, causal)
    torch.cuda.synchronize()
    return lse


@pytest.mark.parametrize("B,H,S,D,layout", [
    (2, 3, 333, 128, "fused"), (1, 4, 520, 64, "fused"), (2, 2, 257, 128, "interleaved"), (1, 5, 130, 64, "padded")])
def test_strided_views_match_contiguous_bitwise(B, H, S, D, layout):
    from tests import gpu_util as G

    cfg, bits = I.random_case_bits(9000 + S + H, B, H, S, D)
    out = _contiguous_reference(bits, cfg.scale, True)
    dev = {t: G.to_dev(bits[t]) for t in ("q", "k", "v", "dO")}           # [B,H,S,D]
    fill = lambda *shape: torch.full(shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    if layout == "fused":            # QKV linear output [S, B, 3, H, D]; activations [S, B, H, D]
        qkv, dqkv = fill(S, B, 3, H, D), fill(S, B, 3, H, D)
        view = lambda buf, i: buf[:, :, i].permute(1, 2, 0, 3)
        act = lambda: fill(S, B, H, D)
        as_view = lambda a: a.permute(1, 2, 0, 3)
    elif layout == "interleaved":    # per-head interleaving [S, B, H, 3, D]
        qkv, dqkv = fill(S, B, H, 3, D), fill(S, B, H, 3, D)
        view = lambda buf, i: buf[:, :, :, i].permute(1, 2, 0, 3)
        act = lambda: fill(S, B, H, D)
        as_view = lambda a: a.permute(1, 2, 0, 3)
    else:                            # head-major with padded rows [B, H, S, D + 8]
        qkv, dqkv = fill(3, B, H, S, D + 8), fill(3, B, H, S, D + 8)
        view = lambda buf, i: buf[i, :, :, :, :D]
        act = lambda: fill(B, H, S, D + 8)
        as_view = lambda a: a[..., :D]
    views = {}
    for i, t in enumerate(("q", "k", "v")):
        views[t] = view(qkv, i); views[t].copy_(dev[t])
        views["d" + t] = view(dqkv, i)
    o_buf, g_buf = act(), act()
    views["o"], views["dO"] = as_view(o_buf), as_view(g_buf)
    views["dO"].copy_(dev["dO"])
    assert not views["q"].is_contiguous()
    lse = _run_strided(views, (B, H, S), cfg.scale, True)
    assert torch.equal(lse, out["lse"])
    for n in ("o", "dq", "dk", "dv"):
        assert torch.equal(views[n].contiguous().view(torch.int16), out[n].view(torch.int16)), n
    if layout == "padded":           # the padding columns were never written
        assert torch.isnan(o_buf[..., D:]).all() and torch.isnan(dqkv[..., D:]).all()


@pytest.mark.parametrize("BH", [1, 2, 3, 4, 5, 6, 7, 12])
def test_head_counts_not_multiple_of_eight(BH):
    """Each head is split into parts that go to different XCDs; tiles 0..T-1 must each be
    done exactly once (any tile done twice or skipped shows as a parity failure, since the
    outputs start as NaN)."""
    S = 1500          # 6 forward tiles, 12 dK/dV tiles: not a multiple of 4 or 8 parts
    cfg, bits = I.random_case_bits(4200 + BH, 1, BH, S, 128)
    _contiguous_reference(bits, cfg.scale, True)


def test_full_attention_strided():
    from tests import gpu_util as G

    B, H, S, D = 1, 2, 200, 128
    cfg, bits = I.random_case_bits(4300, B, H, S, D)
    out = _contiguous_reference(bits, cfg.scale, False)
    buf = torch.zeros(S, B, H, 8, D, dtype=torch.bfloat16, device="cuda")
    names = ("q", "k", "v", "dO", "o", "dq", "dk", "dv")
    views = {n: buf[:, :, :, i].permute(1, 2, 0, 3) for i, n in enumerate(names)}
    for t in ("q", "k", "v", "dO"):
        views[t].copy_(G.to_dev(bits[t]))
    lse = _run_strided(views, (B, H, S), cfg.scale, False)
    assert torch.equal(lse, out["lse"])
    for n in ("o", "dq", "dk", "dv"):
        assert torch.equal(views[n].contiguous().view(torch.int16), out[n].view(torch.int16)), n


def test_row_stride_of_sixteen_mebibytes():
    """Rows 2^23 elements apart (the tile copies then use lane offsets of up to 1e9 bytes and 64-bit
    tile bases): same bits as the contiguous call."""
    from tests import gpu_util as G

    B, H, S, D = 1, 2, 100, 128
    row = 1 << 23
    cfg, bits = I.random_case_bits(4400, B, H, S, D)
    out = _contiguous_reference(bits, cfg.scale, True)
    buf = torch.empty((S - 1) * row + 8 * H * D, dtype=torch.bfloat16, device="cuda")     # 1.6 GiB, mostly untouched
    names = ("q", "k", "v", "dO", "o", "dq", "dk", "dv")
    views = {n: torch.as_strided(buf, (B, H, S, D), (0, D, row, 1), storage_offset=i * H * D) for i, n in enumerate(names)}
    for t in ("q", "k", "v", "dO"):
        views[t].copy_(G.to_dev(bits[t]))
    lse = _run_strided(views, (B, H, S), cfg.scale, True)
    assert torch.equal(lse, out["lse"])
    for n in ("o", "dq", "dk", "dv"):
        assert torch.equal(views[n].contiguous().view(torch.int16), out[n].view(torch.int16)), n
