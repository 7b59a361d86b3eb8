"""HIP path at the full benchmark sizes (configs 2-5) against the oracle on samples.

Query rows (O, LSE, dQ): 256 stratified (batch*head, row) samples per config, evaluated by
the oracle inside the test (a row needs only the keys before it).  Key columns (dK, dV):
the stored float32 expectations of ``tests/golden/sampled_cols_cfg<N>.npz``, written by
``tests/golden/make_sampled_cols.py`` from the oracle alone.  The kernels run in the same
launch configuration as ``bench.py``.
"""
import pathlib

import numpy as np
import pytest
import torch

from oracle import attention_ref as A
from paper_2507_00394_amd import inputs as I

pytestmark = pytest.mark.gpu
GOLDEN = pathlib.Path(__file__).parent / "golden"


def _rows_check(cfg, bits, out, G):
    rows = I.sample_rows(cfg)
    by_head = {}
    for bh, i in rows:
        by_head.setdefault(bh, []).append(i)
    BH = cfg.B * cfg.H
    flat = {t: bits[t].reshape(BH, cfg.S, cfg.D) for t in bits}
    dev = {n: out[n].view(BH, cfg.S, -1) if n != "lse" else out[n].view(BH, cfg.S) for n in ("o", "dq", "lse")}
    errs = {"o": [], "dq": [], "lse": []}
    for bh, idx in sorted(by_head.items()):
        idx = sorted(set(idx))
        hi = max(idx) + 1
        f = {t: I.bf16_bits_to_float(flat[t][bh, :hi]) for t in ("q", "k", "v", "dO")}
        o, lse, dq = A.head_rows(f["q"], f["k"], f["v"], f["dO"], idx, cfg.scale, cfg.causal)
        sel = torch.tensor(idx, device="cuda")
        errs["o"].append(np.abs(G.to_f64(dev["o"][bh][sel]) - o))
        errs["dq"].append(np.abs(G.to_f64(dev["dq"][bh][sel]) - dq))
        errs["lse"].append(np.abs(G.to_f64(dev["lse"][bh][sel]) - lse))
    return {n: np.concatenate([e.ravel() for e in v]) for n, v in errs.items()}


def _cols_check(cfg, out, G):
    gold = np.load(GOLDEN / f"sampled_cols_cfg{cfg.cfg_id}.npz")
    BH = cfg.B * cfg.H
    idx = torch.from_numpy(gold["bh"].astype(np.int64) * cfg.S + gold["j"].astype(np.int64)).cuda()
    errs = {}
    for n in ("dk", "dv"):
        got = G.to_f64(out[n].view(BH * cfg.S, cfg.D)[idx])
        assert np.isfinite(got).all()
        errs[n] = np.abs(got - gold[n].astype(np.float64)).ravel()
    return errs


@pytest.mark.parametrize("cfg_id", [2, 3, 4, 5])
def test_config_sampled(cfg_id):
    from tests import gpu_util as G

    cfg = I.CONFIGS[cfg_id]
    print(f"config {cfg_id}: generating inputs", flush=True)
    bits = I.all_inputs_bits(cfg, threads=16)
    print(f"config {cfg_id}: running HIP path", flush=True)
    out = G.run_fwd_bwd(bits, cfg.scale, cfg.causal)
    for n in ("o", "dq", "dk", "dv", "lse"):
        assert bool(torch.isfinite(out[n].float()).all()), n
    print(f"config {cfg_id}: oracle on sampled rows", flush=True)
    errs = _rows_check(cfg, bits, out, G)
    errs.update(_cols_check(cfg, out, G))
    report = {n: (float(e.max()), float(e.mean())) for n, e in errs.items()}
    print(f"config {cfg_id} sampled errors (max, mean): {report}", flush=True)
    assert report["lse"][0] <= G.TOL_LSE, report
    for n in ("o", "dq", "dk", "dv"):
        assert report[n][0] <= G.TOL_MAX and report[n][1] <= G.TOL_MEAN, (n, report)


def test_two_micro_batches_equal_two_calls_and_runs_repeat():
    """B = 2 in one call is bit-identical to two B = 1 calls (the two micro batches a stage
    holds are independent), and repeating a call reproduces every bit (no atomics)."""
    from tests import gpu_util as G

    cfg, bits = I.random_case_bits(501, 2, 5, 2304, 128, k_mult=2.0)
    both = G.run_fwd_bwd(bits, cfg.scale, True)
    again = G.run_fwd_bwd(bits, cfg.scale, True)
    for n in ("o", "lse", "dq", "dk", "dv"):
        assert torch.equal(both[n], again[n]), n
    for b in range(2):
        one = G.run_fwd_bwd({t: np.ascontiguousarray(bits[t][b:b + 1]) for t in bits}, cfg.scale, True)
        for n in ("o", "lse", "dq", "dk", "dv"):
            assert torch.equal(one[n][0], both[n][b]), (n, b)


def test_beyond_the_longest_sequence_of_the_paper():
    """S = 2 * 131072 + 45 (ragged, twice the paper's longest sequence), two heads: sampled query
    rows and the key columns of the last 512 positions against the oracle."""
    from tests import gpu_util as G

    S, H, D = 2 * 131072 + 45, 2, 128
    cfg, bits = I.random_case_bits(777, 1, H, S, D)
    out = G.run_fwd_bwd(bits, cfg.scale, True)
    flat = {t: bits[t].reshape(H, S, D) for t in bits}
    rows = sorted({0, 1, 63, 64, 255, 256, 4095, 131071, 131072, 200000, S - 257, S - 46, S - 45, S - 2, S - 1})
    worst = {}
    for bh in range(H):
        f = {t: I.bf16_bits_to_float(flat[t][bh]) for t in ("q", "k", "v", "dO")}
        o, lse, dq = A.head_rows(f["q"], f["k"], f["v"], f["dO"], rows, cfg.scale, True)
        sel = torch.tensor(rows, device="cuda")
        G.check("o", G.to_f64(out["o"][0, bh][sel]), o)
        G.check("dq", G.to_f64(out["dq"][0, bh][sel]), dq)
        assert np.abs(G.to_f64(out["lse"][0, bh][sel]) - lse).max() <= G.TOL_LSE
        start = S - 512
        lse_t, delta_t = A.head_stats(f["q"], f["k"], f["v"], f["dO"], cfg.scale, True, row_start=start)
        cols = sorted({start, start + 1, start + 100, S - 129, S - 128, S - 46, S - 45, S - 33, S - 2, S - 1})
        dk, dv = A.head_cols(f["q"], f["k"], f["v"], f["dO"], cols, lse_t, delta_t, cfg.scale, True, row_start=start)
        csel = torch.tensor(cols, device="cuda")
        worst[bh] = (G.check("dk", G.to_f64(out["dk"][0, bh][csel]), dk), G.check("dv", G.to_f64(out["dv"][0, bh][csel]), dv))
    print("beyond-paper case, (max, mean) errors of dk, dv per head:", worst, flush=True)
