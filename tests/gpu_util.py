"""Helpers of the GPU parity tests: upload bf16 bit patterns, run the HIP path through
the C-ABI binding, download results as float64."""
import numpy as np
import torch

from paper_2507_00394_amd import binding as hx
from paper_2507_00394_amd import inputs as I

TOL_MAX, TOL_MEAN, TOL_LSE = 2e-2, 2e-3, 1e-3   # max abs / mean abs for O, dQ, dK, dV; |dLSE|


def to_dev(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def to_f64(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return I.bf16_bits_to_float(t.view(torch.int16).cpu().numpy().view(np.uint16))
    return t.double().cpu().numpy()


def run_fwd_bwd(bits, scale, causal=True, fused_bwd=True):
    """bits: dict q,k,v,dO of uint16 [B,H,S,D].  Returns dict of device tensors."""
    q, k, v, g = (to_dev(bits[t]) for t in ("q", "k", "v", "dO"))
    B, H, S, D = q.shape
    nan = float("nan")   # outputs start as NaN so that anything the kernels leave unwritten fails the checks
    o = torch.full_like(q, nan); lse = torch.full((B, H, S), nan, dtype=torch.float32, device="cuda")
    hx.helix_attn_fwd(q, k, v, o, lse, scale, causal)
    dq, dk, dv = torch.full_like(q, nan), torch.full_like(q, nan), torch.full_like(q, nan)
    if fused_bwd:
        ws = torch.empty(hx.helix_attn_bwd_workspace_bytes(B, H, S, D), dtype=torch.uint8, device="cuda")
        hx.helix_attn_bwd(q, k, v, o, lse, g, dq, dk, dv, ws, scale, causal)
    else:
        stats = torch.empty(hx.helix_attn_bwd_workspace_bytes(B, H, S, D), dtype=torch.uint8, device="cuda")
        hx.helix_attn_bwd_preprocess(o, g, lse, stats)
        if causal:
            hx.helix_attn_bwd_delta_head(q, k, v, g, lse, stats, hx.DELTA_HEAD_ROWS, scale, causal)
        hx.helix_attn_bwd_dkdv(q, k, v, g, stats, dk, dv, scale, causal)
        hx.helix_attn_bwd_dq(q, k, v, g, stats, dq, scale, causal)
    torch.cuda.synchronize()
    return {"q": q, "k": k, "v": v, "dO": g, "o": o, "lse": lse, "dq": dq, "dk": dk, "dv": dv}


def check(name, got, ref, tol_max=TOL_MAX, tol_mean=TOL_MEAN):
    err = np.abs(got - ref)
    assert np.isfinite(got).all(), f"{name}: non-finite output"
    mx, mean = float(err.max()), float(err.mean())
    assert mx <= tol_max and mean <= tol_mean, f"{name}: max abs {mx:.4g} (tol {tol_max}), mean abs {mean:.4g} (tol {tol_mean}), max|ref| {np.abs(ref).max():.3g}"
    return mx, mean
