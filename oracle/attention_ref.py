"""Plain fp64 reference of exact (causal) multi-head self-attention and its gradients.

TEST INFRASTRUCTURE ONLY -- see the package docstring.

What is computed.  The paper treats attention as the parameter-free middle part of a
standard GPT-3 transformer layer (Section 2.1 "Model Architecture", Figure 1), trained
for next-token prediction (Section 4.6), with dropout omitted and biases neglected
(Table 1 caption).  It never prints the formula; the textbook definition is used, per
(batch, head) slice, with q, k, v, g = dO of shape [S, D]:

    s_ij  = scale * sum_d q_id k_jd          for j <= i (causal); entries j > i are absent
    m_i   = max_j s_ij,  Z_i = sum_j exp(s_ij - m_i),  LSE_i = m_i + ln Z_i   (natural log)
    p_ij  = exp(s_ij - LSE_i)
    o_id  = sum_j p_ij v_jd
    dv_jd = sum_i p_ij g_id
    dp_ij = sum_d g_id v_jd
    delta_i = sum_j p_ij dp_ij               ( = sum_d g_id o_id )
    ds_ij = p_ij (dp_ij - delta_i)
    dq_id = scale * sum_j ds_ij k_jd
    dk_jd = scale * sum_i ds_ij q_id

Attention has no parameters, so the backward pass produces exactly dq, dk, dv
(Table 1: the "Backward W" entry of the Attention column is empty).

Structure: blocks of query rows against FULL score rows and a plain two-pass softmax.
There is no key tiling, no running maximum and no rescaling, so the code can be checked
against the formulas above by eye.  ``numpy.matmul`` serves as the contraction step.

Parity pins (tests marked "not gpu"): softmax rows sum to one, causality under
perturbation of later tokens, closed forms for K = 0 and for row 0, shift invariance in
K, a scalar triple-loop C implementation (``brute_force.c``) on tiny shapes and central
finite differences of L = sum(g * o) for every gradient element.
"""
from __future__ import annotations

import numpy as np


def _as_f64(x):
    return np.ascontiguousarray(x, dtype=np.float64)


def head_forward(q, k, v, scale, causal=True, row_block=512, rows=None):
    """Forward of one head.  q, k, v: [S, D] -> (o [R, D], lse [R]) for the requested rows.

    ``rows`` is an optional (start, stop) range of query rows; default all rows.
    """
    q, k, v = _as_f64(q), _as_f64(k), _as_f64(v)
    S = q.shape[0]
    r0, r1 = (0, S) if rows is None else rows
    o = np.empty((r1 - r0, v.shape[1]), dtype=np.float64)
    lse = np.empty(r1 - r0, dtype=np.float64)
    for a in range(r0, r1, row_block):
        b = min(a + row_block, r1)
        nk = b if causal else S                       # keys any row of the block can see
        s = scale * (q[a:b] @ k[:nk].T)               # [rows, nk]
        if causal:
            i = np.arange(a, b)[:, None]
            j = np.arange(nk)[None, :]
            s = np.where(j <= i, s, -np.inf)
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)                             # exp(-inf) = 0 for masked entries
        z = e.sum(axis=1, keepdims=True)
        l = m + np.log(z)
        p = np.exp(s - l)
        o[a - r0:b - r0] = p @ v[:nk]
        lse[a - r0:b - r0] = l[:, 0]
    return o, lse


def head_backward(q, k, v, g, scale, causal=True, row_block=512):
    """Forward + analytic gradients of one head.  All inputs [S, D].

    Returns dict with o, lse, delta, dq, dk, dv (fp64).
    """
    q, k, v, g = _as_f64(q), _as_f64(k), _as_f64(v), _as_f64(g)
    S, D = q.shape
    o, lse = head_forward(q, k, v, scale, causal, row_block)
    dq = np.zeros((S, D)); dk = np.zeros((S, k.shape[1])); dv = np.zeros((S, v.shape[1]))
    delta = np.empty(S)
    for a in range(0, S, row_block):
        b = min(a + row_block, S)
        nk = b if causal else S
        s = scale * (q[a:b] @ k[:nk].T)
        p = np.exp(s - lse[a:b, None])
        if causal:
            i = np.arange(a, b)[:, None]
            j = np.arange(nk)[None, :]
            p = np.where(j <= i, p, 0.0)
        dp = g[a:b] @ v[:nk].T
        dl = (p * dp).sum(axis=1)                     # delta by its definition
        ds = p * (dp - dl[:, None])
        delta[a:b] = dl
        dv[:nk] += p.T @ g[a:b]
        dq[a:b] = scale * (ds @ k[:nk])
        dk[:nk] += scale * (ds.T @ q[a:b])
    # identity used by the GPU preprocess: delta_i = sum_d g_id o_id
    alt = (g * o).sum(axis=1)
    tol = 1e-9 * (1.0 + np.abs(alt).max())
    if not np.all(np.abs(alt - delta) <= tol):
        raise AssertionError("delta computed two ways disagrees")
    return {"o": o, "lse": lse, "delta": delta, "dq": dq, "dk": dk, "dv": dv}


def attn_fwd_ref(q, k, v, scale, causal=True):
    """q, k, v: [B, H, S, D] -> (o [B, H, S, D], lse [B, H, S]) in fp64."""
    B, H, S, D = q.shape
    o = np.empty((B, H, S, v.shape[-1])); lse = np.empty((B, H, S))
    for b in range(B):
        for h in range(H):
            o[b, h], lse[b, h] = head_forward(q[b, h], k[b, h], v[b, h], scale, causal)
    return o, lse


def attn_bwd_ref(q, k, v, g, scale, causal=True):
    """q, k, v, g: [B, H, S, D] -> dict of o, lse, delta, dq, dk, dv in fp64."""
    B, H, S, D = q.shape
    out = {n: np.empty((B, H, S, D)) for n in ("o", "dq", "dk", "dv")}
    out["lse"] = np.empty((B, H, S)); out["delta"] = np.empty((B, H, S))
    for b in range(B):
        for h in range(H):
            r = head_backward(q[b, h], k[b, h], v[b, h], g[b, h], scale, causal)
            for n, val in r.items():
                out[n][b, h] = val
    return out


def head_rows(q, k, v, g, rows, scale, causal=True):
    """o, lse, dq of selected query rows of one head; needs only keys 0..i of each row i.

    q, k, v, g: [S, D]; rows: iterable of row indices.  Returns (o [n, D], lse [n], dq [n, D]).
    """
    q, k, v, g = _as_f64(q), _as_f64(k), _as_f64(v), _as_f64(g)
    S = q.shape[0]
    rows = list(rows)
    o = np.empty((len(rows), v.shape[1])); lse = np.empty(len(rows)); dq = np.empty((len(rows), q.shape[1]))
    for n, i in enumerate(rows):
        nk = i + 1 if causal else S
        s = scale * (k[:nk] @ q[i])
        m = s.max()
        l = m + np.log(np.exp(s - m).sum())
        p = np.exp(s - l)
        oi = p @ v[:nk]
        dp = v[:nk] @ g[i]
        dl = p @ dp
        ds = p * (dp - dl)
        o[n], lse[n], dq[n] = oi, l, scale * (ds @ k[:nk])
    return o, lse, dq


def head_stats(q, k, v, g, scale, causal=True, row_start=0, row_block=512):
    """lse_i and delta_i for rows i >= row_start of one head (what key-column gradients need)."""
    o, lse = head_forward(q, k, v, scale, causal, row_block, rows=(row_start, q.shape[0]))
    p_dp = (_as_f64(g)[row_start:] * o).sum(axis=1)
    return lse, p_dp


def head_cols(q, k, v, g, cols, lse, delta, scale, causal=True, row_start=0, row_block=4096):
    """dk, dv of selected key columns of one head.

    ``lse`` and ``delta`` cover rows row_start..S-1 (from ``head_stats``); every requested
    column must satisfy j >= row_start when causal (rows before j do not see key j) or
    row_start must be 0.  Returns (dk [n, D], dv [n, D]).
    """
    q, k, v, g = _as_f64(q), _as_f64(k), _as_f64(v), _as_f64(g)
    S = q.shape[0]
    cols = np.asarray(list(cols), dtype=np.int64)
    if row_start > 0 and not (causal and cols.min() >= row_start):
        raise ValueError("columns need rows before row_start")
    kj, vj = k[cols], v[cols]
    dk = np.zeros((len(cols), q.shape[1])); dv = np.zeros((len(cols), g.shape[1]))
    first = int(cols.min()) if causal else 0
    for a in range(max(first, row_start), S, row_block):
        b = min(a + row_block, S)
        s = scale * (q[a:b] @ kj.T)                                   # [rows, n]
        p = np.exp(s - lse[a - row_start:b - row_start, None])
        if causal:
            p = np.where(cols[None, :] <= np.arange(a, b)[:, None], p, 0.0)
        dp = g[a:b] @ vj.T
        ds = p * (dp - delta[a - row_start:b - row_start, None])
        dv += p.T @ g[a:b]
        dk += scale * (ds.T @ q[a:b])
    return dk, dv


def attn_flops(B, H, S, D, causal=True):
    """Matrix FLOPs of the path, following Table 1's convention (matrix products only).

    Table 1 gives 4*b*h*s^2 forward and 8*b*h*s^2 backward for a full (non-causal) score
    matrix with hidden size h = H*D; per unmasked (query, key) pair per head that is 4*D
    forward and 8*D backward.  ``bwd_recompute`` adds the score recomputation a backward
    pass that stores no S x S matrix must do (10*D per pair).
    """
    pairs = S * (S + 1) // 2 if causal else S * S
    unit = B * H * pairs * D
    return {"fwd": 4 * unit, "bwd_table1": 8 * unit, "bwd_recompute": 10 * unit,
            "fwd_bwd": 14 * unit, "fwd_bwd_table1": 12 * unit}
