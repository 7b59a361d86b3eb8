"""Pins of the CPU oracle against what mathematics and the paper fix (no GPU).

Each test would fail for a plausible mistake in ``oracle/attention_ref.py``: a dropped
term, a wrong sign, a transposed operand, an off-by-one mask or a misplaced scale.
"""
import pathlib

import numpy as np
import pytest

from oracle import attention_ref as A

GOLDEN = pathlib.Path(__file__).parent / "golden"


def rnd(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def test_softmax_rows_sum_to_one_and_mask():
    S, D, scale = 40, 8, 0.37
    q, k, v = rnd(1, S, D), rnd(2, S, D), rnd(3, S, D)
    _, lse = A.head_forward(q, k, v, scale, causal=True, row_block=7)
    s = scale * q @ k.T
    p = np.exp(s - lse[:, None])
    p_causal = np.tril(p)
    assert np.abs(p_causal.sum(axis=1) - 1.0).max() <= 1e-12
    assert (p_causal >= 0).all()
    _, lse_nc = A.head_forward(q, k, v, scale, causal=False)
    assert np.abs(np.exp(s - lse_nc[:, None]).sum(axis=1) - 1.0).max() <= 1e-12


def test_causality_bit_for_bit():
    S, D, scale = 33, 16, 0.25
    q, k, v, g = rnd(4, S, D), rnd(5, S, D), rnd(6, S, D), rnd(7, S, D)
    o, lse = A.head_forward(q, k, v, scale, row_block=S)
    for t in (1, 10, 32):
        q2, k2, v2 = q.copy(), k.copy(), v.copy()
        q2[t:] += 3.0; k2[t:] -= 5.0; v2[t:] *= -2.0
        o2, lse2 = A.head_forward(q2, k2, v2, scale, row_block=S)
        assert np.array_equal(o2[:t], o[:t]) and np.array_equal(lse2[:t], lse[:t])
        assert not np.allclose(o2[t:], o[t:])
    # gradients: dq_i depends only on tokens <= i
    r = A.head_backward(q, k, v, g, scale, row_block=S)
    q2, k2, v2, g2 = q.copy(), k.copy(), v.copy(), g.copy()
    q2[20:] += 1.0; k2[20:] += 1.0; v2[20:] += 1.0; g2[20:] += 1.0
    r2 = A.head_backward(q2, k2, v2, g2, scale, row_block=S)
    assert np.array_equal(r2["dq"][:20], r["dq"][:20])


def test_row_zero_and_k_zero_closed_forms():
    S, D, scale = 29, 8, 0.5
    q, k, v, g = rnd(8, S, D), rnd(9, S, D), rnd(10, S, D), rnd(11, S, D)
    o, lse = A.head_forward(q, k, v, scale)
    assert np.allclose(o[0], v[0], rtol=0, atol=1e-15)
    assert abs(lse[0] - scale * q[0] @ k[0]) <= 1e-14
    # K = 0: uniform attention over the visible prefix
    r = A.head_backward(q, np.zeros_like(k), v, g, scale)
    n = np.arange(1, S + 1)
    assert np.abs(r["o"] - np.cumsum(v, axis=0) / n[:, None]).max() <= 1e-13
    assert np.abs(r["lse"] - np.log(n)).max() <= 1e-13
    dv_closed = np.cumsum((g / n[:, None])[::-1], axis=0)[::-1]       # sum_{i>=j} g_i/(i+1)
    assert np.abs(r["dv"] - dv_closed).max() <= 1e-13
    assert np.abs(r["dq"]).max() <= 1e-15                              # ds rows sum to zero, k = 0


def test_constant_v_shift_in_k_and_equal_keys():
    S, D, scale = 21, 8, 0.3
    q, k, v, g = rnd(12, S, D), rnd(13, S, D), rnd(14, S, D), rnd(15, S, D)
    c = rnd(16, D)
    o, lse = A.head_forward(q, k, np.tile(c, (S, 1)), scale)
    assert np.abs(o - c).max() <= 1e-14
    o1, lse1 = A.head_forward(q, k, v, scale)
    o2, lse2 = A.head_forward(q, k + c, v, scale)
    assert np.abs(o2 - o1).max() <= 1e-12
    assert np.abs(lse2 - lse1 - scale * q @ c).max() <= 1e-12
    # all keys equal: every score row is constant, so sum_j ds_ij = 0 makes dq vanish,
    # and p_ij = 1/(i+1) regardless of q
    r = A.head_backward(q, np.tile(c, (S, 1)), v, g, scale)
    assert np.abs(r["dq"]).max() <= 1e-13
    # total mass: sum_j dv_j = sum_i g_i since every row of p sums to one
    r = A.head_backward(q, k, v, g, scale)
    assert np.abs(r["dv"].sum(axis=0) - g.sum(axis=0)).max() <= 1e-12


def test_noncausal_single_row_is_textbook_softmax():
    S, D, scale = 13, 4, 0.7
    q, k, v = rnd(17, S, D), rnd(18, S, D), rnd(19, S, D)
    o, lse = A.head_forward(q, k, v, scale, causal=False)
    for i in (0, 5, 12):
        w = np.exp(scale * k @ q[i]); w /= w.sum()
        assert np.abs(o[i] - w @ v).max() <= 1e-14
    # last causal row sees every key, so it equals the non-causal row
    oc, lsec = A.head_forward(q, k, v, scale, causal=True)
    assert np.abs(oc[-1] - o[-1]).max() <= 1e-14 and abs(lsec[-1] - lse[-1]) <= 1e-14


@pytest.mark.parametrize("S,D,causal", [(1, 4, True), (2, 4, True), (5, 8, True), (17, 8, True), (17, 4, False), (64, 16, True)])
def test_against_scalar_loops(brute, S, D, causal):
    scale = 1.0 / np.sqrt(D)
    for h in range(2):
        q, k, v, g = (rnd(100 * S + 10 * h + t, S, D) for t in range(4))
        r = A.head_backward(q, k, v, g, scale, causal, row_block=5)
        o, lse = brute.head_forward(q, k, v, scale, causal)
        dq, dk, dv = brute.head_backward(q, k, v, g, scale, causal)
        for name, ref in (("o", o), ("lse", lse), ("dq", dq), ("dk", dk), ("dv", dv)):
            assert np.abs(r[name] - ref).max() <= 1e-12, name


@pytest.mark.parametrize("S,D,causal", [(6, 4, True), (11, 8, True), (7, 4, False)])
def test_gradients_by_central_differences(S, D, causal):
    """Every element of dq, dk, dv against central differences of L = sum(g * o), rel err <= 1e-6."""
    scale = 0.6
    q, k, v, g = (rnd(200 + S + t, S, D) for t in range(4))
    r = A.head_backward(q, k, v, g, scale, causal)

    def loss(q_, k_, v_):
        o, _ = A.head_forward(q_, k_, v_, scale, causal)
        return float((g * o).sum())

    for name, idx in (("dq", 0), ("dk", 1), ("dv", 2)):
        fd = np.empty((S, D))
        for i in range(S):
            for d in range(D):
                args = [q.copy(), k.copy(), v.copy()]
                h = 1e-5 * max(1.0, abs(args[idx][i, d]))
                args[idx][i, d] += h; lp = loss(*args)
                args[idx][i, d] -= 2 * h; lm = loss(*args)
                fd[i, d] = (lp - lm) / (2 * h)
        rel = np.abs(fd - r[name]).max() / np.abs(r[name]).max()
        assert rel <= 1e-6, (name, rel)


def test_scale_homogeneity_and_head_permutation():
    B, H, S, D, scale, a = 2, 3, 19, 8, 0.4, 4.0
    q, k, v, g = (rnd(300 + t, B, H, S, D) for t in range(4))
    r1 = A.attn_bwd_ref(q, k, v, g, scale)
    r2 = A.attn_bwd_ref(q * a, k, v, g, scale / a)
    assert np.abs(r1["o"] - r2["o"]).max() <= 1e-13
    assert np.abs(r1["dk"] - r2["dk"]).max() <= 1e-12
    assert np.abs(r1["dq"] - a * r2["dq"]).max() <= 1e-12
    perm = np.random.default_rng(0).permutation(B * H)

    def sh(x):
        return x.reshape(B * H, *x.shape[2:])[perm].reshape(x.shape)

    r3 = A.attn_bwd_ref(sh(q), sh(k), sh(v), sh(g), scale)
    for n in ("o", "lse", "dq", "dk", "dv"):
        assert np.array_equal(r3[n], sh(r1[n])), n


def test_sampled_rows_and_columns_agree_with_full():
    S, D, scale = 300, 16, 0.25
    q, k, v, g = (rnd(400 + t, S, D) for t in range(4))
    r = A.head_backward(q, k, v, g, scale, row_block=64)
    rows = [0, 1, 31, 32, 150, 298, 299]
    o, lse, dq = A.head_rows(q, k, v, g, rows, scale)
    assert np.abs(o - r["o"][rows]).max() <= 1e-13 and np.abs(lse - r["lse"][rows]).max() <= 1e-13
    assert np.abs(dq - r["dq"][rows]).max() <= 1e-13
    lse_f, delta_f = A.head_stats(q, k, v, g, scale)
    cols = [0, 1, 127, 128, 299]
    dk, dv = A.head_cols(q, k, v, g, cols, lse_f, delta_f, scale, row_block=50)
    assert np.abs(dk - r["dk"][cols]).max() <= 1e-13 and np.abs(dv - r["dv"][cols]).max() <= 1e-13
    lse_t, delta_t = A.head_stats(q, k, v, g, scale, row_start=200)
    cols = [200, 250, 299]
    dk, dv = A.head_cols(q, k, v, g, cols, lse_t, delta_t, scale, row_start=200)
    assert np.abs(dk - r["dk"][cols]).max() <= 1e-13 and np.abs(dv - r["dv"][cols]).max() <= 1e-13
    with pytest.raises(ValueError):
        A.head_cols(q, k, v, g, [100], lse_t, delta_t, scale, row_start=200)


@pytest.mark.parametrize("causal", [True, False])
def test_batched_forward_against_scalar_loops_per_slice(brute, causal):
    """attn_fwd_ref on a [B, H, S, D] batch with B != H and every slice different: each slice must
    equal the scalar-loop result of ITS OWN (b, h) inputs; an implementation that swapped the
    batch and head index (or reused one slice) cannot pass, which the last assertion shows."""
    B, H, S, D, scale = 2, 3, 11, 4, 0.6
    q, k, v = (rnd(500 + t, B, H, S, D) for t in range(3))
    o, lse = A.attn_fwd_ref(q, k, v, scale, causal)
    assert o.shape == (B, H, S, D) and lse.shape == (B, H, S)
    for b in range(B):
        for h in range(H):
            ob, lb = brute.head_forward(q[b, h], k[b, h], v[b, h], scale, causal)
            assert np.abs(o[b, h] - ob).max() <= 1e-12 and np.abs(lse[b, h] - lb).max() <= 1e-12, (b, h)
    # the same call on inputs with batch and head exchanged gives the exchanged result, and that
    # differs from the original wherever (b, h) != (h, b) in flat order: slices are not interchangeable
    ot, _ = A.attn_fwd_ref(*(x.swapaxes(0, 1).copy() for x in (q, k, v)), scale, causal)
    assert np.array_equal(ot.swapaxes(0, 1), o)
    assert not np.allclose(o.reshape(B * H, S, D), ot.reshape(B * H, S, D))
    # and the backward wrapper reports the same forward
    rb = A.attn_bwd_ref(q, k, v, rnd(503, B, H, S, D), scale, causal)
    assert np.array_equal(rb["o"], o) and np.array_equal(rb["lse"], lse)


def test_sampled_rows_and_columns_noncausal(brute):
    """head_rows / head_stats / head_cols with causal=False: every row sees every key.  Pinned
    against the full non-causal result and, independently, against the scalar loops."""
    S, D, scale = 37, 8, 0.35
    q, k, v, g = (rnd(600 + t, S, D) for t in range(4))
    r = A.head_backward(q, k, v, g, scale, causal=False, row_block=16)
    dq_b, dk_b, dv_b = brute.head_backward(q, k, v, g, scale, False)
    o_b, lse_b = brute.head_forward(q, k, v, scale, False)
    rows = [0, 1, 17, 36]
    o, lse, dq = A.head_rows(q, k, v, g, rows, scale, causal=False)
    assert np.abs(o - r["o"][rows]).max() <= 1e-13 and np.abs(lse - r["lse"][rows]).max() <= 1e-13
    assert np.abs(dq - r["dq"][rows]).max() <= 1e-13
    assert np.abs(o - o_b[rows]).max() <= 1e-12 and np.abs(lse - lse_b[rows]).max() <= 1e-12 and np.abs(dq - dq_b[rows]).max() <= 1e-12
    lse_f, delta_f = A.head_stats(q, k, v, g, scale, causal=False)
    assert np.abs(lse_f - lse_b).max() <= 1e-12
    cols = [0, 5, 36]
    dk, dv = A.head_cols(q, k, v, g, cols, lse_f, delta_f, scale, causal=False, row_block=10)
    assert np.abs(dk - r["dk"][cols]).max() <= 1e-13 and np.abs(dv - r["dv"][cols]).max() <= 1e-13
    assert np.abs(dk - dk_b[cols]).max() <= 1e-12 and np.abs(dv - dv_b[cols]).max() <= 1e-12
    # the causal result is a different one: the flag is not ignored
    dkc, _ = A.head_cols(q, k, v, g, cols, *A.head_stats(q, k, v, g, scale, causal=True), scale, causal=True)
    assert not np.allclose(dkc, dk)
    # a row window is refused without the causal mask (column j needs every row)
    with pytest.raises(ValueError):
        A.head_cols(q, k, v, g, [20], lse_f[10:], delta_f[10:], scale, causal=False, row_start=10)


def test_flop_counter_matches_table1():
    for line in (GOLDEN / "table1_attention_flops.txt").read_text().splitlines():
        if line.startswith("#") or not line.strip():
            continue
        b, hidden, s, fwd, bwd = (int(x) for x in line.split())
        D = 128
        f = A.attn_flops(b, hidden // D, s, D, causal=False)
        assert f["fwd"] == fwd and f["bwd_table1"] == bwd
        fc = A.attn_flops(b, hidden // D, s, D, causal=True)
        assert fc["fwd"] * 2 * s == fwd * (s + 1)          # exact triangle, not s^2/2
        assert fc["fwd_bwd"] == 14 * b * (hidden // D) * D * (s * (s + 1) // 2)
