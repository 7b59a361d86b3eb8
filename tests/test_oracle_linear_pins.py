"""Pins of the linear-layer oracle to things other than itself: scalar triple loops, the
identity weight, linearity and central finite differences (Table 1's QKV linear column:
one product forward, one each for backward B and backward W)."""
import numpy as np

from oracle import linear_ref as L


def _case(M, K, N, seed=0):
    r = np.random.default_rng(seed)
    return r.standard_normal((M, K)), r.standard_normal((K, N)), r.standard_normal((M, N))


def test_triple_loops_on_tiny_shapes():
    for M, K, N in ((1, 1, 1), (3, 5, 2), (4, 7, 6)):
        a, w, g = _case(M, K, N, seed=M + K + N)
        out = np.zeros((M, N)); da = np.zeros((M, K)); dw = np.zeros((K, N))
        for m in range(M):
            for n in range(N):
                for k in range(K):
                    out[m, n] += a[m, k] * w[k, n]
                    da[m, k] += g[m, n] * w[k, n]
                    dw[k, n] += a[m, k] * g[m, n]
        ref = L.linear_bwd_ref(a, w, g)
        assert np.allclose(L.linear_fwd_ref(a, w), out, rtol=0, atol=1e-12)
        assert np.allclose(ref["da"], da, rtol=0, atol=1e-12) and np.allclose(ref["dw"], dw, rtol=0, atol=1e-12)


def test_identity_weight_and_linearity():
    a, w, g = _case(6, 5, 5, seed=3)
    eye = np.eye(5)
    assert np.array_equal(L.linear_fwd_ref(a, eye), a)
    b = L.linear_bwd_ref(a, eye, g)
    assert np.array_equal(b["da"], g) and np.allclose(b["dw"], a.T @ g)
    a2 = np.random.default_rng(4).standard_normal(a.shape)
    assert np.allclose(L.linear_fwd_ref(2 * a + a2, w), 2 * L.linear_fwd_ref(a, w) + L.linear_fwd_ref(a2, w), atol=1e-12)
    # a transposed operand by mistake would change the shapes or fail this asymmetric case
    assert L.linear_bwd_ref(a, w, g)["da"].shape == a.shape and L.linear_bwd_ref(a, w, g)["dw"].shape == w.shape


def test_gradients_by_central_differences():
    a, w, g = _case(4, 6, 3, seed=9)
    loss = lambda a_, w_: float((g * L.linear_fwd_ref(a_, w_)).sum())
    ref = L.linear_bwd_ref(a, w, g)
    h = 1e-6
    for name, x, grad in (("da", a, ref["da"]), ("dw", w, ref["dw"])):
        for idx in np.ndindex(x.shape):
            xp, xm = x.copy(), x.copy()
            xp[idx] += h; xm[idx] -= h
            num = (loss(xp, w) - loss(xm, w)) / (2 * h) if name == "da" else (loss(a, xp) - loss(a, xm)) / (2 * h)
            assert abs(num - grad[idx]) <= 1e-6 * max(1.0, abs(grad[idx])), (name, idx)


def test_flop_count_matches_table1():
    b, s, h = 2, 4096, 1024
    assert L.linear_flops(b * s, h, 3 * h) == 6 * b * s * h * h
