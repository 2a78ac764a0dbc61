"""Pins of the oracle's Norm(.) (root-mean-square normalisation of every output row, the reading of the
Norm in O = Norm((Q K^T (.) M) V) of Sec. 3.1, Eq. (2)) to things other than itself (CPU only)."""
import numpy as np
import pytest


def test_hand_values(oracle):
    # o = (3, 4): mean square 12.5; (6, 8, 0, 0): mean square 25 -> rstd 1/5
    y, rstd = oracle.norm_fwd(np.array([[3.0, 4.0]]), 0.0)
    np.testing.assert_allclose(rstd, [1.0 / np.sqrt(12.5)], rtol=1e-15)
    np.testing.assert_allclose(y, [[3.0 / np.sqrt(12.5), 4.0 / np.sqrt(12.5)]], rtol=1e-15)
    y, rstd = oracle.norm_fwd(np.array([[6.0, 8.0, 0.0, 0.0]]), 0.0)
    np.testing.assert_allclose(rstd, [0.2], rtol=1e-15)
    np.testing.assert_allclose(y, [[1.2, 1.6, 0.0, 0.0]], rtol=1e-15)
    # eps enters under the root: o = (0, 0), eps = 0.25 -> rstd 2, y = 0
    y, rstd = oracle.norm_fwd(np.zeros((1, 2)), 0.25)
    np.testing.assert_allclose(rstd, [2.0])
    assert np.all(y == 0)


def test_unit_rms_and_scale_invariance(oracle):
    rng = np.random.default_rng(1)
    o = rng.standard_normal((2, 3, 7, 16))
    y, rstd = oracle.norm_fwd(o, 0.0)
    np.testing.assert_allclose(np.mean(y * y, axis=-1), 1.0, rtol=1e-13)
    y2, rstd2 = oracle.norm_fwd(3.5 * o, 0.0)
    np.testing.assert_allclose(y2, y, rtol=1e-13)
    np.testing.assert_allclose(rstd2, rstd / 3.5, rtol=1e-13)
    # rows are independent: permuting tokens permutes the result
    perm = rng.permutation(7)
    np.testing.assert_array_equal(oracle.norm_fwd(o[:, :, perm], 0.0)[0], y[:, :, perm])


@pytest.mark.parametrize("eps", [0.0, 1e-3, 0.5])
def test_backward_by_finite_differences(oracle, eps):
    rng = np.random.default_rng(2)
    o = rng.standard_normal((1, 2, 5, 6))
    dy = rng.standard_normal(o.shape)
    y, rstd = oracle.norm_fwd(o, eps)
    do = oracle.norm_bwd(dy, y, rstd)
    L = lambda x: float(np.sum(oracle.norm_fwd(x, eps)[0] * dy))
    h = 1e-6
    for idx in [(0, 0, 0, 0), (0, 1, 4, 5), (0, 1, 2, 3), (0, 0, 3, 1)]:
        p, m = o.copy(), o.copy()
        p[idx] += h
        m[idx] -= h
        np.testing.assert_allclose(do[idx], (L(p) - L(m)) / (2 * h), rtol=1e-7, atol=1e-9)
    if eps == 0.0:
        # y does not change along o (scale invariance), so the gradient has no component along o
        np.testing.assert_allclose(np.sum(do * o, axis=-1), 0.0, atol=1e-12)


def test_composed_with_attention_by_finite_differences(oracle):
    """Whole normalised path: L = sum(Norm(o(q,k,v)) * dy); dq from bwd_brute(dout = norm_bwd(...))."""
    rng = np.random.default_rng(3)
    B, H, N, D = 1, 2, 8, 4
    q, k, v, dy = (rng.standard_normal((B, H, N, D)) for _ in range(4))
    decay = np.array([0.8, 0.95])
    eps = 1e-4
    def L(q_, k_, v_):
        return float(np.sum(oracle.norm_fwd(oracle.fwd_brute(q_, k_, v_, decay)[0], eps)[0] * dy))
    y, rstd = oracle.norm_fwd(oracle.fwd_brute(q, k, v, decay)[0], eps)
    dq, dk, dv, _ = oracle.bwd_brute(q, k, v, oracle.norm_bwd(dy, y, rstd), decay)
    h = 1e-6
    for which, grad in (("q", dq), ("k", dk), ("v", dv)):
        for idx in [(0, 0, 2, 1), (0, 1, 7, 3), (0, 1, 0, 0)]:
            args = {"q": q.copy(), "k": k.copy(), "v": v.copy()}
            a2 = {n: x.copy() for n, x in args.items()}
            args[which][idx] += h
            a2[which][idx] -= h
            fd = (L(args["q"], args["k"], args["v"]) - L(a2["q"], a2["k"], a2["v"])) / (2 * h)
            np.testing.assert_allclose(grad[idx], fd, rtol=1e-6, atol=1e-8)
