"""Pins of the oracle's grouped key/value heads (CPU only): expansion is a repeat of heads, its
gradient the sum over a group; checked by hand values and by finite differences through the attention."""
import numpy as np


def test_expand_and_reduce_by_hand(oracle):
    x = np.arange(2 * 2 * 1 * 1, dtype=np.float64).reshape(2, 2, 1, 1)      # heads (0, 1) and (2, 3)
    e = oracle.group_expand(x, 3)
    assert e.shape == (2, 6, 1, 1)
    assert e[:, :, 0, 0].tolist() == [[0, 0, 0, 1, 1, 1], [2, 2, 2, 3, 3, 3]]
    d = np.arange(2 * 6, dtype=np.float64).reshape(2, 6, 1, 1)
    r = oracle.group_reduce(d, 3)
    assert r[:, :, 0, 0].tolist() == [[0 + 1 + 2, 3 + 4 + 5], [6 + 7 + 8, 9 + 10 + 11]]


def test_shared_head_gradient_by_finite_differences(oracle):
    rng = np.random.default_rng(5)
    B, H, G, N, D = 1, 4, 2, 6, 3
    q, do = rng.standard_normal((B, H, N, D)), rng.standard_normal((B, H, N, D))
    k, v = rng.standard_normal((B, H // G, N, D)), rng.standard_normal((B, H // G, N, D))
    decay = np.array([0.7, 0.8, 0.9, 1.0])
    L = lambda k_, v_: float(np.sum(oracle.fwd_brute(q, oracle.group_expand(k_, G), oracle.group_expand(v_, G), decay)[0] * do))
    _, dk, dv, _ = oracle.bwd_brute(q, oracle.group_expand(k, G), oracle.group_expand(v, G), do, decay)
    dk, dv = oracle.group_reduce(dk, G), oracle.group_reduce(dv, G)
    L0 = L(k, v)
    for idx in [(0, 0, 0, 0), (0, 1, 5, 2), (0, 1, 2, 1)]:
        k2, v2 = k.copy(), v.copy()
        k2[idx] += 1.0
        v2[idx] += 1.0
        np.testing.assert_allclose(L(k2, v) - L0, dk[idx], rtol=1e-10, atol=1e-10)   # the loss is linear in k alone
        np.testing.assert_allclose(L(k, v2) - L0, dv[idx], rtol=1e-10, atol=1e-10)
