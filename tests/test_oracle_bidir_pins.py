"""Pins of the oracle's bidirectional (unmasked) linear attention, O = (Q K^T) V = Q (K^T V) of
Sec. 3.1, Eq. (3), to things other than itself (CPU only): a hand-computed example, the separately
pinned causal oracle (causal + anti-causal - diagonal), invariance under a reordering of the
key/value tokens, exact finite differences of the trilinear loss, and the two forms against each other."""
import json
import os

import numpy as np

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hand_example_bidirectional.json")


def rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_hand_example(oracle):
    g = json.load(open(GOLD))
    a = lambda name: np.array(g[name], dtype=np.float64)[None, None]
    q, k, v, do = a("q"), a("k"), a("v"), a("dout")
    assert np.array_equal(oracle.bidir_state(k, v), a("kv"))
    assert np.array_equal(oracle.bidir_state(q, do), a("dkv"))
    assert np.array_equal(oracle.bidir_fwd_left(q, k, v), a("out"))
    assert np.array_equal(oracle.bidir_fwd_right(q, a("kv")), a("out"))
    dq, dk, dv = oracle.bidir_bwd_left(q, k, v, do)
    assert np.array_equal(dq, a("dq")) and np.array_equal(dk, a("dk")) and np.array_equal(dv, a("dv"))
    rows = np.array([[0, 0, 0], [0, 0, 1]])
    assert np.array_equal(oracle.bidir_fwd_rows(q, k, v, rows), a("out")[0, 0])
    rq, rk, rv = oracle.bidir_bwd_rows(q, k, v, do, rows)
    assert np.array_equal(rq, a("dq")[0, 0]) and np.array_equal(rk, a("dk")[0, 0]) and np.array_equal(rv, a("dv")[0, 0])


def test_equals_causal_plus_anticausal_minus_diagonal(oracle):
    """Without decay the unmasked sum over all i splits into i <= s (the causal oracle), i >= s (the
    causal oracle on the reversed sequence) and the doubly counted i = s."""
    B, H, N, D = 2, 3, 37, 5
    q, k, v = rand((B, H, N, D), 1), rand((B, H, N, D), 2), rand((B, H, N, D), 3)
    ones = np.ones(H)
    rev = lambda x: np.ascontiguousarray(x[:, :, ::-1])
    causal = oracle.fwd_brute(q, k, v, ones)[0]
    anti = rev(oracle.fwd_brute(rev(q), rev(k), rev(v), ones)[0])
    diag = np.sum(q * k, axis=-1, keepdims=True) * v
    np.testing.assert_allclose(oracle.bidir_fwd_left(q, k, v), causal + anti - diag, rtol=1e-12, atol=1e-12)
    # the state is the causal oracle's final state from zero
    np.testing.assert_allclose(oracle.bidir_state(k, v), oracle.fwd_brute(q, k, v, ones)[1], rtol=1e-12, atol=1e-12)


def test_gradients_equal_causal_plus_anticausal_minus_diagonal(oracle):
    B, H, N, D = 1, 2, 23, 4
    q, k, v, do = (rand((B, H, N, D), s) for s in (4, 5, 6, 7))
    ones = np.ones(H)
    rev = lambda x: np.ascontiguousarray(x[:, :, ::-1])
    c = oracle.bwd_brute(q, k, v, do, ones)[:3]
    a = [rev(x) for x in oracle.bwd_brute(rev(q), rev(k), rev(v), rev(do), ones)[:3]]
    dov, qk = np.sum(do * v, axis=-1, keepdims=True), np.sum(q * k, axis=-1, keepdims=True)
    diag = (dov * k, dov * q, qk * do)
    got = oracle.bidir_bwd_left(q, k, v, do)
    for g, cc, aa, dd in zip(got, c, a, diag):
        np.testing.assert_allclose(g, cc + aa - dd, rtol=1e-12, atol=1e-12)


def test_key_value_order_does_not_matter(oracle):
    B, H, N, D = 1, 2, 19, 6
    q, k, v = rand((B, H, N, D), 8), rand((B, H, N, D), 9), rand((B, H, N, D), 10)
    perm = np.random.default_rng(11).permutation(N)
    np.testing.assert_allclose(oracle.bidir_fwd_left(q, k[:, :, perm], v[:, :, perm]), oracle.bidir_fwd_left(q, k, v),
                               rtol=1e-12, atol=1e-12)
    # permuting k alone is a different function
    assert np.abs(oracle.bidir_fwd_left(q, k[:, :, perm], v) - oracle.bidir_fwd_left(q, k, v)).max() > 1e-3


def test_left_and_right_products_agree_and_state_is_additive(oracle):
    B, H, N, D = 2, 2, 41, 7
    q, k, v, do = (rand((B, H, N, D), s) for s in (12, 13, 14, 15))
    kv = oracle.bidir_state(k, v)
    assert kv.shape == (B, H, D, D)
    np.testing.assert_allclose(kv[1, 0, 2, 5], np.sum(k[1, 0, :, 2] * v[1, 0, :, 5]), rtol=1e-12)   # rows: key feature
    np.testing.assert_allclose(oracle.bidir_fwd_right(q, kv), oracle.bidir_fwd_left(q, k, v), rtol=1e-11, atol=1e-11)
    # the state of a sequence is the sum of the states of its pieces (what sub-sequences exchange)
    parts = sum(oracle.bidir_state(k[:, :, a:b], v[:, :, a:b]) for a, b in ((0, 10), (10, 11), (11, 41)))
    np.testing.assert_allclose(parts, kv, rtol=1e-12, atol=1e-12)
    # right-product gradients: dQ = dO KV^T, dK = V dKV^T, dV = K dKV with dKV = Q^T dO
    dkv = oracle.bidir_state(q, do)
    dq, dk, dv = oracle.bidir_bwd_left(q, k, v, do)
    np.testing.assert_allclose(dq, do @ np.swapaxes(kv, -1, -2), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dk, v @ np.swapaxes(dkv, -1, -2), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dv, k @ dkv, rtol=1e-11, atol=1e-11)


def test_gradients_by_finite_differences(oracle):
    """L = sum(O * dout) is linear in each of q, k, v alone, so a unit step gives the derivative exactly."""
    B, H, N, D = 1, 2, 9, 3
    q, k, v, do = (rand((B, H, N, D), s) for s in (16, 17, 18, 19))
    L = lambda q_, k_, v_: float(np.sum(oracle.bidir_fwd_left(q_, k_, v_) * do))
    dq, dk, dv = oracle.bidir_bwd_left(q, k, v, do)
    L0 = L(q, k, v)
    for idx in [(0, 0, 0, 0), (0, 1, 8, 2), (0, 1, 4, 1), (0, 0, 7, 2)]:
        for which, grad in enumerate((dq, dk, dv)):
            args = [q.copy(), k.copy(), v.copy()]
            args[which][idx] += 1.0
            np.testing.assert_allclose(L(*args) - L0, grad[idx], rtol=1e-10, atol=1e-10)


def test_sampled_rows_match_full(oracle):
    B, H, N, D = 2, 3, 29, 4
    q, k, v, do = (rand((B, H, N, D), s) for s in (20, 21, 22, 23))
    rows = np.array([[0, 0, 0], [1, 2, 28], [0, 1, 13], [1, 0, 5]])
    b, h, s = rows[:, 0], rows[:, 1], rows[:, 2]
    np.testing.assert_allclose(oracle.bidir_fwd_rows(q, k, v, rows), oracle.bidir_fwd_left(q, k, v)[b, h, s], rtol=1e-12, atol=1e-12)
    full = oracle.bidir_bwd_left(q, k, v, do)
    for r, f in zip(oracle.bidir_bwd_rows(q, k, v, do, rows), full):
        np.testing.assert_allclose(r, f[b, h, s], rtol=1e-12, atol=1e-12)
