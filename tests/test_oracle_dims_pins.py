"""Pins of the oracle for key and value dimensions that differ (d_k for q, k; d_v for v, out; state
[d_k][d_v]), CPU only: at d_k = d_v it must reproduce the separately pinned C oracle; at d_k != d_v it
must equal that oracle on inputs padded with zero columns (an exact identity: zero features add
nothing to a dot product, and the padded rows / columns of the state stay zero), and its gradients
must match exact unit-step finite differences."""
import numpy as np
import pytest


def rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def make(B, H, N, dk, dv, seed):
    q, k = rand((B, H, N, dk), seed), rand((B, H, N, dk), seed + 1)
    v, do = rand((B, H, N, dv), seed + 2), rand((B, H, N, dv), seed + 3)
    s0, G = rand((B, H, dk, dv), seed + 4), rand((B, H, dk, dv), seed + 5)
    return q, k, v, do, s0, G


def pad(x, axis, to):
    w = [(0, 0)] * x.ndim
    w[axis] = (0, to - x.shape[axis])
    return np.pad(x, w)


def test_equal_dims_reproduce_the_c_oracle(oracle):
    B, H, N, D = 2, 3, 21, 4
    q, k, v, do, s0, G = make(B, H, N, D, D, 1)
    decay = np.array([0.8, 0.95, 1.0])
    o, kv = oracle.dims_fwd_brute(q, k, v, decay, s0)
    o2, kv2 = oracle.fwd_brute(q, k, v, decay, s0)
    np.testing.assert_allclose(o, o2, rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(kv, kv2, rtol=1e-11, atol=1e-11)
    for got, ref in zip(oracle.dims_bwd_brute(q, k, v, do, decay, s0, G), oracle.bwd_brute(q, k, v, do, decay, s0, G)):
        np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-11)
    lg = np.log(np.random.default_rng(2).uniform(0.5, 1.0, (B, H, N)))
    o, kv = oracle.dims_fwd_brute(q, k, v, None, s0, log_g=lg)
    o2, kv2 = oracle.gated_fwd_brute(q, k, v, lg, s0)
    np.testing.assert_allclose(o, o2, rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(kv, kv2, rtol=1e-11, atol=1e-11)
    for got, ref in zip(oracle.dims_bwd_brute(q, k, v, do, None, s0, G, log_g=lg), oracle.gated_bwd_brute(q, k, v, do, lg, s0, G)):
        np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-10)


@pytest.mark.parametrize("dk,dv", [(2, 5), (6, 3)])
def test_unequal_dims_equal_the_zero_padded_problem(oracle, dk, dv):
    B, H, N = 1, 2, 17
    D = max(dk, dv)
    q, k, v, do, s0, G = make(B, H, N, dk, dv, 10 + dk)
    decay = np.array([0.9, 0.97])
    qp, kp, vp, dop = pad(q, 3, D), pad(k, 3, D), pad(v, 3, D), pad(do, 3, D)
    s0p, Gp = pad(pad(s0, 2, D), 3, D), pad(pad(G, 2, D), 3, D)
    o, kv = oracle.dims_fwd_brute(q, k, v, decay, s0)
    o2, kv2 = oracle.fwd_brute(qp, kp, vp, decay, s0p)
    np.testing.assert_allclose(o, o2[..., :dv], rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(kv, kv2[:, :, :dk, :dv], rtol=1e-11, atol=1e-11)
    assert np.all(o2[..., dv:] == 0) and np.all(kv2[:, :, dk:, :] == 0) and np.all(kv2[:, :, :, dv:] == 0)
    dq, dkk, dvv, din = oracle.dims_bwd_brute(q, k, v, do, decay, s0, G)
    dq2, dk2, dv2, din2 = oracle.bwd_brute(qp, kp, vp, dop, decay, s0p, Gp)
    np.testing.assert_allclose(dq, dq2[..., :dk], rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dkk, dk2[..., :dk], rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dvv, dv2[..., :dv], rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(din, din2[:, :, :dk, :dv], rtol=1e-11, atol=1e-11)
    lg = np.log(np.random.default_rng(3).uniform(0.6, 1.0, (B, H, N)))
    got = oracle.dims_bwd_brute(q, k, v, do, None, s0, G, log_g=lg)
    ref = oracle.gated_bwd_brute(qp, kp, vp, dop, lg, s0p, Gp)
    for g, r, sl in zip(got, ref, ((..., slice(0, dk)), (..., slice(0, dk)), (..., slice(0, dv)), (...,),
                                   (slice(None), slice(None), slice(0, dk), slice(0, dv)))):
        np.testing.assert_allclose(g, r[sl], rtol=1e-10, atol=1e-10)


def test_unequal_dims_gradients_by_finite_differences(oracle):
    """L = sum(out * dout) + <kv_out, G> is linear in each of q, k, v, kv_in alone: a unit step is exact."""
    B, H, N, dk, dv = 1, 2, 7, 3, 5
    q, k, v, do, s0, G = make(B, H, N, dk, dv, 30)
    decay = np.array([0.85, 1.0])

    def L(q_, k_, v_, s_):
        o, kv = oracle.dims_fwd_brute(q_, k_, v_, decay, s_)
        return float(np.sum(o * do) + np.sum(kv * G))

    dq, dkk, dvv, din = oracle.dims_bwd_brute(q, k, v, do, decay, s0, G)
    L0 = L(q, k, v, s0)
    for which, grad, idxs in ((0, dq, [(0, 0, 0, 0), (0, 1, 6, 2)]), (1, dkk, [(0, 0, 3, 1), (0, 1, 0, 2)]),
                              (2, dvv, [(0, 0, 6, 4), (0, 1, 2, 0)]), (3, din, [(0, 0, 2, 4), (0, 1, 0, 0)])):
        for idx in idxs:
            args = [q.copy(), k.copy(), v.copy(), s0.copy()]
            args[which][idx] += 1.0
            np.testing.assert_allclose(L(*args) - L0, grad[idx], rtol=1e-10, atol=1e-10)
