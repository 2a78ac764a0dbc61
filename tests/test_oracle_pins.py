"""Pins of the fp64 oracle to things other than itself (CPU only).

Each test ties a form of the oracle to what the paper or the mathematics fixes:
hand-computed values (tests/golden/hand_examples.json), textbook routines at
lambda = 1, closed forms, exact finite differences, structural identities, and
agreement of the brute-force definition with the recurrent and chunked forms
and with T-way splitting (the premise of Alg. 2 / Alg. 3).
"""
import json
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
TOL = 1e-11


def rel(a, b):
    return np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300)


def rand_case(seed, B=2, H=3, N=24, D=5, lam=None, states=True):
    rng = np.random.default_rng(seed)
    q, k, v, do = (rng.standard_normal((B, H, N, D)) for _ in range(4))
    decay = np.array(lam if lam is not None else rng.uniform(0.6, 1.0, H))
    kv_in = rng.standard_normal((B, H, D, D)) if states else None
    g = rng.standard_normal((B, H, D, D)) if states else None
    return q, k, v, do, decay, kv_in, g


def loss(o, kv_out, do, g):
    return float(np.sum(o * do) + (np.sum(kv_out * g) if g is not None else 0.0))


# ---------------------------------------------------------------- hand examples
def _examples():
    with open(os.path.join(HERE, "golden", "hand_examples.json")) as f:
        return json.load(f)["examples"]


@pytest.mark.parametrize("ex", _examples(), ids=lambda e: e["name"])
@pytest.mark.parametrize("form", ["brute", "recurrent", "chunk1", "chunkN"])
def test_hand_examples(oracle, ex, form):
    a = lambda x: None if x is None else np.array(x, dtype=np.float64)[None, None]
    q, k, v, do = a(ex["q"]), a(ex["k"]), a(ex["v"]), a(ex["dout"])
    decay = np.array([ex["lambda"]])
    kv_in, g = a(ex["kv_in"]), a(ex["dkv_out"])
    if form == "brute":
        o, kvo = oracle.fwd_brute(q, k, v, decay, kv_in)
        dq, dk, dv, gi = oracle.bwd_brute(q, k, v, do, decay, kv_in, g)
    elif form == "recurrent":
        o, kvo = oracle.fwd_recurrent(q, k, v, decay, kv_in)
        dq, dk, dv, gi = oracle.bwd_recurrent(q, k, v, do, decay, kv_in, g)
    else:
        C = 1 if form == "chunk1" else ex["N"]
        o, kvo = oracle.fwd_chunked(q, k, v, decay, C, kv_in)
        dq, dk, dv, gi = oracle.bwd_chunked(q, k, v, do, decay, C, kv_in, g)
    for got, key in [(o, "out"), (kvo, "kv_out"), (dq, "dq"), (dk, "dk"), (dv, "dv"), (gi, "dkv_in")]:
        np.testing.assert_allclose(got[0, 0], np.array(ex[key], dtype=np.float64), rtol=0, atol=1e-13, err_msg=key)


# ---------------------------------------------------------------- textbook, lambda = 1
def test_lambda_one_is_tril_matmul(oracle):
    """lambda = 1 is ordinary causal linear attention: O = tril(Q K^T) V, kv_out = K0 + K^T V."""
    q, k, v, do, _, kv_in, _ = rand_case(1, lam=[1.0, 1.0, 1.0])
    decay = np.ones(3)
    o, kvo = oracle.fwd_brute(q, k, v, decay, kv_in)
    for b in range(2):
        for h in range(3):
            ref = np.tril(q[b, h] @ k[b, h].T) @ v[b, h] + q[b, h] @ kv_in[b, h]
            assert rel(o[b, h], ref) < TOL
            assert rel(kvo[b, h], kv_in[b, h] + k[b, h].T @ v[b, h]) < TOL


def test_lambda_one_backward_is_triu_matmul(oracle):
    """At lambda = 1 and zero states: dQ = tril(dO V^T) K, dK = tril(dO V^T)^T Q, dV = tril(Q K^T)^T dO."""
    q, k, v, do, _, _, _ = rand_case(2, states=False)
    decay = np.ones(3)
    dq, dk, dv, gi = oracle.bwd_brute(q, k, v, do, decay)
    for b in range(2):
        for h in range(3):
            ds = np.tril(do[b, h] @ v[b, h].T)
            s = np.tril(q[b, h] @ k[b, h].T)
            assert rel(dq[b, h], ds @ k[b, h]) < TOL
            assert rel(dk[b, h], ds.T @ q[b, h]) < TOL
            assert rel(dv[b, h], s.T @ do[b, h]) < TOL
            assert rel(gi[b, h], q[b, h].T @ do[b, h]) < TOL


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("lam", [1.0, 0.9, 0.5, 1.0 - 2.0 ** -12])
def test_geometric_series(oracle, lam):
    """q_s = k_s = e_1, v_s = c  =>  o_s = c (1 - lam^s)/(1 - lam)  (= s c at lam = 1)."""
    N, D = 40, 4
    c = np.array([1.0, -2.0, 0.5, 3.0])
    q = np.zeros((1, 1, N, D)); q[..., 0] = 1.0
    k = q.copy()
    v = np.broadcast_to(c, (1, 1, N, D)).copy()
    s = np.arange(1, N + 1, dtype=np.float64)
    geo = s if lam == 1.0 else (1.0 - lam ** s) / (1.0 - lam)
    for fwd in (oracle.fwd_brute, oracle.fwd_recurrent, lambda *a: oracle.fwd_chunked(*a, 8)):
        o, kvo = fwd(q, k, v, np.array([lam]))
        assert rel(o[0, 0], geo[:, None] * c[None, :]) < 1e-9
        assert rel(kvo[0, 0, 0], geo[-1] * c) < 1e-9
        assert np.all(kvo[0, 0, 1:] == 0.0)


def test_single_impulse_and_causality(oracle):
    """Only token j carries a key/value: o_s = lam^(s-j) (q_s.k_j) v_j for s >= j, exactly 0 before."""
    N, D, j, lam = 17, 3, 6, 0.8   # j is 1-based
    rng = np.random.default_rng(3)
    q = rng.standard_normal((1, 1, N, D))
    k = np.zeros((1, 1, N, D)); v = np.zeros((1, 1, N, D))
    kj, vj = rng.standard_normal(D), rng.standard_normal(D)
    k[0, 0, j - 1], v[0, 0, j - 1] = kj, vj
    for fwd in (oracle.fwd_brute, oracle.fwd_recurrent, lambda *a: oracle.fwd_chunked(*a, 1)):
        o, kvo = fwd(q, k, v, np.array([lam]))
        assert np.all(o[0, 0, : j - 1] == 0.0)
        for s in range(j, N + 1):
            assert rel(o[0, 0, s - 1], lam ** (s - j) * (q[0, 0, s - 1] @ kj) * vj) < 1e-12
        assert rel(kvo[0, 0], lam ** (N - j) * np.outer(kj, vj)) < 1e-12


def test_carried_state_row_factor_is_one_based(oracle):
    """fwd(K0) - fwd(0) = Lambda Q K0 with Lambda = diag(lam^1..lam^N): the first
    token already sees the incoming state decayed once."""
    q, k, v, _, decay, kv_in, _ = rand_case(4, B=1, H=2, N=9, D=3)
    o1, kv1 = oracle.fwd_brute(q, k, v, decay, kv_in)
    o0, kv0 = oracle.fwd_brute(q, k, v, decay, None)
    for h in range(2):
        lam = decay[h]
        pw = lam ** np.arange(1, 10)
        assert rel((o1 - o0)[0, h], pw[:, None] * (q[0, h] @ kv_in[0, h])) < TOL
        assert rel((kv1 - kv0)[0, h], lam ** 9 * kv_in[0, h]) < TOL


# ---------------------------------------------------------------- gradients
def test_finite_differences_are_exact(oracle):
    """The loss is linear in each of Q, K, V, K0 separately, so central
    differences carry no truncation error."""
    q, k, v, do, decay, kv_in, g = rand_case(5, B=1, H=2, N=7, D=3)
    dq, dk, dv, gi = oracle.bwd_brute(q, k, v, do, decay, kv_in, g)

    def L(q_, k_, v_, s_):
        o, kvo = oracle.fwd_brute(q_, k_, v_, decay, s_)
        return loss(o, kvo, do, g)

    rng = np.random.default_rng(6)
    eps = 0.5
    for which, grad in (("q", dq), ("k", dk), ("v", dv), ("s", gi)):
        base = {"q": q, "k": k, "v": v, "s": kv_in}
        for _ in range(12):
            idx = tuple(rng.integers(0, n) for n in base[which].shape)
            plus = {n: a.copy() for n, a in base.items()}
            minus = {n: a.copy() for n, a in base.items()}
            plus[which][idx] += eps
            minus[which][idx] -= eps
            fd = (L(plus["q"], plus["k"], plus["v"], plus["s"]) -
                  L(minus["q"], minus["k"], minus["v"], minus["s"])) / (2 * eps)
            assert abs(fd - grad[idx]) <= 1e-9 * max(1.0, abs(fd)), (which, idx, fd, grad[idx])


def test_backward_is_three_forwards(oracle):
    """dQ = fwd(q<-dO, k<-V, v<-K, K0<-K0^T); with zero incoming gradient state
    dK and dV are time-reversed forwards and dkv_in = lam * kv_out(k<-rev Q, v<-rev dO)."""
    q, k, v, do, decay, kv_in, _ = rand_case(7)
    dq, dk, dv, gi = oracle.bwd_brute(q, k, v, do, decay, kv_in, None)
    dq2, _ = oracle.fwd_brute(do, v, k, decay, np.swapaxes(kv_in, -1, -2))
    assert rel(dq, dq2) < TOL
    r = lambda x: x[:, :, ::-1].copy()
    dv2, kvr = oracle.fwd_brute(r(k), r(q), r(do), decay)
    dk2, _ = oracle.fwd_brute(r(v), r(do), r(q), decay)
    assert rel(dv, r(dv2)) < TOL
    assert rel(dk, r(dk2)) < TOL
    assert rel(gi, decay[None, :, None, None] * kvr) < TOL


# ---------------------------------------------------------------- forms agree
@pytest.mark.parametrize("states", [False, True])
def test_forms_agree(oracle, states):
    q, k, v, do, decay, kv_in, g = rand_case(8, states=states)
    o, kvo = oracle.fwd_brute(q, k, v, decay, kv_in)
    grads = oracle.bwd_brute(q, k, v, do, decay, kv_in, g)
    o2, kvo2 = oracle.fwd_recurrent(q, k, v, decay, kv_in)
    assert rel(o2, o) < TOL and rel(kvo2, kvo) < TOL
    for a, b in zip(oracle.bwd_recurrent(q, k, v, do, decay, kv_in, g), grads):
        assert rel(a, b) < TOL
    for C in (1, 2, 3, 8, 24):
        o3, kvo3 = oracle.fwd_chunked(q, k, v, decay, C, kv_in)
        assert rel(o3, o) < TOL and rel(kvo3, kvo) < TOL, C
        for a, b in zip(oracle.bwd_chunked(q, k, v, do, decay, C, kv_in, g), grads):
            assert rel(a, b) < TOL, C


@pytest.mark.parametrize("T", [1, 2, 4])
def test_split_with_state_passing_equals_unsplit(oracle, T):
    q, k, v, do, decay, kv_in, g = rand_case(9)
    o, kvo = oracle.fwd_brute(q, k, v, decay, kv_in)
    grads = oracle.bwd_brute(q, k, v, do, decay, kv_in, g)
    for fwd, bwd, kw in ((oracle.fwd_brute, oracle.bwd_brute, {}),
                         (oracle.fwd_recurrent, oracle.bwd_recurrent, {}),
                         (oracle.fwd_chunked, oracle.bwd_chunked, {"chunk": 3})):
        o2, kvo2, kv_ins = oracle.fwd_split(fwd, q, k, v, decay, T, kv_in=kv_in, **kw)
        assert rel(o2, o) < TOL and rel(kvo2, kvo) < TOL
        for a, b in zip(oracle.bwd_split(bwd, q, k, v, do, decay, T, kv_ins, dkv_out=g, **kw), grads):
            assert rel(a, b) < TOL


def test_rows_variants_match_full(oracle):
    q, k, v, do, decay, kv_in, g = rand_case(10)
    rows = np.array([[0, 0, 0], [1, 2, 23], [0, 1, 11], [1, 0, 5]])
    o, _ = oracle.fwd_brute(q, k, v, decay, kv_in)
    dq, dk, dv, _ = oracle.bwd_brute(q, k, v, do, decay, kv_in, g)
    orow = oracle.fwd_brute_rows(q, k, v, decay, rows, kv_in)
    dqr, dkr, dvr = oracle.bwd_brute_rows(q, k, v, do, decay, rows, kv_in, g)
    for i, (b, h, s) in enumerate(rows):
        assert np.array_equal(orow[i], o[b, h, s])
        assert np.array_equal(dqr[i], dq[b, h, s])
        assert np.array_equal(dkr[i], dk[b, h, s])
        assert np.array_equal(dvr[i], dv[b, h, s])


def test_long_block_small_lambda_no_overflow(oracle):
    """Powers are taken directly (never lam^i * lam^-j): lam = 0.5 over 2048 tokens stays finite."""
    rng = np.random.default_rng(11)
    N, D = 2048, 2
    q, k, v = (rng.standard_normal((1, 1, N, D)) for _ in range(3))
    o, kvo = oracle.fwd_chunked(q, k, v, np.array([0.5]), 1024)
    o2, kvo2 = oracle.fwd_recurrent(q, k, v, np.array([0.5]))
    assert np.all(np.isfinite(o)) and rel(o, o2) < 1e-10 and rel(kvo, kvo2) < 1e-10
