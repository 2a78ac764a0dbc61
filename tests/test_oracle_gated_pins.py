"""Pins of the per-token-decay half of the fp64 oracle (CPU only).

The operation is the general recurrent form of App. A.4 with a scalar
oscillation state per head and token: kv_s = g_s kv_{s-1} + k_s v_s^T,
o_s = kv_s^T q_s. Each test ties a form of the oracle to something other than
itself: a hand-computed example, the fixed-decay oracle (itself pinned) at
constant g, textbook routines at g = 1, explicit products written in numpy,
finite differences of the forward pass, and agreement of the brute-force
definition with the recurrent and chunked forms and with T-way splitting.
"""
import json
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
TOL = 1e-11


def rel(a, b):
    return np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300)


def rand_case(seed, B=2, H=3, N=24, D=5, states=True, lo=0.5):
    rng = np.random.default_rng(seed)
    q, k, v, do = (rng.standard_normal((B, H, N, D)) for _ in range(4))
    log_g = np.log(rng.uniform(lo, 1.0, (B, H, N)))
    kv_in = rng.standard_normal((B, H, D, D)) if states else None
    g = rng.standard_normal((B, H, D, D)) if states else None
    return q, k, v, do, log_g, kv_in, g


def loss(o, kv_out, do, g):
    return float(np.sum(o * do) + (np.sum(kv_out * g) if g is not None else 0.0))


FORMS = ["brute", "recurrent", "chunk1", "chunk3", "chunkN"]


def run_form(oracle, form, q, k, v, do, log_g, kv_in, g):
    N = q.shape[2]
    if form == "brute":
        o, kvo = oracle.gated_fwd_brute(q, k, v, log_g, kv_in)
        grads = oracle.gated_bwd_brute(q, k, v, do, log_g, kv_in, g)
    elif form == "recurrent":
        o, kvo = oracle.gated_fwd_recurrent(q, k, v, log_g, kv_in)
        grads = oracle.gated_bwd_recurrent(q, k, v, do, log_g, kv_in, g)
    else:
        C = {"chunk1": 1, "chunk3": 3, "chunkN": N}[form]
        if N % C:
            C = 1
        o, kvo = oracle.gated_fwd_chunked(q, k, v, log_g, C, kv_in)
        grads = oracle.gated_bwd_chunked(q, k, v, do, log_g, C, kv_in, g)
    return (o, kvo) + tuple(grads)


NAMES = ("out", "kv_out", "dq", "dk", "dv", "dlog_g", "dkv_in")


# ---------------------------------------------------------------- hand example
@pytest.mark.parametrize("form", ["brute", "recurrent", "chunk1", "chunkN"])
def test_hand_example(oracle, form):
    with open(os.path.join(HERE, "golden", "hand_example_token_decay.json")) as f:
        ex = json.load(f)
    a = lambda x: np.array(x, dtype=np.float64)[None, None]
    got = run_form(oracle, form, a(ex["q"]), a(ex["k"]), a(ex["v"]), a(ex["dout"]), np.log(a(ex["g"])),
                   a(ex["kv_in"]), a(ex["dkv_out"]))
    for x, key in zip(got, NAMES):
        np.testing.assert_allclose(x[0, 0], np.array(ex[key], dtype=np.float64), rtol=0, atol=1e-13, err_msg=key)


# ---------------------------------------------------------------- reduction to the fixed decay
@pytest.mark.parametrize("form", FORMS)
def test_constant_g_equals_fixed_decay(oracle, form):
    """g_s = lambda_h for every token is the TNL/RetNet row of Table 6: same results as the fixed-decay
    oracle, and the sum of dlog_g over tokens is lambda dL/dlambda of that oracle (central difference)."""
    q, k, v, do, _, kv_in, g = rand_case(11, N=12)
    B, H, N, _ = q.shape
    lam = np.array([0.7, 0.9, 1.0])
    log_g = np.broadcast_to(np.log(lam)[None, :, None], (B, H, N)).copy()
    got = run_form(oracle, form, q, k, v, do, log_g, kv_in, g)
    o, kvo = oracle.fwd_brute(q, k, v, lam, kv_in)
    dq, dk, dv, gin = oracle.bwd_brute(q, k, v, do, lam, kv_in, g)
    for x, ref in zip(got, (o, kvo, dq, dk, dv, None, gin)):
        if ref is not None:
            assert rel(x, ref) < TOL
    dlg = got[5]
    h = 1e-6
    for hh in range(H):
        lp, lm = lam.copy(), lam.copy()
        lp[hh] *= np.exp(h)
        lm[hh] *= np.exp(-h)
        Lp = loss(*oracle.fwd_brute(q, k, v, lp, kv_in), do, g)
        Lm = loss(*oracle.fwd_brute(q, k, v, lm, kv_in), do, g)
        # only head hh changes between Lp and Lm
        np.testing.assert_allclose(dlg[:, hh].sum(), (Lp - Lm) / (2 * h), rtol=1e-7)


def test_g_one_is_textbook_linear_attention(oracle):
    q, k, v, do, _, _, _ = rand_case(12, B=1, H=2, N=16, D=4, states=False)
    log_g = np.zeros((1, 2, 16))
    o, kvo = oracle.gated_fwd_brute(q, k, v, log_g)
    dq, dk, dv, dlg, gin = oracle.gated_bwd_brute(q, k, v, do, log_g)
    for hh in range(2):
        Q, K, V, dO = q[0, hh], k[0, hh], v[0, hh], do[0, hh]
        assert rel(o[0, hh], np.tril(Q @ K.T) @ V) < TOL
        assert rel(kvo[0, hh], K.T @ V) < TOL
        assert rel(dq[0, hh], np.tril(dO @ V.T) @ K) < TOL
        assert rel(dk[0, hh], np.tril(dO @ V.T).T @ Q) < TOL
        assert rel(dv[0, hh], np.tril(Q @ K.T).T @ dO) < TOL
        assert rel(gin[0, hh], Q.T @ dO) < TOL


# ---------------------------------------------------------------- explicit products
@pytest.mark.parametrize("form", FORMS)
def test_weights_are_products_of_g_after_the_source(oracle, form):
    """One key/value impulse at token i: o_s = (g_{i+1} ... g_s)(q_s.k_i) v_i for s >= i, 0 before;
    the incoming state is weighted by g_1 ... g_s (g of the receiving token included)."""
    rng = np.random.default_rng(13)
    N, D, i0 = 9, 3, 3  # impulse at 0-based token 3
    q = rng.standard_normal((1, 1, N, D))
    k = np.zeros((1, 1, N, D))
    v = np.zeros((1, 1, N, D))
    k[0, 0, i0], v[0, 0, i0] = rng.standard_normal(D), rng.standard_normal(D)
    gs = rng.uniform(0.3, 0.95, N)
    log_g = np.log(gs)[None, None]
    K0 = rng.standard_normal((1, 1, D, D))
    do = rng.standard_normal((1, 1, N, D))
    o = run_form(oracle, form, q, k, v, do, log_g, K0, None)[0]
    for s in range(N):
        ref = np.prod(gs[: s + 1]) * (K0[0, 0].T @ q[0, 0, s])
        if s >= i0:
            ref = ref + np.prod(gs[i0 + 1: s + 1]) * (q[0, 0, s] @ k[0, 0, i0]) * v[0, 0, i0]
        np.testing.assert_allclose(o[0, 0, s], ref, rtol=1e-12, atol=1e-14)


def test_kv_out_and_dkv_in_explicit(oracle):
    q, k, v, do, log_g, kv_in, g = rand_case(14, B=1, H=1, N=7, D=3)
    gs = np.exp(log_g[0, 0])
    N = 7
    kvo = oracle.gated_fwd_brute(q, k, v, log_g, kv_in)[1]
    ref = np.prod(gs) * kv_in[0, 0]
    for i in range(N):
        ref = ref + np.prod(gs[i + 1:]) * np.outer(k[0, 0, i], v[0, 0, i])
    assert rel(kvo[0, 0], ref) < TOL
    gin = oracle.gated_bwd_brute(q, k, v, do, log_g, kv_in, g)[4]
    ref = np.prod(gs) * g[0, 0]
    for s in range(N):
        ref = ref + np.prod(gs[: s + 1]) * np.outer(q[0, 0, s], do[0, 0, s])
    assert rel(gin[0, 0], ref) < TOL


# ---------------------------------------------------------------- finite differences
@pytest.mark.parametrize("form", ["brute", "recurrent", "chunk3"])
@pytest.mark.parametrize("states", [True, False])
def test_gradients_by_finite_differences(oracle, form, states):
    """dq, dk, dv, dkv_in exactly (the loss is linear in each of q, k, v, kv_in taken alone);
    dlog_g by central differences of the brute-force forward pass."""
    q, k, v, do, log_g, kv_in, g = rand_case(15, B=1, H=2, N=9, D=3, states=states)
    got = run_form(oracle, form, q, k, v, do, log_g, kv_in, g)
    dq, dk, dv, dlg, gin = got[2:]
    L = lambda q_, k_, v_, lg_, s_: loss(*oracle.gated_fwd_brute(q_, k_, v_, lg_, s_), do, g)
    L0 = L(q, k, v, log_g, kv_in)
    rng = np.random.default_rng(16)
    for _ in range(12):
        idx = (0, rng.integers(2), rng.integers(9), rng.integers(3))
        for which, grad in (("q", dq), ("k", dk), ("v", dv)):
            args = {"q": q.copy(), "k": k.copy(), "v": v.copy()}
            args[which][idx] += 1.0
            np.testing.assert_allclose(L(args["q"], args["k"], args["v"], log_g, kv_in) - L0, grad[idx], rtol=1e-9,
                                       atol=1e-9)
    if states:
        for _ in range(6):
            idx = (0, rng.integers(2), rng.integers(3), rng.integers(3))
            s2 = kv_in.copy()
            s2[idx] += 1.0
            np.testing.assert_allclose(L(q, k, v, log_g, s2) - L0, gin[idx], rtol=1e-9, atol=1e-9)
    h = 1e-5
    for hh in range(2):
        for s in range(9):
            lp, lm = log_g.copy(), log_g.copy()
            lp[0, hh, s] += h
            lm[0, hh, s] -= h
            fd = (L(q, k, v, lp, kv_in) - L(q, k, v, lm, kv_in)) / (2 * h)
            np.testing.assert_allclose(dlg[0, hh, s], fd, rtol=2e-7, atol=1e-8)


# ---------------------------------------------------------------- agreement of the forms
@pytest.mark.parametrize("form", ["recurrent", "chunk1", "chunk2", "chunk3", "chunk8", "chunkN"])
@pytest.mark.parametrize("states", [True, False])
def test_forms_agree_with_brute_force(oracle, form, states):
    q, k, v, do, log_g, kv_in, g = rand_case(17, N=24, states=states, lo=0.2)
    ref = run_form(oracle, "brute", q, k, v, do, log_g, kv_in, g)
    if form.startswith("chunk") and form not in ("chunk1", "chunk3", "chunkN"):
        C = int(form[5:])
        got = oracle.gated_fwd_chunked(q, k, v, log_g, C, kv_in) + oracle.gated_bwd_chunked(q, k, v, do, log_g, C, kv_in, g)
    else:
        got = run_form(oracle, form, q, k, v, do, log_g, kv_in, g)
    for x, r, name in zip(got, ref, NAMES):
        assert rel(x, r) < 1e-10, name


def test_checkpointed_recurrence_across_block_boundaries(oracle):
    """N larger than, and not a multiple of, the checkpoint spacing of the recurrent backward."""
    q, k, v, do, log_g, kv_in, g = rand_case(18, B=1, H=1, N=150, D=3)
    ref = oracle.gated_bwd_brute(q, k, v, do, log_g, kv_in, g)
    got = oracle.gated_bwd_recurrent(q, k, v, do, log_g, kv_in, g)
    for x, r in zip(got, ref):
        assert rel(x, r) < 1e-10


@pytest.mark.parametrize("T", [2, 4])
def test_split_with_state_passing(oracle, T):
    """T sub-sequences chained through kv / dkv give the unsplit result, dlog_g included
    (its boundary term <dkv_out, kv_out> is what links the pieces)."""
    q, k, v, do, log_g, kv_in, g = rand_case(19, N=24)
    ref = run_form(oracle, "brute", q, k, v, do, log_g, kv_in, g)
    o, kvo, kv_ins, _ = oracle.gated_fwd_split(oracle.gated_fwd_brute, q, k, v, log_g, T, kv_in=kv_in)
    grads = oracle.gated_bwd_split(oracle.gated_bwd_brute, q, k, v, do, log_g, T, kv_ins, dkv_out=g)
    for x, r, name in zip((o, kvo) + tuple(grads), ref, NAMES):
        assert rel(x, r) < 1e-10, name


def test_strong_decay_resets_the_state(oracle):
    """g_s = e^-700 at one token cuts the sequence there (no overflow, no NaN): outputs from that
    token on equal a fresh run over the tail alone."""
    q, k, v, do, log_g, kv_in, g = rand_case(20, B=1, H=1, N=16, D=3)
    log_g[0, 0, 8] = -700.0
    for form in ("brute", "recurrent", "chunk1", "chunkN"):
        got = run_form(oracle, form, q, k, v, do, log_g, kv_in, None)
        assert all(np.all(np.isfinite(x)) for x in got)
        tail = oracle.gated_fwd_brute(q[:, :, 8:], k[:, :, 8:], v[:, :, 8:], log_g[:, :, 8:])
        assert rel(got[0][:, :, 8:], tail[0]) < 1e-10
        assert rel(got[1], tail[1]) < 1e-10


def test_sampled_rows_match_full(oracle):
    q, k, v, do, log_g, kv_in, g = rand_case(21, N=20)
    rows = np.array([[0, 0, 0], [1, 2, 19], [0, 1, 7], [1, 0, 12]])
    o = oracle.gated_fwd_brute(q, k, v, log_g, kv_in)[0]
    dq, dk, dv, _, _ = oracle.gated_bwd_brute(q, k, v, do, log_g, kv_in, g)
    orows = oracle.gated_fwd_brute_rows(q, k, v, log_g, rows, kv_in)
    dqr, dkr, dvr = oracle.gated_bwd_brute_rows(q, k, v, do, log_g, rows, kv_in, g)
    b, h, s = rows[:, 0], rows[:, 1], rows[:, 2]
    for full, part in ((o, orows), (dq, dqr), (dk, dkr), (dv, dvr)):
        assert np.array_equal(full[b, h, s], part)
