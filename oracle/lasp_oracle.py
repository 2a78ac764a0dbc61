"""ctypes front end of the fp64 CPU oracle (oracle/lasp_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
cpu_baseline leg of bench.py. It imports nothing from the GPU package.

All functions take numpy arrays of any float dtype (converted exactly to
float64) in the layouts of the C file: q/k/v/dout [B,H,N,D], states [B,H,D,D],
decay [H]; they return float64 arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lasp_oracle.c")
_LIB = os.path.join(_HERE, "liblasp_oracle.so")

_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_longlong)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over heads/rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _d(x):
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


def _p(x):
    return x.ctypes.data_as(_dp) if x is not None else None


def _shape(q):
    if q.ndim != 4:
        raise ValueError("expected [B,H,N,D]")
    return tuple(int(x) for x in q.shape)


def _opt_state(x, B, H, D):
    if x is None:
        return None
    x = _d(x)
    if x.shape != (B, H, D, D):
        raise ValueError("state must be [B,H,D,D]")
    return x


def num_threads() -> int:
    return int(_load().lasp_oracle_num_threads())


def set_num_threads(n: int) -> None:
    """Threads the OpenMP loops use from now on (for timing the oracle on one core; the arithmetic is untouched)."""
    _load()
    ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))


def _fwd(name, q, k, v, decay, kv_in, chunk=None):
    lib = _load()
    q, k, v, decay = _d(q), _d(k), _d(v), _d(decay)
    B, H, N, D = _shape(q)
    assert k.shape == q.shape and v.shape == q.shape and decay.shape == (H,)
    kv_in = _opt_state(kv_in, B, H, D)
    out = np.empty_like(q)
    kv_out = np.empty((B, H, D, D), dtype=np.float64)
    fn = getattr(lib, name)
    args = [ctypes.c_int(B), ctypes.c_int(H), ctypes.c_longlong(N), ctypes.c_int(D)]
    if chunk is not None:
        args.append(ctypes.c_int(int(chunk)))
    args += [_p(q), _p(k), _p(v), _p(kv_in), _p(decay), _p(out), _p(kv_out)]
    rc = fn(*args)
    if rc != 0:
        raise RuntimeError(f"{name} failed with code {rc}")
    return out, kv_out


def _bwd(name, q, k, v, dout, decay, kv_in, dkv_out, chunk=None):
    lib = _load()
    q, k, v, dout, decay = _d(q), _d(k), _d(v), _d(dout), _d(decay)
    B, H, N, D = _shape(q)
    assert k.shape == q.shape and v.shape == q.shape and dout.shape == q.shape and decay.shape == (H,)
    kv_in = _opt_state(kv_in, B, H, D)
    dkv_out = _opt_state(dkv_out, B, H, D)
    dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
    dkv_in = np.empty((B, H, D, D), dtype=np.float64)
    fn = getattr(lib, name)
    args = [ctypes.c_int(B), ctypes.c_int(H), ctypes.c_longlong(N), ctypes.c_int(D)]
    if chunk is not None:
        args.append(ctypes.c_int(int(chunk)))
    args += [_p(q), _p(k), _p(v), _p(dout), _p(kv_in), _p(dkv_out), _p(decay), _p(dq), _p(dk), _p(dv), _p(dkv_in)]
    rc = fn(*args)
    if rc != 0:
        raise RuntimeError(f"{name} failed with code {rc}")
    return dq, dk, dv, dkv_in


def fwd_brute(q, k, v, decay, kv_in=None):
    """Definition: o_s = sum_{i<=s} lam^(s-i) (q_s.k_i) v_i + lam^s K0^T q_s; returns (out, kv_out)."""
    return _fwd("lasp_oracle_fwd_brute", q, k, v, decay, kv_in)


def fwd_recurrent(q, k, v, decay, kv_in=None):
    return _fwd("lasp_oracle_fwd_recurrent", q, k, v, decay, kv_in)


def fwd_chunked(q, k, v, decay, chunk, kv_in=None):
    return _fwd("lasp_oracle_fwd_chunked", q, k, v, decay, kv_in, chunk=chunk)


def bwd_brute(q, k, v, dout, decay, kv_in=None, dkv_out=None):
    """Returns (dq, dk, dv, dkv_in) for the loss sum(out*dout) + sum(kv_out*dkv_out)."""
    return _bwd("lasp_oracle_bwd_brute", q, k, v, dout, decay, kv_in, dkv_out)


def bwd_recurrent(q, k, v, dout, decay, kv_in=None, dkv_out=None):
    return _bwd("lasp_oracle_bwd_recurrent", q, k, v, dout, decay, kv_in, dkv_out)


def bwd_chunked(q, k, v, dout, decay, chunk, kv_in=None, dkv_out=None):
    return _bwd("lasp_oracle_bwd_chunked", q, k, v, dout, decay, kv_in, dkv_out, chunk=chunk)


def _rows(rows, B, H, N):
    rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
    if rows.ndim != 2 or rows.shape[1] != 3:
        raise ValueError("rows must be [n,3] of (b,h,s0)")
    return rows


def fwd_brute_rows(q, k, v, decay, rows, kv_in=None):
    """Brute-force outputs for selected (b, h, s0) rows only; returns [n, D]."""
    lib = _load()
    q, k, v, decay = _d(q), _d(k), _d(v), _d(decay)
    B, H, N, D = _shape(q)
    kv_in = _opt_state(kv_in, B, H, D)
    rows = _rows(rows, B, H, N)
    out = np.empty((rows.shape[0], D), dtype=np.float64)
    rc = lib.lasp_oracle_fwd_brute_rows(
        ctypes.c_int(B), ctypes.c_int(H), ctypes.c_longlong(N), ctypes.c_int(D), _p(q), _p(k), _p(v),
        _p(kv_in), _p(decay), ctypes.c_longlong(rows.shape[0]), rows.ctypes.data_as(_ip), _p(out))
    if rc != 0:
        raise RuntimeError(f"fwd_brute_rows failed with code {rc}")
    return out


def bwd_brute_rows(q, k, v, dout, decay, rows, kv_in=None, dkv_out=None):
    """Brute-force (dq, dk, dv) for selected (b, h, s0) rows only; each [n, D]."""
    lib = _load()
    q, k, v, dout, decay = _d(q), _d(k), _d(v), _d(dout), _d(decay)
    B, H, N, D = _shape(q)
    kv_in = _opt_state(kv_in, B, H, D)
    dkv_out = _opt_state(dkv_out, B, H, D)
    rows = _rows(rows, B, H, N)
    n = rows.shape[0]
    dq, dk, dv = (np.empty((n, D), dtype=np.float64) for _ in range(3))
    rc = lib.lasp_oracle_bwd_brute_rows(
        ctypes.c_int(B), ctypes.c_int(H), ctypes.c_longlong(N), ctypes.c_int(D), _p(q), _p(k), _p(v),
        _p(dout), _p(kv_in), _p(dkv_out), _p(decay), ctypes.c_longlong(n), rows.ctypes.data_as(_ip),
        _p(dq), _p(dk), _p(dv))
    if rc != 0:
        raise RuntimeError(f"bwd_brute_rows failed with code {rc}")
    return dq, dk, dv


def fwd_split(fwd_fn, q, k, v, decay, T, kv_in=None, **kw):
    """T sub-sequences processed in order, kv_out of one handed to the next as
    kv_in (the ring of Alg. 2 folded into a loop). Returns (out, kv_out, kv_ins)
    where kv_ins[t] is the state sub-sequence t received (kept for backward)."""
    q, k, v = _d(q), _d(k), _d(v)
    N = q.shape[2]
    assert N % T == 0
    n = N // T
    outs, kv_ins = [], []
    state = kv_in
    for t in range(T):
        sl = slice(t * n, (t + 1) * n)
        kv_ins.append(state)
        o, state = fwd_fn(q[:, :, sl], k[:, :, sl], v[:, :, sl], decay, kv_in=state, **kw)
        outs.append(o)
    return np.concatenate(outs, axis=2), state, kv_ins


def bwd_split(bwd_fn, q, k, v, dout, decay, T, kv_ins, dkv_out=None, **kw):
    """Reverse loop of Alg. 3: sub-sequence t receives dkv from t+1 and hands
    its dkv_in to t-1. Returns (dq, dk, dv, dkv_in)."""
    q, k, v, dout = _d(q), _d(k), _d(v), _d(dout)
    N = q.shape[2]
    n = N // T
    dqs, dks, dvs = [None] * T, [None] * T, [None] * T
    g = dkv_out
    for t in reversed(range(T)):
        sl = slice(t * n, (t + 1) * n)
        dqs[t], dks[t], dvs[t], g = bwd_fn(q[:, :, sl], k[:, :, sl], v[:, :, sl], dout[:, :, sl], decay,
                                           kv_in=kv_ins[t], dkv_out=g, **kw)
    return np.concatenate(dqs, axis=2), np.concatenate(dks, axis=2), np.concatenate(dvs, axis=2), g


# ---------------------------------------------------------------------------
# Per-token decay g_s (general recurrent form of App. A.4 with a scalar
# oscillation state): kv_s = g_s kv_{s-1} + k_s v_s^T. log_g is [B,H,N], the
# natural logarithm of g. Backward returns (dq, dk, dv, dlog_g, dkv_in).
# ---------------------------------------------------------------------------
def _lg(log_g, B, H, N):
    log_g = _d(log_g)
    if log_g.shape != (B, H, N):
        raise ValueError("log_g must be [B,H,N]")
    return log_g


def _gated_fwd(name, q, k, v, log_g, kv_in, chunk=None):
    lib = _load()
    q, k, v = _d(q), _d(k), _d(v)
    B, H, N, D = _shape(q)
    log_g = _lg(log_g, B, H, N)
    kv_in = _opt_state(kv_in, B, H, D)
    out = np.empty_like(q)
    kv_out = np.empty((B, H, D, D), dtype=np.float64)
    args = [ctypes.c_int(B), ctypes.c_int(H), ctypes.c_longlong(N), ctypes.c_int(D)]
    if chunk is not None:
        args.append(ctypes.c_int(int(chunk)))
    args += [_p(q), _p(k), _p(v), _p(log_g), _p(kv_in), _p(out), _p(kv_out)]
    rc = getattr(lib, name)(*args)
    if rc != 0:
        raise RuntimeError(f"{name} failed with code {rc}")
    return out, kv_out


def _gated_bwd(name, q, k, v, dout, log_g, kv_in, dkv_out, chunk=None):
    lib = _load()
    q, k, v, dout = _d(q), _d(k), _d(v), _d(dout)
    B, H, N, D = _shape(q)
    log_g = _lg(log_g, B, H, N)
    kv_in = _opt_state(kv_in, B, H, D)
    dkv_out = _opt_state(dkv_out, B, H, D)
    dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
    dlg = np.empty((B, H, N), dtype=np.float64)
    dkv_in = np.empty((B, H, D, D), dtype=np.float64)
    args = [ctypes.c_int(B), ctypes.c_int(H), ctypes.c_longlong(N), ctypes.c_int(D)]
    if chunk is not None:
        args.append(ctypes.c_int(int(chunk)))
    args += [_p(q), _p(k), _p(v), _p(dout), _p(log_g), _p(kv_in), _p(dkv_out), _p(dq), _p(dk), _p(dv), _p(dlg),
             _p(dkv_in)]
    rc = getattr(lib, name)(*args)
    if rc != 0:
        raise RuntimeError(f"{name} failed with code {rc}")
    return dq, dk, dv, dlg, dkv_in


def gated_fwd_brute(q, k, v, log_g, kv_in=None):
    """Definition: o_s = sum_{i<=s} (prod_{l=i+1..s} g_l)(q_s.k_i) v_i + (prod_{l<=s} g_l) K0^T q_s."""
    return _gated_fwd("lasp_oracle_gated_fwd_brute", q, k, v, log_g, kv_in)


def gated_fwd_recurrent(q, k, v, log_g, kv_in=None):
    return _gated_fwd("lasp_oracle_gated_fwd_recurrent", q, k, v, log_g, kv_in)


def gated_fwd_chunked(q, k, v, log_g, chunk, kv_in=None):
    return _gated_fwd("lasp_oracle_gated_fwd_chunked", q, k, v, log_g, kv_in, chunk=chunk)


def gated_bwd_brute(q, k, v, dout, log_g, kv_in=None, dkv_out=None):
    return _gated_bwd("lasp_oracle_gated_bwd_brute", q, k, v, dout, log_g, kv_in, dkv_out)


def gated_bwd_recurrent(q, k, v, dout, log_g, kv_in=None, dkv_out=None):
    return _gated_bwd("lasp_oracle_gated_bwd_recurrent", q, k, v, dout, log_g, kv_in, dkv_out)


def gated_bwd_chunked(q, k, v, dout, log_g, chunk, kv_in=None, dkv_out=None):
    return _gated_bwd("lasp_oracle_gated_bwd_chunked", q, k, v, dout, log_g, kv_in, dkv_out, chunk=chunk)


def gated_fwd_brute_rows(q, k, v, log_g, rows, kv_in=None):
    lib = _load()
    q, k, v = _d(q), _d(k), _d(v)
    B, H, N, D = _shape(q)
    log_g = _lg(log_g, B, H, N)
    kv_in = _opt_state(kv_in, B, H, D)
    rows = _rows(rows, B, H, N)
    out = np.empty((rows.shape[0], D), dtype=np.float64)
    rc = lib.lasp_oracle_gated_fwd_brute_rows(
        ctypes.c_int(B), ctypes.c_int(H), ctypes.c_longlong(N), ctypes.c_int(D), _p(q), _p(k), _p(v),
        _p(log_g), _p(kv_in), ctypes.c_longlong(rows.shape[0]), rows.ctypes.data_as(_ip), _p(out))
    if rc != 0:
        raise RuntimeError(f"gated_fwd_brute_rows failed with code {rc}")
    return out


def gated_bwd_brute_rows(q, k, v, dout, log_g, rows, kv_in=None, dkv_out=None):
    lib = _load()
    q, k, v, dout = _d(q), _d(k), _d(v), _d(dout)
    B, H, N, D = _shape(q)
    log_g = _lg(log_g, B, H, N)
    kv_in = _opt_state(kv_in, B, H, D)
    dkv_out = _opt_state(dkv_out, B, H, D)
    rows = _rows(rows, B, H, N)
    n = rows.shape[0]
    dq, dk, dv = (np.empty((n, D), dtype=np.float64) for _ in range(3))
    rc = lib.lasp_oracle_gated_bwd_brute_rows(
        ctypes.c_int(B), ctypes.c_int(H), ctypes.c_longlong(N), ctypes.c_int(D), _p(q), _p(k), _p(v),
        _p(dout), _p(log_g), _p(kv_in), _p(dkv_out), ctypes.c_longlong(n), rows.ctypes.data_as(_ip),
        _p(dq), _p(dk), _p(dv))
    if rc != 0:
        raise RuntimeError(f"gated_bwd_brute_rows failed with code {rc}")
    return dq, dk, dv


def gated_fwd_split(fwd_fn, q, k, v, log_g, T, kv_in=None, **kw):
    """T sub-sequences in order, the state handed on; returns (out, kv_out, kv_ins, kv_outs)."""
    q, k, v, log_g = _d(q), _d(k), _d(v), _d(log_g)
    N = q.shape[2]
    assert N % T == 0
    n = N // T
    outs, kv_ins, kv_outs = [], [], []
    state = kv_in
    for t in range(T):
        sl = slice(t * n, (t + 1) * n)
        kv_ins.append(state)
        o, state = fwd_fn(q[:, :, sl], k[:, :, sl], v[:, :, sl], log_g[:, :, sl], kv_in=state, **kw)
        kv_outs.append(state)
        outs.append(o)
    return np.concatenate(outs, axis=2), state, kv_ins, kv_outs


def gated_bwd_split(bwd_fn, q, k, v, dout, log_g, T, kv_ins, dkv_out=None, **kw):
    """Reverse loop: sub-sequence t receives dkv from t+1; returns (dq, dk, dv, dlog_g, dkv_in)."""
    q, k, v, dout, log_g = _d(q), _d(k), _d(v), _d(dout), _d(log_g)
    N = q.shape[2]
    n = N // T
    dqs, dks, dvs, dls = [None] * T, [None] * T, [None] * T, [None] * T
    g = dkv_out
    for t in reversed(range(T)):
        sl = slice(t * n, (t + 1) * n)
        dqs[t], dks[t], dvs[t], dls[t], g = bwd_fn(q[:, :, sl], k[:, :, sl], v[:, :, sl], dout[:, :, sl],
                                                   log_g[:, :, sl], kv_in=kv_ins[t], dkv_out=g, **kw)
    cat = lambda xs: np.concatenate(xs, axis=2)
    return cat(dqs), cat(dks), cat(dvs), cat(dls), g


# ---------------------------------------------------------------------------
# Norm(.) of the normalised linear attention O = Norm((Q K^T (.) M) V) (Sec. 3.1, Eq. (2),
# linear-attention paragraph): read as the parameter-free root-mean-square
# normalisation of every output row over the head dimension,
#     y_s = o_s / sqrt(mean_c o_s[c]^2 + eps).
# It acts on one token at a time, so it composes with any form of the oracle
# above: forward = norm_fwd(fwd_*(...)), backward = bwd_*(..., dout = norm_bwd(...)).
# ---------------------------------------------------------------------------
def norm_fwd(o, eps):
    """Returns (y, rstd): y = o * rstd, rstd = (mean(o^2, last axis) + eps)^(-1/2), rstd shaped like o[..., 0]."""
    o = _d(o)
    rstd = 1.0 / np.sqrt(np.mean(o * o, axis=-1) + float(eps))
    return o * rstd[..., None], rstd


def norm_bwd(dy, y, rstd):
    """Gradient w.r.t. o of sum(y * dy), from the normalised output and rstd:
    do_s = rstd_s (dy_s - y_s mean_c(dy_s[c] y_s[c]))."""
    dy, y, rstd = _d(dy), _d(y), _d(rstd)
    m = np.mean(dy * y, axis=-1)
    return rstd[..., None] * (dy - y * m[..., None])


# ---------------------------------------------------------------------------
# Grouped key/value heads (multi-query / grouped-query attention, which the
# method is indifferent to, Sec. 1): kv_heads K/V heads serve H query heads,
# query heads h*G .. h*G+G-1 share K/V head h (G = H / kv_heads). By definition
# this is ordinary multi-head attention on K, V repeated G times along the head
# axis; the gradient of a shared head is the sum over the heads it serves.
# ---------------------------------------------------------------------------
def group_expand(x, G):
    """[B, kv_heads, N, D] -> [B, kv_heads * G, N, D], each K/V head repeated for its G query heads."""
    return np.repeat(_d(x), int(G), axis=1)


def group_reduce(dx, G):
    """Gradient of group_expand: [B, H, N, D] -> [B, H / G, N, D], summed over each group."""
    dx = _d(dx)
    B, H, N, D = dx.shape
    return dx.reshape(B, H // int(G), int(G), N, D).sum(axis=2)


# ---------------------------------------------------------------------------
# Bidirectional (unmasked) linear attention, Sec. 3.1: without the causal mask
# the attention is O = (Q K^T) V, which associativity turns into the
# right-product form O = Q (K^T V) of Eq. (3) (both without the Norm, which
# composes as above). No decay, no order among the tokens: the d x d state
# K^T V is a plain sum over every token of the sequence.
# `*_left` is the definition (N x N scores); `*_right` is Eq. (3).
# ---------------------------------------------------------------------------
def _t(x):
    return np.swapaxes(x, -1, -2)


def bidir_fwd_left(q, k, v):
    """O = (Q K^T) V per (batch, head): the definition, with the N x N score matrix."""
    q, k, v = _d(q), _d(k), _d(v)
    return np.matmul(np.matmul(q, _t(k)), v)


def bidir_state(x, y):
    """[B,H,N,D] x [B,H,N,D] -> [B,H,D,D]: sum over tokens of x_s y_s^T (K^T V of Eq. (3))."""
    return np.matmul(_t(_d(x)), _d(y))


def bidir_fwd_right(q, kv):
    """O = Q KV, Eq. (3), for a given state KV [B,H,D,D]."""
    return np.matmul(_d(q), _d(kv))


def bidir_bwd_left(q, k, v, dout):
    """Gradients of sum(O * dout) for O = (Q K^T) V, from the N x N matrices S = Q K^T and dS = dout V^T:
    dQ = dS K, dK = dS^T Q, dV = S^T dout."""
    q, k, v, dout = _d(q), _d(k), _d(v), _d(dout)
    s = np.matmul(q, _t(k))
    ds = np.matmul(dout, _t(v))
    return np.matmul(ds, k), np.matmul(_t(ds), q), np.matmul(_t(s), dout)


def bidir_fwd_rows(q, k, v, rows):
    """Sampled output rows from the definition: o_s = sum_i (q_s . k_i) v_i. rows: [n,3] of (b,h,s)."""
    q, k, v = _d(q), _d(k), _d(v)
    out = np.empty((len(rows), q.shape[-1]))
    for n, (b, h, s) in enumerate(np.asarray(rows, dtype=np.int64)):
        out[n] = (k[b, h] @ q[b, h, s]) @ v[b, h]
    return out


def bidir_bwd_rows(q, k, v, dout, rows):
    """Sampled gradient rows from the definition:
    dq_s = sum_i (do_s . v_i) k_i, dk_s = sum_i (do_i . v_s) q_i, dv_s = sum_i (q_i . k_s) do_i."""
    q, k, v, dout = _d(q), _d(k), _d(v), _d(dout)
    D = q.shape[-1]
    dq, dk, dv = (np.empty((len(rows), D)) for _ in range(3))
    for n, (b, h, s) in enumerate(np.asarray(rows, dtype=np.int64)):
        dq[n] = (v[b, h] @ dout[b, h, s]) @ k[b, h]
        dk[n] = (dout[b, h] @ v[b, h, s]) @ q[b, h]
        dv[n] = (q[b, h] @ k[b, h, s]) @ dout[b, h]
    return dq, dk, dv


# ---------------------------------------------------------------------------
# Key and value dimensions that differ (d_k for q, k; d_v for v, out): the
# state is [d_k][d_v] and nothing else changes in Alg. 2 / Alg. 3 or in the
# general recurrent form of App. A.4. Written out from the definition with the
# N x N weight matrix, per (batch, head), for small N:
#     W[s][i] = weight of token i in the state seen by token s (i <= s):
#               lambda^(s-i), or g_{i+1} ... g_s with a decay per token,
#     up[s]   = weight of kv_in at token s, after[i] = weight of token i in kv_out,
#     out     = (Q K^T (.) W) V + diag(up) Q kv_in
#     kv_out  = whole * kv_in + (diag(after) K)^T V
# and the gradients of L = sum(out * dout) + <kv_out, dkv_out>.
# ---------------------------------------------------------------------------
def _weights(N, lam=None, log_g=None):
    if log_g is None:
        cum = np.arange(1, N + 1, dtype=np.float64) * np.log(float(lam)) if lam > 0 else None
    else:
        cum = np.cumsum(np.asarray(log_g, dtype=np.float64))
    W = np.tril(np.exp(cum[:, None] - cum[None, :]))
    return W, np.exp(cum), np.exp(cum[-1] - cum), float(np.exp(cum[-1]))


def dims_fwd_brute(q, k, v, decay=None, kv_in=None, log_g=None):
    """q, k [B,H,N,dk]; v [B,H,N,dv]; decay [H] or log_g [B,H,N]; kv_in [B,H,dk,dv] or None -> (out, kv_out)."""
    q, k, v = _d(q), _d(k), _d(v)
    B, H, N, dk = q.shape
    dv = v.shape[-1]
    out, kv_out = np.empty((B, H, N, dv)), np.empty((B, H, dk, dv))
    for b in range(B):
        for h in range(H):
            W, up, after, whole = _weights(N, None if decay is None else float(decay[h]), None if log_g is None else log_g[b, h])
            s0 = np.zeros((dk, dv)) if kv_in is None else _d(kv_in)[b, h]
            out[b, h] = ((q[b, h] @ k[b, h].T) * W) @ v[b, h] + up[:, None] * (q[b, h] @ s0)
            kv_out[b, h] = whole * s0 + (after[:, None] * k[b, h]).T @ v[b, h]
    return out, kv_out


def dims_bwd_brute(q, k, v, dout, decay=None, kv_in=None, dkv_out=None, log_g=None):
    """-> (dq, dk, dv, dkv_in) for one lambda per head, (dq, dk, dv, dlog_g, dkv_in) with log_g."""
    q, k, v, dout = _d(q), _d(k), _d(v), _d(dout)
    B, H, N, dk = q.shape
    dv = v.shape[-1]
    dq, dkk, dvv = np.empty_like(q), np.empty_like(k), np.empty_like(v)
    dkv_in, dlg = np.empty((B, H, dk, dv)), np.empty((B, H, N))
    for b in range(B):
        for h in range(H):
            W, up, after, whole = _weights(N, None if decay is None else float(decay[h]), None if log_g is None else log_g[b, h])
            s0 = np.zeros((dk, dv)) if kv_in is None else _d(kv_in)[b, h]
            G = np.zeros((dk, dv)) if dkv_out is None else _d(dkv_out)[b, h]
            S = (q[b, h] @ k[b, h].T) * W
            dS = (dout[b, h] @ v[b, h].T) * W
            dq[b, h] = dS @ k[b, h] + up[:, None] * (dout[b, h] @ s0.T)
            dkk[b, h] = dS.T @ q[b, h] + after[:, None] * (v[b, h] @ G.T)
            dvv[b, h] = S.T @ dout[b, h] + after[:, None] * (k[b, h] @ G)
            dkv_in[b, h] = (up[:, None] * q[b, h]).T @ dout[b, h] + whole * G
            if log_g is not None:
                # d L / d log g_s: every weight whose product contains g_s, i.e. pairs (i < s <= t), the
                # kv_in term of tokens t >= s and the kv_out terms of tokens i < s and of kv_in
                P = (dout[b, h] @ v[b, h].T) * (q[b, h] @ k[b, h].T) * W          # contribution of pair (t, i)
                a = up * np.sum((q[b, h] @ s0) * dout[b, h], axis=1)              # kv_in seen by token t
                c = after * np.sum((k[b, h] @ G) * v[b, h], axis=1)               # token i seen by kv_out
                z = whole * float(np.sum(s0 * G))
                for s in range(N):
                    dlg[b, h, s] = P[s:, :s].sum() + a[s:].sum() + c[:s].sum() + z
    if log_g is None:
        return dq, dkk, dvv, dkv_in
    return dq, dkk, dvv, dlg, dkv_in
