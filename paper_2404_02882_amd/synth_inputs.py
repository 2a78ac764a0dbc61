"""Seeded synthetic inputs shared by the tests, the smoke check and bench.py.

This module holds no attention arithmetic: it only draws random tensors with
the shapes and value scales of the workloads, rounds them to the storage type
and lists the named configurations. Both the GPU path and the CPU oracle are
fed the values produced here; neither imports the other.

The tensors stand in for the post-projection Q, K, V of one TransNormerLLM
linear-attention layer (head dimension 128 for the 1B/7B shapes); the path's
cost depends only on the shapes and its numerics on the value scale, so no
dataset or trained weight is needed.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np


@dataclass(frozen=True)
class Config:
    name: str
    B: int
    H: int
    N: int          # whole sequence length
    D: int
    chunk: int
    dtype: str      # "f32" or "bf16"
    T: int = 1      # sub-sequences the sequence is processed in (state passed between them)
    seed: int = 0
    decay: str = "schedule"   # "schedule" or "one"
    fwd_only: bool = False
    k_outlier_frac: float = 0.0
    k_outlier_scale: float = 1.0
    token_decay: bool = False   # a decay g_s per token (log_g) instead of one lambda per head
    norm_eps: Optional[float] = None   # outputs are RMS-normalised per row (fused Norm); dout is then the gradient w.r.t. them
    bidirectional: bool = False   # unmasked attention O = Q (K^T V): no decay, no states handed over
    Dv: int = 0     # value dimension when it differs from the key dimension D (0 = D)


# The five workloads (shapes, decay and value recipe as stated for the build).
CONFIGS = {
    "c1": Config("c1", B=1, H=2, N=256, D=64, chunk=64, dtype="f32", seed=1001, decay="one", fwd_only=True),
    "c2": Config("c2", B=2, H=8, N=4096, D=64, chunk=64, dtype="bf16", T=4, seed=1002),
    "c3": Config("c3", B=1, H=16, N=32768, D=128, chunk=128, dtype="bf16", seed=1003),
    "c4": Config("c4", B=1, H=16, N=262144, D=128, chunk=128, dtype="bf16", T=8, seed=1004),
    "c5": Config("c5", B=4, H=32, N=16384, D=128, chunk=256, dtype="bf16", seed=1005,
                 k_outlier_frac=0.01, k_outlier_scale=8.0),
    # the same shapes as c2 / c3 with a decay per token
    "g2": Config("g2", B=2, H=8, N=4096, D=64, chunk=64, dtype="bf16", T=4, seed=1012, token_decay=True),
    "g3": Config("g3", B=1, H=16, N=32768, D=128, chunk=128, dtype="bf16", seed=1013, token_decay=True),
    # c3's shape with the normalised output
    "n3": Config("n3", B=1, H=16, N=32768, D=128, chunk=128, dtype="bf16", seed=1023, norm_eps=1e-5),
    # c2's / c3's shapes without the causal mask (bidirectional attention)
    "b2": Config("b2", B=2, H=8, N=4096, D=64, chunk=64, dtype="bf16", T=4, seed=1032, decay="one", bidirectional=True),
    "b3": Config("b3", B=1, H=16, N=32768, D=128, chunk=128, dtype="bf16", seed=1033, decay="one", bidirectional=True),
    # c3's shape with a key dimension of 64 and a value dimension of 128
    "m3": Config("m3", B=1, H=16, N=32768, D=64, chunk=128, dtype="bf16", seed=1043, Dv=128),
}


def decay_schedule(H: int) -> np.ndarray:
    """lambda_h = 1 - 2^-(5 + 8h/H), h = 0..H-1, evaluated in fp64 and rounded
    once to fp32 (H=8 gives 1 - 2^-(5+h))."""
    h = np.arange(H, dtype=np.float64)
    return (1.0 - np.exp2(-(5.0 + 8.0 * h / H))).astype(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize(x: np.ndarray, dtype: str) -> np.ndarray:
    """Value of x after storage in `dtype`, returned as fp32 (exactly representable)."""
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(bf16_bits(x))
    raise ValueError(dtype)


@dataclass
class Inputs:
    cfg: Config
    q: np.ndarray       # fp32 arrays holding values exactly representable in cfg.dtype
    k: np.ndarray
    v: np.ndarray
    dout: np.ndarray
    decay: np.ndarray   # fp32 [H]
    kv_in: Optional[np.ndarray] = None     # fp32 [B,H,D,D] or None (zeros)
    dkv_out: Optional[np.ndarray] = None
    log_g: Optional[np.ndarray] = None     # fp32 [B,H,N], natural log of the per-token decay (token_decay configs)


def token_log_decay(cfg: Config, N: int, seed: int, reset_frac: float = 0.001) -> np.ndarray:
    """log g for every head and token: log(lambda_h) * 2u, u ~ U(0,1), so that the mean decay of a head
    is that of the fixed schedule and single tokens range from no decay to twice the head's rate; a
    fraction `reset_frac` of the tokens gets log g = -8 (the gate almost closes, as data-dependent
    gates do at boundaries in the input). Own random stream: q, k, v do not depend on it."""
    rng = np.random.default_rng(seed + 7919)
    lam = decay_schedule(cfg.H).astype(np.float64)
    u = rng.random((cfg.B, cfg.H, N))
    lg = np.log(lam)[None, :, None] * 2.0 * u
    lg[rng.random((cfg.B, cfg.H, N)) < reset_frac] = -8.0
    return lg.astype(np.float32)


def make_inputs(cfg: Config, n_tokens: Optional[int] = None, with_states: bool = False,
                seed: Optional[int] = None) -> Inputs:
    """Q, K, V ~ N(0,1)/sqrt(D), dO ~ N(0,1), rounded to cfg.dtype. `n_tokens`
    overrides the sequence length (the draw for a prefix is not a prefix of the
    full draw; every length is its own seeded sample). With `with_states`,
    kv_in and dkv_out are N(0,1) fp32 states instead of zeros."""
    N = cfg.N if n_tokens is None else int(n_tokens)
    rng = np.random.default_rng(cfg.seed if seed is None else seed)
    shape = (cfg.B, cfg.H, N, cfg.D)
    dv = cfg.Dv or cfg.D
    vshape = (cfg.B, cfg.H, N, dv)
    scale = np.float32(cfg.D ** -0.5)
    q = rng.standard_normal(shape, dtype=np.float32) * scale
    k = rng.standard_normal(shape, dtype=np.float32) * scale
    v = rng.standard_normal(vshape, dtype=np.float32) * np.float32(dv ** -0.5)
    dout = rng.standard_normal(vshape, dtype=np.float32)
    if cfg.k_outlier_frac > 0.0:
        rows = rng.random((cfg.B, cfg.H, N)) < cfg.k_outlier_frac
        k[rows] *= np.float32(cfg.k_outlier_scale)
    decay = np.ones(cfg.H, dtype=np.float32) if cfg.decay == "one" else decay_schedule(cfg.H)
    kv_in = dkv_out = None
    if with_states:
        kv_in = rng.standard_normal((cfg.B, cfg.H, cfg.D, dv), dtype=np.float32)
        dkv_out = rng.standard_normal((cfg.B, cfg.H, cfg.D, dv), dtype=np.float32)
    log_g = token_log_decay(cfg, N, cfg.seed if seed is None else seed) if cfg.token_decay else None
    return Inputs(cfg, quantize(q, cfg.dtype), quantize(k, cfg.dtype), quantize(v, cfg.dtype),
                  quantize(dout, cfg.dtype), decay, kv_in, dkv_out, log_g)


def sample_rows(cfg: Config, N: int, n: int, seed: int) -> np.ndarray:
    """n random (b, h, s0) triples, always including the first and last token of
    the first and last head (boundary rows)."""
    rng = np.random.default_rng(seed)
    rows = np.stack([rng.integers(0, cfg.B, n), rng.integers(0, cfg.H, n), rng.integers(0, N, n)], axis=1)
    fixed = np.array([[0, 0, 0], [0, 0, N - 1], [cfg.B - 1, cfg.H - 1, 0], [cfg.B - 1, cfg.H - 1, N - 1]])
    rows[: min(n, 4)] = fixed[: min(n, 4)]
    return rows.astype(np.int64)
