"""GPU parity of the normalised-output entry points (lasp_fwd_norm / lasp_bwd_norm, through the C-ABI)
against the fp64 oracle: y = Norm(o) with Norm the RMS normalisation of a row, gradients of
sum(y * dy) + sum(kv_out * dkv_out). Tolerances: 1e-4 float, 2e-2 bfloat16 (max-norm and Frobenius)."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
EPS = 1e-5


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "needs a GPU"
    from paper_2404_02882_amd import harness, lasp, synth_inputs
    return harness, lasp, synth_inputs


def oracle_all(oracle, inp, eps, heads=None, chunk=None):
    sel = (lambda x: x) if heads is None else (lambda x: None if x is None else np.ascontiguousarray(x[:, heads]))
    q, k, v, dy = sel(inp.q), sel(inp.k), sel(inp.v), sel(inp.dout)
    decay = inp.decay if heads is None else inp.decay[heads]
    kv_in, g = sel(inp.kv_in), sel(inp.dkv_out)
    if chunk is None:
        o, kvo = oracle.fwd_brute(q, k, v, decay, kv_in)
    else:
        o, kvo = oracle.fwd_chunked(q, k, v, decay, chunk, kv_in)
    y, rstd = oracle.norm_fwd(o, eps)
    do = oracle.norm_bwd(dy, y, rstd)
    if chunk is None:
        dq, dk, dv, gin = oracle.bwd_brute(q, k, v, do, decay, kv_in, g)
    else:
        dq, dk, dv, gin = oracle.bwd_chunked(q, k, v, do, decay, chunk, kv_in, g)
    return dict(out=y, rstd=rstd, kv_out=kvo, dq=dq, dk=dk, dv=dv, dkv_in=gin)


def compare(harness, got, ref, tol, label, heads=None):
    for name, r in ref.items():
        x = got[name] if heads is None else got[name][:, heads]
        emax, efro = harness.rel_errors(x, r)
        say(f"  {label} {name:7s} max-rel {emax:.3e} fro-rel {efro:.3e}")
        assert np.isfinite(emax) and emax <= tol and efro <= tol, (label, name, emax, efro)


SMALL = [
    # dtype, D, chunk, tiles, segments, states
    ("f32", 64, 64, 4, 0, False),
    ("f32", 64, 64, 5, 2, True),
    ("f32", 128, 128, 3, 3, True),
    ("bf16", 64, 64, 5, 2, True),
    ("bf16", 64, 128, 3, 0, True),
    ("bf16", 128, 64, 5, 3, True),
    ("bf16", 128, 128, 4, 2, True),
    ("bf16", 128, 128, 1, 1, False),
]


@pytest.mark.parametrize("dtype,D,chunk,nchunks,segments,states", SMALL)
def test_small_against_brute_force(gpu, oracle, dtype, D, chunk, nchunks, segments, states):
    harness, lasp, si = gpu
    N = chunk * nchunks
    cfg = si.Config("nsmall", B=2, H=3, N=N, D=D, chunk=chunk, dtype=dtype, seed=500 + D + chunk + nchunks)
    say(f"case norm dtype={dtype} D={D} chunk={chunk} N={N} segments={segments} states={states}")
    inp = si.make_inputs(cfg, with_states=states)
    inp.decay = np.array([0.9, 0.97, 1.0 - 2.0 ** -7], dtype=np.float32)
    got = harness.run_gpu(inp, segments=segments, norm_eps=EPS)
    compare(harness, got, oracle_all(oracle, inp, EPS), TOL[dtype], "nsmall")


def test_split_pairs_and_eps(gpu, oracle):
    """T = 3 chained calls on an even tile count (pair cache), a large eps, and a zero output row
    (q = 0 for one token: y = 0, rstd = eps^-1/2, finite gradients)."""
    harness, lasp, si = gpu
    cfg = si.Config("nsplit", B=1, H=2, N=64 * 12, D=128, chunk=64, dtype="bf16", seed=61)
    inp = si.make_inputs(cfg, with_states=False)
    inp.q[0, 1, 100] = 0.0
    for eps in (EPS, 0.5):
        got = harness.run_gpu(inp, T=3, norm_eps=eps)
        assert all(np.all(np.isfinite(x)) for x in got.values())
        compare(harness, got, oracle_all(oracle, inp, eps), TOL["bf16"], f"nsplit/eps{eps}")


def test_c3_shape_full_size(gpu, oracle):
    """c3's shape: full tensors against the chunked oracle on every head."""
    harness, lasp, si = gpu
    cfg = si.CONFIGS["c3"]
    heads = None   # every head
    inp = si.make_inputs(cfg)
    say("case norm c3: gpu run")
    got = harness.run_gpu(inp, norm_eps=EPS)
    say("case norm c3: chunked oracle on all heads")
    ref = oracle_all(oracle, inp, EPS, heads=heads, chunk=cfg.chunk)
    compare(harness, got, ref, TOL["bf16"], "nc3", heads=heads)


@pytest.mark.parametrize("dtype,D,N,segments", [("f32", 64, 32 * 6, 2), ("bf16", 128, 64 * 8, 0), ("bf16", 64, 64 * 5, 3)])
def test_token_decay_with_norm(gpu, oracle, dtype, D, N, segments):
    """Per-token decay and the fused Norm together (lasp_gated_fwd_norm / lasp_gated_bwd_norm), T = 2 where
    the length allows: all gradients including dlog_g against the composed oracle."""
    harness, lasp, si = gpu
    cfg = si.Config("gnorm", B=2, H=3, N=N, D=D, chunk=64, dtype=dtype, seed=900 + N, token_decay=True)
    say(f"case gated+norm dtype={dtype} D={D} N={N} segments={segments}")
    inp = si.make_inputs(cfg, with_states=True)
    rng = np.random.default_rng(cfg.seed)
    inp.log_g = np.log(rng.uniform(0.8, 1.0, (2, 3, N))).astype(np.float32)
    T = 2 if (N // 2) % 64 == 0 else 1
    got = harness.run_gpu(inp, T=T, segments=segments, norm_eps=EPS)
    o, kvo = oracle.gated_fwd_brute(inp.q, inp.k, inp.v, inp.log_g, inp.kv_in)
    y, rstd = oracle.norm_fwd(o, EPS)
    do = oracle.norm_bwd(inp.dout, y, rstd)
    dq, dk, dv, dlg, gin = oracle.gated_bwd_brute(inp.q, inp.k, inp.v, do, inp.log_g, inp.kv_in, inp.dkv_out)
    ref = dict(out=y, rstd=rstd, kv_out=kvo, dq=dq, dk=dk, dv=dv, dlog_g=dlg, dkv_in=gin)
    compare(harness, got, ref, TOL[dtype], f"gnorm/{dtype}")


@pytest.mark.parametrize("dtype,D,N,T,segments,token", [
    ("f32", 64, 200, 1, 0, False), ("f32", 128, 97, 1, 2, True),
    ("bf16", 128, 1000, 1, 0, False),      # 16 tiles (pair kernel), the last one short
    ("bf16", 64, 450, 1, 3, False),        # 8 tiles
    ("bf16", 128, 421, 1, 0, False),       # 7 tiles (odd count)
    ("bf16", 128, 700, 1, 4, True), ("bf16", 64, 1, 1, 0, False),
])
def test_norm_with_a_short_last_tile(gpu, oracle, dtype, D, N, T, segments, token):
    """Sub-sequence lengths that are not a multiple of the tile, with the fused Norm (one lambda per head is
    routed through the per-token-decay kernels; rows past the end are neither read nor written)."""
    harness, lasp, si = gpu
    cfg = si.Config("nragged", B=2, H=3, N=N, D=D, chunk=64, dtype=dtype, seed=950 + N, token_decay=token)
    say(f"case norm ragged dtype={dtype} D={D} N={N} segments={segments} token={token}")
    inp = si.make_inputs(cfg, with_states=True)
    if token:
        inp.log_g = np.log(np.random.default_rng(cfg.seed).uniform(0.8, 1.0, (2, 3, N))).astype(np.float32)
        got = harness.run_gpu(inp, T=T, segments=segments, norm_eps=EPS)
        o, kvo = oracle.gated_fwd_brute(inp.q, inp.k, inp.v, inp.log_g, inp.kv_in)
        y, rstd = oracle.norm_fwd(o, EPS)
        do = oracle.norm_bwd(inp.dout, y, rstd)
        dq, dk, dv, dlg, gin = oracle.gated_bwd_brute(inp.q, inp.k, inp.v, do, inp.log_g, inp.kv_in, inp.dkv_out)
        ref = dict(out=y, rstd=rstd, kv_out=kvo, dq=dq, dk=dk, dv=dv, dlog_g=dlg, dkv_in=gin)
    else:
        inp.decay = np.array([0.9, 0.97, 1.0], dtype=np.float32)
        got = harness.run_gpu(inp, T=T, segments=segments, norm_eps=EPS)
        ref = oracle_all(oracle, inp, EPS)
    compare(harness, got, ref, TOL[dtype], f"nragged/{dtype}")
