"""GPU parity for key and value dimensions that differ (lasp_shape.Dv; q, k are [..,D], v, out are
[..,Dv], states [D][Dv]) against the fp64 oracle written for such dimensions, through the C-ABI.
Tolerances as everywhere: 1e-4 float, 2e-2 bfloat16 (per tensor, max-norm and Frobenius relative
error). Outputs are pre-filled with NaN."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "needs a GPU"
    from paper_2404_02882_amd import harness, lasp, synth_inputs
    return harness, lasp, synth_inputs


def oracle_all(oracle, inp, q=None, k=None, v=None, do=None):
    q = inp.q if q is None else q
    k = inp.k if k is None else k
    v = inp.v if v is None else v
    do = inp.dout if do is None else do
    if inp.log_g is None:
        out, kv = oracle.dims_fwd_brute(q, k, v, inp.decay, inp.kv_in)
        dq, dk, dv, din = oracle.dims_bwd_brute(q, k, v, do, inp.decay, inp.kv_in, inp.dkv_out)
        return dict(out=out, kv_out=kv, dq=dq, dk=dk, dv=dv, dkv_in=din)
    out, kv = oracle.dims_fwd_brute(q, k, v, None, inp.kv_in, log_g=inp.log_g)
    dq, dk, dv, dlg, din = oracle.dims_bwd_brute(q, k, v, do, None, inp.kv_in, inp.dkv_out, log_g=inp.log_g)
    return dict(out=out, kv_out=kv, dq=dq, dk=dk, dv=dv, dlog_g=dlg, dkv_in=din)


def compare(harness, got, ref, tol, label):
    for name, r in ref.items():
        assert got[name].shape == r.shape, (label, name, got[name].shape, r.shape)
        emax, efro = harness.rel_errors(got[name], r)
        say(f"  {label} {name:7s} max-rel {emax:.3e} fro-rel {efro:.3e}")
        assert np.isfinite(emax) and emax <= tol and efro <= tol, (label, name, emax, efro)


CASES = [
    # dtype, D (key), Dv (value), N, T, segments, states, token decay
    ("f32", 64, 128, 256, 1, 0, True, False),
    ("f32", 128, 64, 256, 1, 0, True, False),
    ("f32", 64, 128, 200, 1, 3, True, False),      # short last tile: fixed decay routed to the per-token kernels
    ("f32", 128, 64, 384, 3, 0, True, True),
    ("f32", 64, 128, 300, 1, 2, True, True),
    ("bf16", 64, 128, 512, 1, 0, True, False),
    ("bf16", 128, 64, 512, 2, 0, True, False),
    ("bf16", 64, 128, 448, 1, 0, False, False),    # odd tile count
    ("bf16", 128, 64, 1000, 1, 4, True, False),    # short last tile
    ("bf16", 64, 128, 768, 3, 0, True, True),
    ("bf16", 128, 64, 640, 1, 5, True, True),
]


@pytest.mark.parametrize("dtype,D,Dv,N,T,segments,states,token", CASES)
def test_small_against_definition(gpu, oracle, dtype, D, Dv, N, T, segments, states, token):
    harness, lasp, si = gpu
    cfg = si.Config("dims", B=2, H=3, N=N, D=D, chunk=64, dtype=dtype, seed=700 + D + N, Dv=Dv, token_decay=token)
    say(f"case dims dtype={dtype} D={D} Dv={Dv} N={N} T={T} segments={segments} states={states} token={token}")
    inp = si.make_inputs(cfg, with_states=states)
    if token:   # short sequences: strong, strongly varying decays so that every weight matters
        inp.log_g = np.log(np.random.default_rng(cfg.seed).uniform(0.8, 1.0, (2, 3, N))).astype(np.float32)
    else:
        inp.decay = np.array([0.9, 0.98, 1.0], dtype=np.float32)
    got = harness.run_gpu(inp, T=T, segments=segments)
    compare(harness, got, oracle_all(oracle, inp), TOL[dtype], "dims")


def test_grouped_heads_with_unequal_dims(gpu, oracle):
    harness, lasp, si = gpu
    cfg = si.Config("dimsg", B=1, H=4, N=320, D=64, chunk=64, dtype="bf16", seed=71, Dv=128)
    inp = si.make_inputs(cfg, with_states=True)
    inp.decay = np.array([0.9, 0.95, 0.99, 1.0], dtype=np.float32)
    G = 2
    kfull, vfull = inp.k.copy(), inp.v.copy()
    inp.k, inp.v = np.ascontiguousarray(kfull[:, ::G]), np.ascontiguousarray(vfull[:, ::G])   # two K/V heads
    got = harness.run_gpu(inp, T=1)
    ref = oracle_all(oracle, inp, k=oracle.group_expand(inp.k, G), v=oracle.group_expand(inp.v, G))
    ref["dk"], ref["dv"] = oracle.group_reduce(ref["dk"], G), oracle.group_reduce(ref["dv"], G)
    compare(harness, got, ref, TOL["bf16"], "dimsg")


def test_rejected_combinations(gpu):
    harness, lasp, si = gpu
    assert lasp.check_shape(lasp.make_shape(1, 2, 256, 64, 64, "bf16", Dv=128)) == 0
    assert lasp.check_shape(lasp.make_shape(1, 2, 256, 64, 64, "bf16", Dv=96)) == 2
    assert lasp.bidir_scratch_bytes(lasp.make_shape(1, 2, 256, 64, 64, "bf16", Dv=128)) == 0


def test_m3_full_size(gpu, oracle):
    """c3's shape with d_k = 64, d_v = 128 in the launch configuration bench.py times: the chunked C oracle
    on the zero-padded problem (an identity pinned on the CPU) for every head, and rows of the
    definition over all heads."""
    harness, lasp, si = gpu
    cfg = si.CONFIGS["m3"]
    heads = list(range(cfg.H))   # every head
    say("case m3: generating inputs")
    inp = si.make_inputs(cfg)
    say("case m3: gpu run")
    got = harness.run_gpu(inp, T=cfg.T)
    say("case m3: chunked oracle on the zero-padded problem, all heads")
    sel = lambda x: np.ascontiguousarray(x[:, heads])
    padk = lambda x: np.pad(sel(x), ((0, 0), (0, 0), (0, 0), (0, 128 - x.shape[3])))
    dec = inp.decay[heads]
    o, kv = oracle.fwd_chunked(padk(inp.q), padk(inp.k), sel(inp.v), dec, cfg.chunk)
    dq, dk, dv, din = oracle.bwd_chunked(padk(inp.q), padk(inp.k), sel(inp.v), sel(inp.dout), dec, cfg.chunk)
    ref = dict(out=o, kv_out=kv[:, :, :64], dq=dq[..., :64], dk=dk[..., :64], dv=dv, dkv_in=din[:, :, :64])
    for name, r in ref.items():
        emax, efro = harness.rel_errors(got[name][:, heads], r)
        say(f"  m3 {name:7s} max-rel {emax:.3e} fro-rel {efro:.3e}")
        assert emax <= TOL["bf16"] and efro <= TOL["bf16"], name
    say("case m3: brute-force rows of the zero-padded problem, all heads")
    rows = si.sample_rows(cfg, cfg.N, 128, seed=cfg.seed + 1)
    pad_all = lambda x: np.pad(np.asarray(x, dtype=np.float64), ((0, 0), (0, 0), (0, 0), (0, 128 - x.shape[3])))
    qp, kp = pad_all(inp.q), pad_all(inp.k)
    o = oracle.fwd_brute_rows(qp, kp, inp.v, inp.decay, rows)
    dq, dk, dv = oracle.bwd_brute_rows(qp, kp, inp.v, inp.dout, inp.decay, rows)
    b, h, s = rows[:, 0], rows[:, 1], rows[:, 2]
    for nm, r in (("out", o), ("dq", dq[:, :64]), ("dk", dk[:, :64]), ("dv", dv)):
        emax, efro = harness.rel_errors(got[nm][b, h, s], r)
        say(f"  m3 rows {nm:4s} max-rel {emax:.3e} fro-rel {efro:.3e}")
        assert emax <= TOL["bf16"] and efro <= TOL["bf16"], nm


@pytest.mark.parametrize("dtype,D,Dv,N,T,segments,token", [
    ("f32", 64, 128, 192, 1, 0, False), ("f32", 128, 64, 100, 1, 2, True),
    ("bf16", 64, 128, 512, 2, 0, False), ("bf16", 128, 64, 512, 1, 0, False),
    ("bf16", 128, 64, 448, 1, 3, False),          # odd tile count: the four-wave walk
    ("bf16", 64, 128, 640, 1, 0, True), ("bf16", 128, 64, 333, 1, 0, False),
])
def test_fused_norm_with_unequal_dims(gpu, oracle, dtype, D, Dv, N, T, segments, token):
    """The fused Norm runs over the d_v value features: y = Norm(o), gradients through it."""
    harness, lasp, si = gpu
    eps = 1e-5
    cfg = si.Config("dimsn", B=2, H=3, N=N, D=D, chunk=64, dtype=dtype, seed=760 + D + N, Dv=Dv, token_decay=token)
    say(f"case dims+norm dtype={dtype} D={D} Dv={Dv} N={N} T={T} segments={segments} token={token}")
    inp = si.make_inputs(cfg, with_states=True)
    if token:
        inp.log_g = np.log(np.random.default_rng(cfg.seed).uniform(0.8, 1.0, (2, 3, N))).astype(np.float32)
    else:
        inp.decay = np.array([0.9, 0.98, 1.0], dtype=np.float32)
    got = harness.run_gpu(inp, T=T, segments=segments, norm_eps=eps)
    lg = inp.log_g if token else None
    dec = None if token else inp.decay
    o, kvo = oracle.dims_fwd_brute(inp.q, inp.k, inp.v, dec, inp.kv_in, log_g=lg)
    y, rstd = oracle.norm_fwd(o, eps)
    do = oracle.norm_bwd(inp.dout, y, rstd)
    res = oracle.dims_bwd_brute(inp.q, inp.k, inp.v, do, dec, inp.kv_in, inp.dkv_out, log_g=lg)
    ref = dict(out=y, rstd=rstd, kv_out=kvo, dq=res[0], dk=res[1], dv=res[2], dkv_in=res[-1])
    if token:
        ref["dlog_g"] = res[3]
    compare(harness, got, ref, TOL[dtype], "dimsn")
