"""GPU parity of the per-token-decay entry points (lasp_gated_fwd / lasp_gated_bwd,
called through the C-ABI) against the fp64 oracle on the same seeded inputs.
Tolerances as for the fixed decay (per output tensor, max-norm and Frobenius
relative error): 1e-4 for float data, 2e-2 for bfloat16 data; dlog_g is held to
the same bound. Outputs are pre-filled with NaN."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
NAMES = ("out", "kv_out", "dq", "dk", "dv", "dlog_g", "dkv_in")


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "needs a GPU"
    from paper_2404_02882_amd import harness, lasp, synth_inputs
    return harness, lasp, synth_inputs


def oracle_all(oracle, inp, form="brute", chunk=None, heads=None):
    sel = (lambda x: x) if heads is None else (lambda x: None if x is None else np.ascontiguousarray(x[:, heads]))
    q, k, v, do, lg = sel(inp.q), sel(inp.k), sel(inp.v), sel(inp.dout), sel(inp.log_g)
    kv_in, g = sel(inp.kv_in), sel(inp.dkv_out)
    if form == "brute":
        fwd = oracle.gated_fwd_brute(q, k, v, lg, kv_in)
        bwd = oracle.gated_bwd_brute(q, k, v, do, lg, kv_in, g)
    elif form == "recurrent":
        fwd = oracle.gated_fwd_recurrent(q, k, v, lg, kv_in)
        bwd = oracle.gated_bwd_recurrent(q, k, v, do, lg, kv_in, g)
    else:
        fwd = oracle.gated_fwd_chunked(q, k, v, lg, chunk, kv_in)
        bwd = oracle.gated_bwd_chunked(q, k, v, do, lg, chunk, kv_in, g)
    return dict(zip(NAMES, tuple(fwd) + tuple(bwd)))


def compare(harness, got, ref, tol, label, heads=None):
    for name in NAMES:
        x = got[name] if heads is None else got[name][:, heads]
        emax, efro = harness.rel_errors(x, ref[name])
        say(f"  {label} {name:7s} max-rel {emax:.3e} fro-rel {efro:.3e}")
        assert np.isfinite(emax) and emax <= tol and efro <= tol, (label, name, emax, efro)


SMALL = [
    # dtype, D, chunk, tiles, segments, states
    ("f32", 64, 64, 4, 0, False),
    ("f32", 64, 64, 5, 2, True),
    ("f32", 128, 128, 3, 3, True),
    ("f32", 128, 64, 7, 1, True),
    ("bf16", 64, 64, 5, 2, True),
    ("bf16", 64, 128, 3, 0, True),
    ("bf16", 128, 64, 5, 3, True),
    ("bf16", 128, 128, 4, 2, True),
    ("bf16", 128, 128, 1, 1, False),
    ("bf16", 64, 256, 2, 0, False),
]


@pytest.mark.parametrize("dtype,D,chunk,nchunks,segments,states", SMALL)
def test_small_against_brute_force(gpu, oracle, dtype, D, chunk, nchunks, segments, states):
    harness, lasp, si = gpu
    N = chunk * nchunks
    cfg = si.Config("gsmall", B=2, H=3, N=N, D=D, chunk=chunk, dtype=dtype, seed=300 + D + chunk + nchunks,
                    token_decay=True)
    say(f"case gated dtype={dtype} D={D} chunk={chunk} N={N} segments={segments} states={states}")
    inp = si.make_inputs(cfg, with_states=states)
    # short sequences: strong, strongly varying decays so that every weight matters
    rng = np.random.default_rng(cfg.seed)
    inp.log_g = np.log(rng.uniform(0.8, 1.0, (2, 3, N))).astype(np.float32)
    assert lasp.check_log_decay(inp.log_g) == 0
    got = harness.run_gpu(inp, segments=segments)
    compare(harness, got, oracle_all(oracle, inp), TOL[dtype], "gsmall")


def test_constant_gate_matches_fixed_decay_path(gpu, oracle):
    """log g = log lambda_h for every token: the per-token kernels must reproduce the fixed-decay ones
    (same oracle values; the two GPU paths agree with each other far inside the tolerance)."""
    harness, lasp, si = gpu
    cfg = si.Config("gconst", B=1, H=4, N=64 * 6, D=128, chunk=64, dtype="f32", seed=41)
    inp = si.make_inputs(cfg, with_states=True)
    inp.decay = np.array([0.9, 0.97, 0.995, 1.0], dtype=np.float32)
    fixed = harness.run_gpu(inp, segments=3)
    inp.log_g = np.broadcast_to(np.log(inp.decay.astype(np.float64))[None, :, None], (1, 4, cfg.N)).astype(np.float32)
    gated = harness.run_gpu(inp, segments=3)
    for name in ("out", "kv_out", "dq", "dk", "dv", "dkv_in"):
        emax, _ = harness.rel_errors(gated[name], fixed[name])
        say(f"  gconst {name:7s} gated vs fixed max-rel {emax:.3e}")
        assert emax <= 1e-5, name
    compare(harness, gated, oracle_all(oracle, inp), TOL["f32"], "gconst")


def test_ragged_segments_and_determinism(gpu, oracle):
    harness, lasp, si = gpu
    cfg = si.Config("gragged", B=1, H=2, N=64 * 11, D=64, chunk=64, dtype="bf16", seed=45, token_decay=True)
    inp = si.make_inputs(cfg, with_states=True)
    ref = oracle_all(oracle, inp)
    for segments in (1, 2, 3, 4, 7, 11):
        say(f"case gated ragged segments={segments}")
        got = harness.run_gpu(inp, segments=segments)
        compare(harness, got, ref, TOL["bf16"], f"gseg{segments}")
        if segments == 4:
            again = harness.run_gpu(inp, segments=segments)
            for name in NAMES:
                assert np.array_equal(got[name], again[name]), name


def test_even_tile_counts_pair_cache(gpu, oracle):
    """Even tile counts use the paired state cache and the 128-token local pass; segment requests
    that are odd or do not divide the tiles are rounded to whole pairs."""
    harness, lasp, si = gpu
    for D in (64, 128):
        cfg = si.Config("gpairs", B=1, H=2, N=64 * 12, D=D, chunk=64, dtype="bf16", seed=46 + D, token_decay=True)
        inp = si.make_inputs(cfg, with_states=True)
        rng = np.random.default_rng(cfg.seed)
        inp.log_g = np.log(rng.uniform(0.85, 1.0, (1, 2, cfg.N))).astype(np.float32)
        ref = oracle_all(oracle, inp)
        for segments in (1, 2, 3, 5, 6, 12):
            say(f"case gated pairs D={D} segments={segments}")
            got = harness.run_gpu(inp, segments=segments)
            compare(harness, got, ref, TOL["bf16"], f"gD{D}/seg{segments}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_extreme_gates(gpu, oracle, dtype):
    """No decay at all, gates that almost close (the state is cut there), and a head whose every
    token decays so strongly that a tile's product underflows: finite results, parity."""
    harness, lasp, si = gpu
    cfg = si.Config("gext", B=1, H=4, N=512, D=64, chunk=128, dtype=dtype, seed=47, token_decay=True)
    inp = si.make_inputs(cfg, with_states=True)
    lg = np.zeros((1, 4, 512), dtype=np.float32)            # head 0: g = 1
    lg[0, 1] = -1e-6                                          # head 1: almost 1
    lg[0, 2, ::37] = -30.0                                    # head 2: the gate closes every 37 tokens
    lg[0, 3] = -3.0                                           # head 3: e^-192 per 64-token tile
    inp.log_g = lg
    got = harness.run_gpu(inp, segments=4)
    for name in NAMES:
        assert np.all(np.isfinite(got[name])), name
    compare(harness, got, oracle_all(oracle, inp), TOL[dtype], f"gext/{dtype}")


def test_g2_split_and_unsplit(gpu, oracle):
    """c2's shape with a decay per token, as one call and as T=4 chained calls (dlog_g's boundary
    term <dkv_out, kv_out> links the pieces), against the recurrent oracle."""
    harness, lasp, si = gpu
    cfg = si.CONFIGS["g2"]
    inp = si.make_inputs(cfg)
    say("case g2 oracle (recurrent, full)")
    ref = oracle_all(oracle, inp, form="recurrent")
    one = harness.run_gpu(inp, T=1)
    compare(harness, one, ref, TOL["bf16"], "g2/T1")
    four = harness.run_gpu(inp, T=cfg.T)
    compare(harness, four, ref, TOL["bf16"], "g2/T4")
    rows = si.sample_rows(cfg, cfg.N, 64, seed=cfg.seed + 1)
    o = oracle.gated_fwd_brute_rows(inp.q, inp.k, inp.v, inp.log_g, rows)
    dq, dk, dv = oracle.gated_bwd_brute_rows(inp.q, inp.k, inp.v, inp.dout, inp.log_g, rows)
    b, h, s = rows[:, 0], rows[:, 1], rows[:, 2]
    for nm, r in (("out", o), ("dq", dq), ("dk", dk), ("dv", dv)):
        emax, efro = harness.rel_errors(four[nm][b, h, s], r)
        say(f"  g2 rows {nm:4s} max-rel {emax:.3e} fro-rel {efro:.3e}")
        assert emax <= TOL["bf16"] and efro <= TOL["bf16"], nm


def test_g3_full_size(gpu, oracle):
    """The benchmark shape with a decay per token, in the launch configuration bench.py times:
    full tensors against the chunked oracle on every head, brute-force rows over all heads."""
    harness, lasp, si = gpu
    cfg = si.CONFIGS["g3"]
    heads = None   # every head
    say("case g3: generating inputs")
    inp = si.make_inputs(cfg)
    say("case g3: gpu run")
    got = harness.run_gpu(inp, T=cfg.T)
    say("case g3: chunked oracle on all heads")
    ref = oracle_all(oracle, inp, form="chunked", chunk=cfg.chunk, heads=heads)
    compare(harness, got, ref, TOL["bf16"], "g3", heads=heads)
    say("case g3: brute-force rows")
    rows = si.sample_rows(cfg, cfg.N, 256, seed=cfg.seed + 1)
    o = oracle.gated_fwd_brute_rows(inp.q, inp.k, inp.v, inp.log_g, rows)
    dq, dk, dv = oracle.gated_bwd_brute_rows(inp.q, inp.k, inp.v, inp.dout, inp.log_g, rows)
    b, h, s = rows[:, 0], rows[:, 1], rows[:, 2]
    for nm, r in (("out", o), ("dq", dq), ("dk", dk), ("dv", dv)):
        emax, efro = harness.rel_errors(got[nm][b, h, s], r)
        say(f"  g3 rows {nm:4s} max-rel {emax:.3e} fro-rel {efro:.3e}")
        assert emax <= TOL["bf16"] and efro <= TOL["bf16"], nm
