"""GPU parity: the HIP path, called through the C-ABI, against the fp64 oracle
on the same seeded inputs. Tolerances (per output tensor, both the max-norm and
the Frobenius relative error): 1e-4 for float data, 2e-2 for bfloat16 data.
The oracle sees the already-rounded inputs, so input quantisation is not
charged to the GPU. Outputs are pre-filled with NaN, so an unwritten element
fails the comparison."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
NAMES = ("out", "kv_out", "dq", "dk", "dv", "dkv_in")


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
    q, k, v, do = sel(inp.q), sel(inp.k), sel(inp.v), sel(inp.dout)
    decay = inp.decay if heads is None else inp.decay[heads]
    kv_in, g = sel(inp.kv_in), sel(inp.dkv_out)
    ref = {}
    if form == "brute":
        ref["out"], ref["kv_out"] = oracle.fwd_brute(q, k, v, decay, kv_in)
        if not inp.cfg.fwd_only:
            ref["dq"], ref["dk"], ref["dv"], ref["dkv_in"] = oracle.bwd_brute(q, k, v, do, decay, kv_in, g)
    else:
        ref["out"], ref["kv_out"] = oracle.fwd_chunked(q, k, v, decay, chunk, kv_in)
        if not inp.cfg.fwd_only:
            ref["dq"], ref["dk"], ref["dv"], ref["dkv_in"] = oracle.bwd_chunked(q, k, v, do, decay, chunk, kv_in, g)
    return ref


def compare(harness, got, ref, tol, label, heads=None):
    worst = 0.0
    for name in NAMES:
        if name not in ref:
            continue
        x = got[name] if heads is None else got[name][:, heads]
        emax, efro = harness.rel_errors(x, ref[name])
        say(f"  {label} {name:7s} max-rel {emax:.3e} fro-rel {efro:.3e}")
        assert np.isfinite(emax) and emax <= tol and efro <= tol, (label, name, emax, efro)
        worst = max(worst, emax, efro)
    return worst


# ------------------------------------------------------------------ small cases, every tile shape
SMALL = [
    # dtype, D, chunk, tiles, segments, states, lam
    ("f32", 64, 64, 4, 0, False, "one"),
    ("f32", 64, 64, 5, 2, True, "schedule"),
    ("f32", 128, 128, 3, 3, True, "schedule"),
    ("f32", 128, 64, 7, 1, True, "schedule"),
    ("bf16", 64, 64, 5, 2, True, "schedule"),
    ("bf16", 64, 128, 3, 0, True, "schedule"),
    ("bf16", 128, 64, 5, 3, True, "schedule"),
    ("bf16", 128, 128, 5, 2, True, "schedule"),
    ("bf16", 128, 128, 1, 1, False, "schedule"),
    ("bf16", 128, 256, 3, 2, True, "schedule"),
    ("bf16", 64, 256, 2, 0, True, "one"),
]


@pytest.mark.parametrize("dtype,D,chunk,nchunks,segments,states,lam", SMALL)
def test_small_against_brute_force(gpu, oracle, dtype, D, chunk, nchunks, segments, states, lam):
    harness, lasp, si = gpu
    N = chunk * nchunks
    cfg = si.Config("small", B=2, H=3, N=N, D=D, chunk=chunk, dtype=dtype, seed=100 + D + chunk + nchunks, decay=lam)
    say(f"case dtype={dtype} D={D} chunk={chunk} N={N} segments={segments} states={states} decay={lam}")
    inp = si.make_inputs(cfg, with_states=states)
    if lam == "schedule":   # short sequences: use strong decays so that the mask matters
        inp.decay = np.array([0.9, 0.97, 1.0 - 2.0 ** -7], dtype=np.float32)
    got = harness.run_gpu(inp, segments=segments)
    ref = oracle_all(oracle, inp)
    compare(harness, got, ref, TOL[dtype], "small")


def test_ragged_segments_and_determinism(gpu, oracle):
    """Segment counts that do not divide the tile count, and bit-identical reruns (no atomics)."""
    harness, lasp, si = gpu
    cfg = si.Config("ragged", B=1, H=2, N=64 * 11, D=64, chunk=64, dtype="bf16", seed=5)
    inp = si.make_inputs(cfg, with_states=True)
    ref = oracle_all(oracle, inp)
    first = None
    for segments in (1, 2, 3, 4, 7, 11):
        say(f"case ragged segments={segments}")
        got = harness.run_gpu(inp, segments=segments)
        compare(harness, got, ref, TOL["bf16"], f"seg{segments}")
        if segments == 4:
            again = harness.run_gpu(inp, segments=segments)
            for name in NAMES:
                assert np.array_equal(got[name], again[name]), name
        first = first or got


def test_even_tile_counts_pair_cache(gpu, oracle):
    """Even tile counts use the paired state cache (one cached state per two tiles);
    segment requests that are odd or do not divide the tiles are rounded to whole pairs."""
    harness, lasp, si = gpu
    for D in (64, 128):
        cfg = si.Config("pairs", B=1, H=2, N=64 * 12, D=D, chunk=64, dtype="bf16", seed=6 + D)
        inp = si.make_inputs(cfg, with_states=True)
        inp.decay = np.array([0.95, 1.0 - 2.0 ** -9], dtype=np.float32)
        ref = oracle_all(oracle, inp)
        for segments in (1, 2, 3, 5, 6, 12):
            say(f"case pairs D={D} segments={segments}")
            got = harness.run_gpu(inp, segments=segments)
            compare(harness, got, ref, TOL["bf16"], f"D{D}/seg{segments}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_extreme_decays(gpu, oracle, dtype):
    """Degenerate decays in one launch: lambda = 1 (no decay), lambda close to 1, and
    decays so strong that lambda^tile underflows to zero. Nothing may overflow or go NaN."""
    harness, lasp, si = gpu
    cfg = si.Config("decays", B=1, H=4, N=512, D=64, chunk=128, dtype=dtype, seed=21)
    inp = si.make_inputs(cfg, with_states=True)
    inp.decay = np.array([1.0, 1.0 - 2.0 ** -20, 0.05, 1e-4], dtype=np.float32)
    got = harness.run_gpu(inp, segments=4)
    ref = oracle_all(oracle, inp)
    for name in NAMES:
        assert np.all(np.isfinite(got[name])), name
    compare(harness, got, ref, TOL[dtype], f"decays/{dtype}")


def test_single_head_single_tile_and_reuse(gpu, oracle):
    """Smallest launches (one head, one tile) and a second call on the same workspace
    with different data: stale scratch or cache contents must not leak into results."""
    harness, lasp, si = gpu
    for dtype, n in (("bf16", 64), ("f32", 64), ("bf16", 128)):
        cfg = si.Config("tiny", B=1, H=1, N=n, D=128, chunk=64, dtype=dtype, seed=31)
        a = si.make_inputs(cfg, with_states=True)
        b = si.make_inputs(cfg, with_states=False, seed=32)
        for inp in (a, b):
            got = harness.run_gpu(inp)
            compare(harness, got, oracle_all(oracle, inp), TOL[dtype], f"tiny/{dtype}/{n}")


def test_lambda_one_chunk1_limit(gpu, oracle):
    """lambda = 1 (ordinary linear attention) in float: textbook tril(QK^T)V."""
    harness, lasp, si = gpu
    cfg = si.Config("lam1", B=1, H=2, N=128, D=64, chunk=64, dtype="f32", seed=9, decay="one")
    inp = si.make_inputs(cfg)
    got = harness.run_gpu(inp)
    for h in range(2):
        q, k, v = (x[0, h].astype(np.float64) for x in (inp.q, inp.k, inp.v))
        ref = np.tril(q @ k.T) @ v
        emax, _ = harness.rel_errors(got["out"][0, h], ref)
        assert emax <= 1e-4
        emax, _ = harness.rel_errors(got["kv_out"][0, h], k.T @ v)
        assert emax <= 1e-4


# ------------------------------------------------------------------ the named configurations
def test_c1_fp32_forward(gpu, oracle):
    harness, lasp, si = gpu
    inp = si.make_inputs(si.CONFIGS["c1"])
    say("case c1")
    got = harness.run_gpu(inp, backward=False)
    ref = oracle_all(oracle, inp)
    compare(harness, got, ref, TOL["f32"], "c1")
    o2, kv2 = oracle.fwd_recurrent(inp.q, inp.k, inp.v, inp.decay)
    assert harness.rel_errors(got["out"], o2)[0] <= 1e-4


def test_c2_split_and_unsplit(gpu, oracle):
    harness, lasp, si = gpu
    cfg = si.CONFIGS["c2"]
    inp = si.make_inputs(cfg)
    say("case c2 oracle (brute force, full)")
    ref = oracle_all(oracle, inp)
    say("case c2 unsplit")
    one = harness.run_gpu(inp, T=1)
    compare(harness, one, ref, TOL["bf16"], "c2/T1")
    say("case c2 T=4")
    four = harness.run_gpu(inp, T=cfg.T)
    compare(harness, four, ref, TOL["bf16"], "c2/T4")
    for name in NAMES:
        emax, efro = harness.rel_errors(four[name], one[name])
        assert emax <= TOL["bf16"] and efro <= TOL["bf16"], name


def _big_config(gpu, oracle, name, heads, nrows=256, also_unsplit=False):
    """Full-size run in the launch configuration bench.py uses (segments = auto);
    full-tensor comparison (every output tensor and both states) against the chunked
    oracle on `heads` (None = every head), and brute-force rows sampled over all heads. `also_unsplit`: the whole sequence
    once more as a single call (the largest N one call sees)."""
    harness, lasp, si = gpu
    cfg = si.CONFIGS[name]
    say(f"case {name}: generating inputs")
    inp = si.make_inputs(cfg)
    say(f"case {name}: chunked oracle on heads {'all' if heads is None else heads}")
    ref = oracle_all(oracle, inp, form="chunked", chunk=cfg.chunk, heads=heads)
    say(f"case {name}: brute-force rows")
    rows = si.sample_rows(cfg, cfg.N, nrows, seed=cfg.seed + 1)
    o = oracle.fwd_brute_rows(inp.q, inp.k, inp.v, inp.decay, rows)
    dq, dk, dv = oracle.bwd_brute_rows(inp.q, inp.k, inp.v, inp.dout, inp.decay, rows)
    b, h, s = rows[:, 0], rows[:, 1], rows[:, 2]
    for T in ((cfg.T, 1) if also_unsplit and cfg.T != 1 else (cfg.T,)):
        say(f"case {name}: gpu run T={T}")
        got = harness.run_gpu(inp, T=T)
        compare(harness, got, ref, TOL[cfg.dtype], f"{name}/T{T}", heads=heads)
        for nm, r in (("out", o), ("dq", dq), ("dk", dk), ("dv", dv)):
            x = got[nm][b, h, s]
            emax, efro = harness.rel_errors(x, r)
            say(f"  {name}/T{T} rows {nm:4s} max-rel {emax:.3e} fro-rel {efro:.3e}")
            assert emax <= TOL[cfg.dtype] and efro <= TOL[cfg.dtype], (name, nm)
        del got


def test_c3_full_size(gpu, oracle):
    _big_config(gpu, oracle, "c3", heads=None)   # every head, every tensor


def test_c5_outlier_rows(gpu, oracle):
    _big_config(gpu, oracle, "c5", heads=list(range(0, 32, 2)) + [31], nrows=128)   # 17 of 32 heads, all four batch entries


def test_c4_long_sequence(gpu, oracle):
    import torch
    harness, lasp, si = gpu
    torch.cuda.reset_peak_memory_stats()
    _big_config(gpu, oracle, "c4", heads=list(range(1, 16, 2)) + [0], nrows=64, also_unsplit=True)   # 9 of 16 heads
    say(f"  c4 peak device memory {torch.cuda.max_memory_allocated() / 2**30:.2f} GiB")
