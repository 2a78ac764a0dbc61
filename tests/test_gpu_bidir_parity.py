"""GPU parity of the bidirectional entry points (lasp_bidir_state / lasp_bidir_fwd / lasp_bidir_bwd,
called through the C-ABI) against the fp64 oracle's definition O = (Q K^T) V on the same seeded
inputs. Tolerances as for the causal path (per tensor, max-norm and Frobenius relative error):
1e-4 for float data, 2e-2 for bfloat16 data. Outputs and states are pre-filled with NaN."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
NAMES = ("out", "kv", "dq", "dk", "dv", "dkv")


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "needs a GPU"
    from paper_2404_02882_amd import harness, lasp, synth_inputs
    return harness, lasp, synth_inputs


def oracle_all(oracle, inp, heads=None):
    sel = (lambda x: x) if heads is None else (lambda x: np.ascontiguousarray(x[:, heads]))
    q, k, v, do = sel(inp.q), sel(inp.k), sel(inp.v), sel(inp.dout)
    dq, dk, dv = oracle.bidir_bwd_left(q, k, v, do)
    return dict(out=oracle.bidir_fwd_left(q, k, v), kv=oracle.bidir_state(k, v), dq=dq, dk=dk, dv=dv,
                dkv=oracle.bidir_state(q, do))


def compare(harness, got, ref, tol, label, heads=None):
    for name in NAMES:
        x = got[name] if heads is None else got[name][:, heads]
        emax, efro = harness.rel_errors(x, ref[name])
        say(f"  {label} {name:4s} max-rel {emax:.3e} fro-rel {efro:.3e}")
        assert np.isfinite(emax) and emax <= tol and efro <= tol, (label, name, emax, efro)


SMALL = [
    # dtype, D, N, sub-sequence lengths (None = one), segments
    ("f32", 64, 256, None, 0),
    ("f32", 64, 200, None, 0),          # short last tile
    ("f32", 128, 321, [100, 1, 220], 0),
    ("f32", 128, 96, None, 3),
    ("bf16", 64, 512, None, 0),
    ("bf16", 64, 333, [33, 300], 0),
    ("bf16", 128, 640, None, 0),
    ("bf16", 128, 1000, [1, 487, 512], 0),
    ("bf16", 128, 777, None, 1),
    ("bf16", 128, 777, None, 13),
    ("bf16", 128, 1, None, 0),          # a single token
    ("bf16", 64, 63, None, 0),
]


@pytest.mark.parametrize("dtype,D,N,lengths,segments", SMALL)
def test_small_against_definition(gpu, oracle, dtype, D, N, lengths, segments):
    harness, lasp, si = gpu
    cfg = si.Config("bsmall", B=2, H=3, N=N, D=D, chunk=64, dtype=dtype, seed=500 + D + N, decay="one", bidirectional=True)
    say(f"case bidir dtype={dtype} D={D} N={N} lengths={lengths} segments={segments}")
    inp = si.make_inputs(cfg)
    got = harness.run_gpu_bidir(inp, lengths=lengths, segments=segments)
    compare(harness, got, oracle_all(oracle, inp), TOL[dtype], "bsmall")


def test_split_does_not_change_values_much_and_runs_are_bit_reproducible(gpu, oracle):
    harness, lasp, si = gpu
    cfg = si.Config("bdet", B=1, H=4, N=1536, D=128, chunk=128, dtype="bf16", seed=61, decay="one", bidirectional=True)
    inp = si.make_inputs(cfg)
    ref = oracle_all(oracle, inp)
    one = harness.run_gpu_bidir(inp)
    again = harness.run_gpu_bidir(inp)
    for name in NAMES:
        assert np.array_equal(one[name], again[name]), name
    for lengths in ([768, 768], [512, 1, 1023], [64] * 24):
        got = harness.run_gpu_bidir(inp, lengths=lengths)
        compare(harness, got, ref, TOL["bf16"], f"bsplit{len(lengths)}")


def test_accumulate_adds_to_a_given_state(gpu, oracle):
    """accumulate != 0 adds to whatever the state holds (a partial state received from elsewhere)."""
    import torch
    harness, lasp, si = gpu
    cfg = si.Config("bacc", B=1, H=2, N=300, D=64, chunk=64, dtype="f32", seed=62, decay="one", bidirectional=True)
    inp = si.make_inputs(cfg)
    shp = lasp.make_shape(1, 2, 300, 64, 64, "f32")
    k, v = harness.to_device(inp.k, "f32"), harness.to_device(inp.v, "f32")
    start = np.random.default_rng(63).standard_normal((1, 2, 64, 64)).astype(np.float32)
    state = torch.from_numpy(start.copy()).cuda()
    scratch = torch.empty(lasp.bidir_scratch_bytes(shp), dtype=torch.uint8, device="cuda")
    lasp.lasp_bidir_state(shp, k, v, state, True, scratch)
    torch.cuda.synchronize()
    emax, _ = harness.rel_errors(state.cpu().numpy(), start.astype(np.float64) + oracle.bidir_state(inp.k, inp.v))
    say(f"  bacc state max-rel {emax:.3e}")
    assert emax <= TOL["f32"]


def test_b2_whole_and_in_four_pieces(gpu, oracle):
    harness, lasp, si = gpu
    cfg = si.CONFIGS["b2"]
    inp = si.make_inputs(cfg)
    say("case b2 oracle (definition, full)")
    ref = oracle_all(oracle, inp)
    compare(harness, harness.run_gpu_bidir(inp), ref, TOL["bf16"], "b2/T1")
    compare(harness, harness.run_gpu_bidir(inp, lengths=[cfg.N // cfg.T] * cfg.T), ref, TOL["bf16"], "b2/T4")


def test_b3_full_size(gpu, oracle):
    """The benchmark shape in the launch configuration bench.py times: full tensors against the
    oracle's right-product form (pinned to the definition on the CPU) and rows of the definition itself."""
    harness, lasp, si = gpu
    cfg = si.CONFIGS["b3"]
    say("case b3: generating inputs")
    inp = si.make_inputs(cfg)
    say("case b3: gpu run")
    got = harness.run_gpu_bidir(inp)
    say("case b3: oracle, right-product form, all heads")
    kv, dkv = oracle.bidir_state(inp.k, inp.v), oracle.bidir_state(inp.q, inp.dout)
    T = lambda x: np.swapaxes(x, -1, -2)
    ref = dict(out=oracle.bidir_fwd_right(inp.q, kv), kv=kv, dkv=dkv, dq=oracle.bidir_fwd_right(inp.dout, T(kv)),
               dk=oracle.bidir_fwd_right(inp.v, T(dkv)), dv=oracle.bidir_fwd_right(inp.k, dkv))
    compare(harness, got, ref, TOL["bf16"], "b3")
    say("case b3: rows of the definition")
    rows = si.sample_rows(cfg, cfg.N, 256, seed=cfg.seed + 1)
    o = oracle.bidir_fwd_rows(inp.q, inp.k, inp.v, rows)
    dq, dk, dv = oracle.bidir_bwd_rows(inp.q, inp.k, inp.v, inp.dout, rows)
    b, h, s = rows[:, 0], rows[:, 1], rows[:, 2]
    for nm, r in (("out", o), ("dq", dq), ("dk", dk), ("dv", dv)):
        emax, efro = harness.rel_errors(got[nm][b, h, s], r)
        say(f"  b3 rows {nm:4s} max-rel {emax:.3e} fro-rel {efro:.3e}")
        assert emax <= TOL["bf16"] and efro <= TOL["bf16"], nm
