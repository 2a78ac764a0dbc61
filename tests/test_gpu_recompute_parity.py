"""GPU parity of the backward pass without a state cache (state_cache = NULL: the states are rebuilt from
k, v and kv_in, Sec. 3.4's recomputation instead of caching), through the C-ABI, against the fp64 oracle and
against the cached path (same kernels after the rebuild: bit-identical gradients)."""
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


CASES = [
    # dtype, D, N, T, segments, token decay
    ("f32", 64, 32 * 7, 1, 3, False),
    ("bf16", 64, 64 * 6, 2, 0, False),
    ("bf16", 128, 64 * 12, 1, 4, False),     # even tile count: one cached state per pair of tiles
    ("bf16", 128, 64 * 5, 1, 2, False),      # odd tile count
    ("bf16", 128, 64 * 9 + 21, 3, 0, False), # short last tiles (log g synthesised)
    ("f32", 128, 32 * 6, 2, 2, True),
    ("bf16", 128, 64 * 8, 2, 0, True),
    ("bf16", 64, 64 * 5 + 3, 1, 2, True),
]


@pytest.mark.parametrize("dtype,D,N,T,segments,token", CASES)
def test_recompute_against_oracle_and_cached_path(gpu, oracle, dtype, D, N, T, segments, token):
    harness, lasp, si = gpu
    n_total = N if N % T == 0 else N - N % T
    cfg = si.Config("recompute", B=2, H=3, N=n_total, D=D, chunk=64, dtype=dtype, seed=7000 + N + D, token_decay=token)
    inp = si.make_inputs(cfg, with_states=True)
    if not token:
        inp.decay = np.array([0.9, 0.97, 1.0 - 2.0 ** -7], dtype=np.float32)
    say(f"case recompute dtype={dtype} D={D} N={n_total} T={T} segments={segments} token={token}")
    cached = harness.run_gpu(inp, T=T, segments=segments)
    got = harness.run_gpu(inp, T=T, segments=segments, recompute=True)
    if token:
        ref = dict(zip(("dq", "dk", "dv", "dlog_g", "dkv_in"),
                       oracle.gated_bwd_brute(inp.q, inp.k, inp.v, inp.dout, inp.log_g, inp.kv_in, inp.dkv_out)))
    else:
        ref = dict(zip(("dq", "dk", "dv", "dkv_in"), oracle.bwd_brute(inp.q, inp.k, inp.v, inp.dout, inp.decay, inp.kv_in, inp.dkv_out)))
    for name, r in ref.items():
        emax, efro = harness.rel_errors(got[name], r)
        same = np.array_equal(got[name], cached[name])
        say(f"  recompute {name:7s} max-rel {emax:.3e} fro-rel {efro:.3e} {'= cached path' if same else 'differs from the cached path'}")
        assert np.isfinite(emax) and emax <= TOL[dtype] and efro <= TOL[dtype], name
        assert same, name


def test_recompute_with_norm_and_grouped_heads(gpu, oracle):
    """The rebuilt states serve the fused Norm and grouped K/V heads as well."""
    harness, lasp, si = gpu
    cfg = si.Config("recompute_n", B=1, H=4, N=64 * 6, D=128, chunk=128, dtype="bf16", seed=7100)
    inp = si.make_inputs(cfg, with_states=True)
    a = harness.run_gpu(inp, T=2, norm_eps=1e-5)
    b = harness.run_gpu(inp, T=2, norm_eps=1e-5, recompute=True)
    for name in ("dq", "dk", "dv", "dkv_in"):
        assert np.array_equal(a[name], b[name]), name
    inp.k, inp.v = np.ascontiguousarray(inp.k[:, ::2]), np.ascontiguousarray(inp.v[:, ::2])   # two K/V heads for four query heads
    a = harness.run_gpu(inp, T=1)
    b = harness.run_gpu(inp, T=1, recompute=True)
    for name in ("dq", "dk", "dv", "dkv_in"):
        assert np.array_equal(a[name], b[name]) and np.all(np.isfinite(b[name])), name


@pytest.mark.parametrize("D,Dv,N,T", [(64, 128, 64 * 8, 2), (128, 64, 64 * 6, 1), (64, 128, 64 * 5, 1)])
def test_recompute_with_unequal_dims(gpu, oracle, D, Dv, N, T):
    """Key and value dimensions that differ: the rebuilt cache has the same [d_k][d_v] slots as the stored one."""
    harness, lasp, si = gpu
    cfg = si.Config("recompute_d", B=1, H=3, N=N, D=D, chunk=64, dtype="bf16", seed=7200 + D + N, Dv=Dv)
    inp = si.make_inputs(cfg, with_states=True)
    say(f"case recompute dims D={D} Dv={Dv} N={N} T={T}")
    a = harness.run_gpu(inp, T=T)
    b = harness.run_gpu(inp, T=T, recompute=True)
    ref = dict(zip(("dq", "dk", "dv", "dkv_in"), oracle.dims_bwd_brute(inp.q, inp.k, inp.v, inp.dout, inp.decay, inp.kv_in, inp.dkv_out)))
    for name, r in ref.items():
        emax, efro = harness.rel_errors(b[name], r)
        say(f"  recompute dims {name:7s} max-rel {emax:.3e} fro-rel {efro:.3e}")
        assert emax <= TOL["bf16"] and efro <= TOL["bf16"], name
        assert np.array_equal(a[name], b[name]), name


def test_recompute_full_size_c3(gpu, oracle):
    """c3 in bench.py's launch configuration without a state cache: every gradient tensor of every head."""
    harness, lasp, si = gpu
    cfg = si.CONFIGS["c3"]
    inp = si.make_inputs(cfg)
    say("case recompute c3: gpu run")
    got = harness.run_gpu(inp, T=cfg.T, recompute=True)
    say("case recompute c3: chunked oracle, all heads")
    ref = dict(zip(("dq", "dk", "dv", "dkv_in"), oracle.bwd_chunked(inp.q, inp.k, inp.v, inp.dout, inp.decay, cfg.chunk)))
    for name, r in ref.items():
        emax, efro = harness.rel_errors(got[name], r)
        say(f"  recompute c3 {name:7s} max-rel {emax:.3e} fro-rel {efro:.3e}")
        assert emax <= TOL["bf16"] and efro <= TOL["bf16"], name
