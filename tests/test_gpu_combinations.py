"""Seeded random combinations of everything the causal entry points accept at once (data type, key and
value dimension, length with or without a short last tile, sub-sequences, segments, one lambda per
head or a decay per token, fused Norm, grouped K/V heads, boundary states) against the fp64 oracle
composed from its pinned parts. The options are meant to be independent of each other; this is the
test that they are. Tolerances: 1e-4 float, 2e-2 bfloat16."""
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


def draw_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        dtype = ("f32", "bf16")[int(rng.integers(2))]
        D = (64, 128)[int(rng.integers(2))]
        Dv = (0, 64, 128)[int(rng.integers(3))]
        tile = 32 if dtype == "f32" else 64
        T = int(rng.integers(1, 4))
        if rng.random() < 0.5:      # every sub-sequence a whole number of tiles
            n_sub = tile * int(rng.integers(1, 6))
        else:                        # a short last tile in every sub-sequence
            n_sub = int(rng.integers(1, 5 * tile))
        H = (2, 4, 6)[int(rng.integers(3))]
        groups = [g for g in (1, 2, H) if H % g == 0]
        G = groups[int(rng.integers(len(groups)))]
        ntiles = -(-n_sub // tile)
        segments = int(rng.integers(0, ntiles + 1))
        cases.append(dict(id=i, dtype=dtype, D=D, Dv=Dv, n_sub=n_sub, T=T, H=H, G=G, segments=segments,
                          token=bool(rng.random() < 0.5), norm=bool(rng.random() < 0.5),
                          states=bool(rng.random() < 0.7), seed=int(rng.integers(1 << 30))))
    return cases


CASES = draw_cases(100, 20240402)


@pytest.mark.parametrize("c", CASES, ids=lambda c: f"{c['id']}-{c['dtype']}-D{c['D']}-Dv{c['Dv']}-n{c['n_sub']}x{c['T']}-H{c['H']}g{c['G']}"
                                                       f"-s{c['segments']}{'-tok' if c['token'] else ''}{'-norm' if c['norm'] else ''}")
def test_combination(gpu, oracle, c):
    harness, lasp, si = gpu
    say(f"case combination {c}")
    N = c["n_sub"] * c["T"]
    cfg = si.Config("combo", B=2, H=c["H"], N=N, D=c["D"], chunk=64, dtype=c["dtype"], seed=c["seed"], Dv=c["Dv"],
                    token_decay=c["token"])
    inp = si.make_inputs(cfg, with_states=c["states"])
    rng = np.random.default_rng(c["seed"] + 1)
    if c["token"]:
        inp.log_g = np.log(rng.uniform(0.8, 1.0, (2, c["H"], N))).astype(np.float32)
    else:
        inp.decay = rng.uniform(0.85, 1.0, c["H"]).astype(np.float32)
    G = c["G"]
    if G > 1:   # K/V heads shared by groups of G query heads
        inp.k, inp.v = np.ascontiguousarray(inp.k[:, ::G]), np.ascontiguousarray(inp.v[:, ::G])
    got = harness.run_gpu(inp, T=c["T"], segments=c["segments"], norm_eps=EPS if c["norm"] else None)

    k, v = oracle.group_expand(inp.k, G), oracle.group_expand(inp.v, G)
    lg = inp.log_g if c["token"] else None
    dec = None if c["token"] else inp.decay
    o, kvo = oracle.dims_fwd_brute(inp.q, k, v, dec, inp.kv_in, log_g=lg)
    ref = dict(kv_out=kvo)
    do = inp.dout
    if c["norm"]:
        y, rstd = oracle.norm_fwd(o, EPS)
        do = oracle.norm_bwd(inp.dout, y, rstd)
        ref.update(out=y, rstd=rstd)
    else:
        ref.update(out=o)
    res = oracle.dims_bwd_brute(inp.q, k, v, do, dec, inp.kv_in, inp.dkv_out, log_g=lg)
    ref.update(dq=res[0], dk=oracle.group_reduce(res[1], G), dv=oracle.group_reduce(res[2], G), dkv_in=res[-1])
    if c["token"]:
        ref["dlog_g"] = res[3]
    for name, r in ref.items():
        assert got[name].shape == r.shape, (name, got[name].shape, r.shape)
        emax, efro = harness.rel_errors(got[name], r)
        say(f"  combo {name:7s} max-rel {emax:.3e} fro-rel {efro:.3e}")
        assert np.isfinite(emax) and emax <= TOL[c["dtype"]] and efro <= TOL[c["dtype"]], (name, emax, efro)
