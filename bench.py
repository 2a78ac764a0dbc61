#!/usr/bin/env python3
"""Benchmark of the LASP hot path on one MI355X.

One step = one forward + one backward pass of chunked causal linear attention
over one batch of synthetic input already resident in HBM (config c3:
bf16, B=1, H=16, N=32768, d=128, chunk=128). Prints ONE JSON line:
tokens/s of the whole step (timed as replays of one HIP graph of the step's
C-ABI calls, after a pre-warm by wall time; --eager times the eager launches),
the roofline of the dominant kernel from HIP events recorded on the launch
stream around every kernel (in an eager pass of the same steps right after the
timed replays, since events cannot be captured in the graph; with --eager
inside the timed region itself), and the CPU oracle timed on a bounded sample
of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 MFMA rate

# kernel name fragments of the rows of profiles/<config>_fwd_bwd_kernels.md that hold the HBM traffic per launch
PROFILE_ROW = {"fwd_walk": "k_fwd<", "bwd_walk": "k_bwd", "fwd_local": ("k_local<", ", false, "), "bwd_local": ("k_local<", ", true, "),
               "bwd_apply": "backward (3 products)", "fwd_apply": "forward (1 product)", "state_reduce": "k_bidir_reduce<"}


def traffic_from_profile(config, kernel):
    """HBM bytes one launch of `kernel` moves, read from the committed rocprofv3 summary of this config
    (table 'HBM traffic per launch': read MiB + written MiB, already scaled by the plain-copy calibration).
    Returns (bytes, path) or (None, None) when the summary or the row is missing."""
    import re
    path = os.path.join(ROOT, "profiles", f"{config}_fwd_bwd_kernels.md")
    if not os.path.exists(path):
        return None, None
    want = PROFILE_ROW.get(kernel)
    want = (want,) if isinstance(want, str) else want
    in_table = False
    for line in open(path):
        if line.startswith("## HBM traffic per launch"):
            in_table = True
        if not in_table or not line.startswith("| `"):
            continue
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        name = cells[0]
        # the local passes differ in the BWD template argument (4th); the walks in the kernel name
        if kernel in ("fwd_local", "bwd_local"):
            m = re.match(r"`lasp::k_local<[^,]+, \d+, \d+, (true|false)", name)
            if not m or (m.group(1) == "true") != (kernel == "bwd_local"):
                continue
        elif not all(w in name for w in want) or "k_bwd" in want[0] and "k_bidir" in name:
            continue
        try:
            return int((float(cells[2]) + float(cells[4])) * 2**20), os.path.relpath(path, ROOT)
        except (IndexError, ValueError):
            return None, None
    return None, None


def flop_counts(B, H, N, dk, dv, chunk, tile):
    """Flops of one forward + backward step per the three conventions reported (d_k, d_v; per token-head, times B H N).
    algorithmic: Alg. 2 / Alg. 3 as printed, full C x C tiles at the configured chunk C:
        forward  scores 2 C dk + PV 2 C dv + Q KV 2 dk dv + state update 2 dk dv
        backward scores S, dS 2 C dk + 2 C dv, intra dQ, dK 2 * 2 C dk, intra dV 2 C dv, inter dQ, dK, dV and the dKV update 4 * 2 dk dv
        (= 14 C d + 12 d^2 at dk = dv = d)
    causal_minimal: the same with only the 32 x 32 blocks of a chunk that the causal mask leaves non-zero
    issued: what the kernels execute: tiles of `tile` tokens with the all-zero 32 x 32 blocks skipped, the local passes
        (2 dk dv each, forward and backward), the dKV update done by both wave groups of the backward walk (+ 2 dk dv) and
        the O tile's dQ reaching across the pair (scores and product over the E tile's keys, averaged over both tiles)."""
    th = B * H * N
    intra_f = lambda c: c * (2 * dk + 2 * dv)                 # forward intra terms per token at tile length c
    intra_b = lambda c: c * (2 * dk + 2 * dv + 4 * dk + 2 * dv)  # backward intra terms
    inter = 12 * dk * dv
    nb = lambda c: max(c // 32, 1)
    tri = lambda c: (nb(c) + 1) / (2 * nb(c))                 # share of 32 x 32 blocks on or below the diagonal
    alg = th * (intra_f(chunk) + intra_b(chunk) + inter)
    causal = th * ((intra_f(chunk) + intra_b(chunk)) * tri(chunk) + inter)
    issued = th * ((intra_f(tile) + intra_b(tile)) * tri(tile) + inter + 2 * 2 * dk * dv + 2 * dk * dv
                   + (tile * (2 * dv + 2 * dk)) / 2)
    return {"algorithmic": alg, "causal_minimal": causal, "issued": issued}


class HeadGroups:
    """The heads of a B = 1 workload cut into G groups that are processed one after the other, each with its own
    sequence object (own state caches and workspace). A head slice of a [1, H, ...] tensor is contiguous, so the
    groups run the same library calls on views of the same buffers. forward / backward take the keyword arguments
    of LaspSequence and slice every tensor that has a head axis."""

    def __init__(self, groups, make_sequence, H):
        assert H % groups == 0, "the groups must divide the heads"
        self.hg = H // groups
        self.seqs = [make_sequence(self.hg) for _ in range(groups)]
        self.shape = self.seqs[0].shape

    def _slice(self, x, g):
        import torch
        lo, hi = g * self.hg, (g + 1) * self.hg
        if isinstance(x, (list, tuple)):
            return [self._slice(t, g) for t in x]
        if isinstance(x, torch.Tensor):
            return x[lo:hi] if x.dim() == 1 else x[:, lo:hi]
        return x

    def forward(self, **kw):
        for g, seq in enumerate(self.seqs):
            seq.forward(**{n: self._slice(x, g) for n, x in kw.items()})

    def backward(self, **kw):
        for g, seq in enumerate(self.seqs):
            seq.backward(**{n: self._slice(x, g) for n, x in kw.items()})

    def cache_bytes(self):
        return sum(seq.cache_bytes() for seq in self.seqs)

    def workspace_bytes(self):
        return sum(seq.workspace_bytes() for seq in self.seqs)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="c3", help="named workload (c3 is the headline; g3 = c3 with a decay per token, n3 = c3 with the fused Norm, b3 = c3 without mask and decay, m3 = c3 with d_k = 64, d_v = 128)")
    ap.add_argument("--segments", type=int, default=0)
    ap.add_argument("--sub-sequences", type=int, default=0,
                    help="process the sequence as this many sub-sequences with the state handed over (0 = the config's T)")
    ap.add_argument("--eager", action="store_true",
                    help="time the step as eager launches (one C-ABI call per sub-sequence and pass) instead of replays of "
                         "one HIP graph of the same calls; the per-kernel HIP events then lie inside the timed region")
    ap.add_argument("--graph", action="store_true", help="(the default; kept for older command lines)")
    ap.add_argument("--prewarm-seconds", type=float, default=1.0,
                    help="untimed steps run for this long before the counted warm-up, so that a cold device is at its "
                         "steady clocks when the short timed region starts")
    ap.add_argument("--head-groups", type=int, default=1,
                    help="run the step as this many independent groups of heads, one after the other (local pass, scan "
                         "and walk of a group back to back, so that the walk re-reads what the local pass of the same "
                         "few heads just read); needs B = 1. An experiment on the last-level cache, not the default")
    ap.add_argument("--recompute", action="store_true",
                    help="keep no state cache between the passes: every backward call rebuilds the states of its "
                         "sub-sequence (Sec. 3.4: recomputation instead of caching)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=32768)
    ap.add_argument("--copy-mib", type=int, default=1024,
                    help="size of the plain device-to-device copy timed for reference (0 = skip); under "
                         "rocprofv3 --pmc its known size calibrates FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the ring of ranks is a loop over sub-sequences on one "
              "device); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2404_02882_amd import harness, lasp, synth_inputs as si
    from paper_2404_02882_amd.sequence import GraphedStep, LaspSequence

    cfg = si.CONFIGS[args.config]
    if args.sub_sequences > 0:
        import dataclasses
        cfg = dataclasses.replace(cfg, T=args.sub_sequences)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if cfg.bidirectional:
        return bench_bidirectional(args, cfg, dev)
    inp = si.make_inputs(cfg)
    B, H, N, D, T = cfg.B, cfg.H, cfg.N, cfg.D, cfg.T
    dt = harness.TORCH_DTYPE[cfg.dtype]
    token = cfg.token_decay
    norm = cfg.norm_eps is not None
    dk_, dv_ = D, cfg.Dv or D   # key and value dimensions
    torch.cuda.reset_peak_memory_stats()
    make_sequence = lambda heads: LaspSequence(B, heads, N, D, cfg.chunk, dt, T=T, segments=args.segments, device=dev,
                                               token_decay=token, norm_eps=cfg.norm_eps, Dv=cfg.Dv, recompute=args.recompute)
    if args.head_groups > 1:
        if B != 1:
            sys.exit("bench.py: --head-groups needs a workload with B = 1 (a head slice must be contiguous)")
        seq = HeadGroups(args.head_groups, make_sequence, H)
    else:
        seq = make_sequence(H)
    q, k, v, do = (harness.shards(x, T, cfg.dtype, dev) for x in (inp.q, inp.k, inp.v, inp.dout))
    if token:   # a decay per token: log g shards [B,H,N/T] in, dlog_g shards out
        n = N // T
        decay = [torch.from_numpy(np.ascontiguousarray(inp.log_g[:, :, t * n:(t + 1) * n])).to(dev) for t in range(T)]
        dlg = [torch.empty_like(x) for x in decay]
    else:
        decay = torch.from_numpy(inp.decay).to(dev)
        dlg = None
    out, dq, dk, dv = ([torch.empty_like(x) for x in y] for y in (v, q, k, v))
    rstd = [torch.empty(B, H, N // T, dtype=torch.float32, device=dev) for _ in range(T)] if norm else None
    tile = lasp.tile_tokens(seq.shape)
    nseg = lasp.num_segments(seq.shape)
    fwd_kw = dict(q=q, k=k, v=v, decay=decay, out=out, rstd=rstd)
    bwd_kw = dict(q=q, k=k, v=v, dout=do, decay=decay, dq=dq, dk=dk, dv=dv, dlog_g=dlg, out=out, rstd=rstd)

    def step():
        seq.forward(**fwd_kw)
        seq.backward(**bwd_kw)

    def timed(fn, n):
        """wall-clock milliseconds per call of n calls, bracketed by device synchronisation"""
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n

    # untimed: everything host-side first (graph capture leaves the device idle), then the step itself for
    # `prewarm_seconds` so that a cold device is at its steady clocks, then the counted warm-up
    step()
    graphed = GraphedStep(seq, fwd_kw, bwd_kw)
    fwd_only, bwd_only = GraphedStep(seq, fwd_kw, None), GraphedStep(seq, None, bwd_kw)
    run = step if args.eager else graphed.replay
    t_end = time.perf_counter() + max(args.prewarm_seconds, 0.0)
    while time.perf_counter() < t_end:
        for _ in range(20):
            run()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        run()
    # ---- the timed region: exactly `steps` steps ----
    if args.eager:
        lasp.profile_begin(args.steps * T * args.head_groups)
    ms_per_step = timed(run, args.steps)
    if args.eager:
        kernel_ms, nf, nb_calls = lasp.profile_end()
        eager_ms, graph_ms = ms_per_step, timed(graphed.replay, args.steps)
    else:
        # per-kernel times: HIP events are not captured in a graph, so they come from an eager pass of the same steps
        lasp.profile_begin(args.steps * T * args.head_groups)
        eager_ms = timed(step, args.steps)
        kernel_ms, nf, nb_calls = lasp.profile_end()
        graph_ms = ms_per_step
    tokens_per_s = B * N / (ms_per_step * 1e-3)
    # spread of single steps (HIP events around every step, a separate pass) and the two passes on their own
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    evs[0].record()
    for i in range(args.steps):
        run()
        evs[i + 1].record()
    torch.cuda.synchronize()
    per_step = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(args.steps))
    for g in (fwd_only, bwd_only):
        for _ in range(3):
            g.replay()
    fwd_ms, bwd_ms = timed(fwd_only.replay, args.steps), timed(bwd_only.replay, args.steps)
    peak_mem = torch.cuda.max_memory_allocated()

    # ---- roofline of the dominant kernel (largest share of the step) ----
    tok_heads_per_launch = B * (H // args.head_groups) * (N // T)
    esz = 2 if cfg.dtype == "bf16" else 4
    per_launch_ms = {"fwd_local": kernel_ms["fwd"][0] / nf, "fwd_scan": kernel_ms["fwd"][1] / nf,
                     "fwd_walk": kernel_ms["fwd"][2] / nf, "bwd_local": kernel_ms["bwd"][0] / nb_calls,
                     "bwd_scan": kernel_ms["bwd"][1] / nb_calls, "bwd_walk": kernel_ms["bwd"][2] / nb_calls}
    # algorithmic (compulsory) HBM bytes per token-head: forward walk reads q,k,v and
    # writes o; backward walk reads q,k,v,do and writes dq,dk,dv; local passes read two tensors.
    # With a decay per token every kernel also reads log g (4 B per token-head); dlog_g is written by a
    # separate small kernel.
    # With the fused Norm the forward walk also writes rstd (4 B) and both backward kernels also read the
    # normalised output and rstd (dO is rebuilt from dY on the fly).
    gb = 4 if token else 0
    nb = dv_ * esz + 4 if norm else 0   # the normalised output row and rstd
    alg_bytes = {"fwd_walk": (2 * dk_ + 2 * dv_) * esz + gb + (4 if norm else 0),
                 "bwd_walk": (4 * dk_ + 3 * dv_) * esz + gb + nb,
                 "fwd_local": (dk_ + dv_) * esz + gb, "bwd_local": (dk_ + dv_) * esz + gb + nb}
    dominant = max(("fwd_walk", "bwd_walk", "fwd_local", "bwd_local"), key=lambda n: per_launch_ms[n])
    dom_bytes = alg_bytes[dominant] * tok_heads_per_launch
    achieved = dom_bytes / (per_launch_ms[dominant] * 1e-3) / 1e9
    as_profiled = args.segments == 0 and args.sub_sequences == 0 and args.head_groups == 1   # the committed summaries' launch shape
    traffic, traffic_src = traffic_from_profile(args.config, dominant) if as_profiled else (None, None)
    roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic, "traffic_source": traffic_src,
                "algorithmic_bytes_per_launch": dom_bytes,
                "avg_launch_ms": round(per_launch_ms[dominant], 4),
                "kernel_ms_per_launch": {n: round(x, 4) for n, x in per_launch_ms.items()},
                "kernel_times_from": "HIP events on the launch stream around every kernel of "
                                     + ("the timed eager steps" if args.eager else f"{args.steps} eager steps run right after the timed graph replays")}

    # whole-step figures against both roofs. Flops: see flop_counts(); `chunk` is validated but does not select the
    # kernels' tile (64 tokens for bfloat16, 32 for float), so the algorithmic count at C = chunk is not what is issued.
    flops = flop_counts(B, H, N, dk_, dv_, cfg.chunk, tile)
    min_bytes_step = ((6 * dk_ + 5 * dv_) * esz + 3 * gb + (dv_ * esz + 8 if norm else 0)) * B * H * N
    step_s = ms_per_step * 1e-3
    tf = lambda f: round(f / step_s / 1e12, 2)
    extra = {"timed_as": "eager launches" if args.eager else "hip graph replay",
             "eager_ms_per_step": round(eager_ms, 4), "hip_graph_replay_ms_per_step": round(graph_ms, 4),
             "step_ms_median": round(per_step[len(per_step) // 2], 4), "step_ms_min": round(per_step[0], 4),
             "step_ms_max": round(per_step[-1], 4),
             "forward_only_ms": round(fwd_ms, 4), "backward_only_ms": round(bwd_ms, 4),
             "algorithmic_tflops": tf(flops["algorithmic"]),
             "mfma_bf16_peak_frac": round(flops["algorithmic"] / step_s / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
             "causal_minimal_tflops": tf(flops["causal_minimal"]),
             "causal_minimal_mfma_frac": round(flops["causal_minimal"] / step_s / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
             "issued_tflops": tf(flops["issued"]),
             "issued_mfma_frac": round(flops["issued"] / step_s / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
             "flops_per_step": {n: int(x) for n, x in flops.items()},
             "min_hbm_bytes_per_step": min_bytes_step,
             "step_hbm_frac_at_min_bytes": round(min_bytes_step / step_s / 1e9 / HBM_PEAK_GBS, 4)}

    copy = copy_reference(args, dev)

    # ---- CPU oracle on a bounded sample of the same workload ----
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import lasp_oracle
        n_s = min(args.cpu_sample_tokens, N)
        n_s -= n_s % cfg.chunk

        def oracle_pass(n_tok):
            sl = slice(0, n_tok)
            a = [np.ascontiguousarray(x[:, :, sl], dtype=np.float64) for x in (inp.q, inp.k, inp.v, inp.dout)]
            if dk_ != dv_:   # the C oracle has one head dimension: the narrower side gets zero columns (changes no value)
                dmax = max(dk_, dv_)
                a = [np.pad(x, ((0, 0), (0, 0), (0, 0), (0, dmax - x.shape[3]))) for x in a]
            c0 = time.perf_counter()
            if norm:
                o, _ = lasp_oracle.fwd_chunked(a[0], a[1], a[2], inp.decay, cfg.chunk)
                y, rs = lasp_oracle.norm_fwd(o, cfg.norm_eps)
                lasp_oracle.bwd_chunked(a[0], a[1], a[2], lasp_oracle.norm_bwd(a[3], y, rs), inp.decay, cfg.chunk)
            elif token:
                lg = np.ascontiguousarray(inp.log_g[:, :, sl], dtype=np.float64)
                lasp_oracle.gated_fwd_chunked(a[0], a[1], a[2], lg, cfg.chunk)
                lasp_oracle.gated_bwd_chunked(a[0], a[1], a[2], a[3], lg, cfg.chunk)
            else:
                lasp_oracle.fwd_chunked(a[0], a[1], a[2], inp.decay, cfg.chunk)
                lasp_oracle.bwd_chunked(a[0], a[1], a[2], a[3], inp.decay, cfg.chunk)
            return time.perf_counter() - c0

        cores = lasp_oracle.num_threads()
        secs = oracle_pass(n_s)
        # the same oracle on one core, on a shorter prefix (its cost is linear in the tokens)
        n_1 = max(cfg.chunk, min(n_s, 4096) // cfg.chunk * cfg.chunk)
        lasp_oracle.set_num_threads(1)
        secs_1 = oracle_pass(n_1)
        lasp_oracle.set_num_threads(cores)
        # the definition itself (brute force, quadratic in the tokens) on the small named workload c2, and what
        # that rate extrapolates to for this workload (cost ~ B H N^2 d): an extrapolation, not a measurement
        c2 = si.CONFIGS["c2"]
        i2 = si.make_inputs(c2)
        b0 = time.perf_counter()
        lasp_oracle.fwd_brute(i2.q, i2.k, i2.v, i2.decay)
        lasp_oracle.bwd_brute(i2.q, i2.k, i2.v, i2.dout, i2.decay)
        secs_b = time.perf_counter() - b0
        scale = (B * H * N * N * max(dk_, dv_)) / (c2.B * c2.H * c2.N * c2.N * c2.D)
        cpu = {"value": round(B * n_s / secs, 1), "unit": "tokens/s", "cores": cores,
               "kind": "oracle",
               "sample": f"chunked fp64 oracle (Alg. 2 + Alg. 3), fwd+bwd, first {n_s} of {N} tokens of all "
                         f"{B * H} heads, {secs:.1f} s"
                         + (f"; run at d = {max(dk_, dv_)} with zero columns on the narrower side" if dk_ != dv_ else ""),
               "one_core": {"value": round(B * n_1 / secs_1, 1), "unit": "tokens/s", "cores": 1,
                            "sample": f"the same oracle with one thread, first {n_1} tokens of all {B * H} heads, {secs_1:.1f} s"},
               "brute_force": {"measured_seconds": round(secs_b, 2), "cores": cores,
                               "sample": f"fp64 brute force (the definition), fwd+bwd, all of c2 (B={c2.B} H={c2.H} N={c2.N} d={c2.D})",
                               "extrapolated_seconds_this_workload": round(secs_b * scale, 1),
                               "extrapolation": "measured seconds x (B H N^2 d of this workload / of c2); not a measurement"}}

    line = {"metric": "fwd+bwd tokens/sec, chunked causal linear attention with decay (LASP per-device hot path)"
                      + (", decay per token" if token else "") + (", normalised output" if norm else ""),
            "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
            "config": {"workload": f"{cfg.name}: B={B} H={H} N={N} " + (f"d_k={dk_} d_v={dv_}" if dk_ != dv_ else f"d={D}")
                                   + f" chunk={cfg.chunk} {cfg.dtype}, "
                                   f"T={T} sub-sequence(s), fwd+bwd" + (", decay per token (log_g in, dlog_g out)" if token else "")
                                   + (f", output RMS-normalised per row (eps {cfg.norm_eps})" if norm else ""),
                       "tile_tokens": tile, "chunk_selects_tile": False, "segments_per_head": nseg,
                       "hip_graph": not args.eager, "prewarm_seconds": args.prewarm_seconds,
                       "state_cache": "none (states rebuilt in the backward pass)" if args.recompute else "kept between the passes",
                       "state_cache_bytes": seq.cache_bytes(), "workspace_bytes": seq.workspace_bytes(), "head_groups": args.head_groups,
                       "peak_device_memory_bytes": int(peak_mem)},
            "roofline": roofline, "whole_step": extra, "copy_reference": copy, "cpu_baseline": cpu}
    print(json.dumps(line), flush=True)


def copy_reference(args, dev):
    """Plain device-to-device copy of known size: measured HBM copy bandwidth (and counter calibration)."""
    import torch
    if args.copy_mib <= 0:
        return None
    n = args.copy_mib * (1 << 20)
    src = torch.empty(n, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    copy_ms = e0.elapsed_time(e1) / 10
    return {"bytes_read": n, "bytes_written": n, "ms": round(copy_ms, 4),
            "gbs_read_plus_write": round(2 * n / (copy_ms * 1e-3) / 1e9, 1)}


def bench_bidirectional(args, cfg, dev):
    """One step = forward + backward of the unmasked attention O = Q (K^T V): per sub-sequence the state
    reduction on (K, V), then the output product; backward the reduction on (Q, dO), then the three
    gradient products in one launch."""
    import numpy as np
    import torch
    from paper_2404_02882_amd import harness, lasp, synth_inputs as si
    from paper_2404_02882_amd.sequence import BidirSequence

    inp = si.make_inputs(cfg)
    B, H, N, D, T = cfg.B, cfg.H, cfg.N, cfg.D, cfg.T
    dt = harness.TORCH_DTYPE[cfg.dtype]
    lengths = [N // T] * T
    seq = BidirSequence(B, H, lengths, D, cfg.chunk, dt, segments=args.segments, device=dev)
    q, k, v, do = (harness.shards(x, T, cfg.dtype, dev) for x in (inp.q, inp.k, inp.v, inp.dout))
    out, dq, dk, dv = ([torch.empty_like(x) for x in q] for _ in range(4))

    def step():
        seq.forward(q, k, v, out)
        seq.backward(q, k, v, do, dq, dk, dv)

    def timed(fn, n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n

    # untimed: graph capture first (it leaves the device idle), then the step itself for `prewarm_seconds`
    # so that a cold device is at its steady clocks, then the counted warm-up
    from paper_2404_02882_amd.sequence import GraphedStep
    step()
    graphed = GraphedStep(seq, dict(q=q, k=k, v=v, out=out), dict(q=q, k=k, v=v, dout=do, dq=dq, dk=dk, dv=dv))
    run = step if args.eager else graphed.replay
    t_end = time.perf_counter() + max(args.prewarm_seconds, 0.0)
    while time.perf_counter() < t_end:
        for _ in range(20):
            run()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        run()
    if args.eager:
        lasp.profile_begin(args.steps * 3 * T)
    ms_per_step = timed(run, args.steps)     # the timed region: exactly `steps` steps
    if args.eager:
        kernel_ms, nf, nb = lasp.profile_end()
        eager_ms, graph_ms = ms_per_step, timed(graphed.replay, args.steps)
    else:       # per-kernel HIP events from an eager pass of the same steps (events are not captured in a graph)
        lasp.profile_begin(args.steps * 3 * T)
        eager_ms = timed(step, args.steps)
        kernel_ms, nf, nb = lasp.profile_end()
        graph_ms = ms_per_step
    tokens_per_s = B * N / (ms_per_step * 1e-3)

    # forward-kind records: 2T state calls and T output calls per step; backward-kind: T calls per step
    launches = args.steps * T
    per_launch_ms = {"state_reduce": kernel_ms["fwd"][0] / (2 * launches), "state_sum": kernel_ms["fwd"][1] / (2 * launches),
                     "fwd_apply": kernel_ms["fwd"][2] / launches, "bwd_apply": kernel_ms["bwd"][2] / launches}
    assert nf == 3 * launches and nb == launches, (nf, nb)
    esz = 2 if cfg.dtype == "bf16" else 4
    tok_heads_per_launch = B * H * (N // T)
    # compulsory HBM bytes per token-head: the reduction reads two tensors; the output product reads q and
    # writes o; the gradient products read dO, V, K and write dQ, dK, dV
    alg_bytes = {"state_reduce": 2 * D * esz, "fwd_apply": 2 * D * esz, "bwd_apply": 6 * D * esz}
    dominant = max(alg_bytes, key=lambda n: per_launch_ms[n])
    dom_bytes = alg_bytes[dominant] * tok_heads_per_launch
    achieved = dom_bytes / (per_launch_ms[dominant] * 1e-3) / 1e9
    roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic_from_profile(args.config, dominant)[0] if args.segments == 0 else None,
                "traffic_source": traffic_from_profile(args.config, dominant)[1] if args.segments == 0 else None,
                "algorithmic_bytes_per_launch": dom_bytes,
                "avg_launch_ms": round(per_launch_ms[dominant], 4),
                "kernel_ms_per_launch": {n: round(x, 4) for n, x in per_launch_ms.items()}}
    flops_step = 12 * D * D * B * H * N      # two reductions and four products of 2 d^2 each per token-head
    min_bytes_step = 11 * D * esz * B * H * N
    step_s = ms_per_step * 1e-3
    extra = {"timed_as": "eager launches" if args.eager else "hip graph replay",
             "eager_ms_per_step": round(eager_ms, 4), "hip_graph_replay_ms_per_step": round(graph_ms, 4),
             "algorithmic_tflops": round(flops_step / step_s / 1e12, 2),
             "mfma_bf16_peak_frac": round(flops_step / step_s / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
             "min_hbm_bytes_per_step": min_bytes_step,
             "step_hbm_frac_at_min_bytes": round(min_bytes_step / step_s / 1e9 / HBM_PEAK_GBS, 4)}
    copy = copy_reference(args, dev)

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import lasp_oracle
        n_s = min(args.cpu_sample_tokens, N, 8192)   # the definition is quadratic in the tokens
        a = [np.ascontiguousarray(x[:, :, :n_s], dtype=np.float64) for x in (inp.q, inp.k, inp.v, inp.dout)]
        c0 = time.perf_counter()
        lasp_oracle.bidir_fwd_left(a[0], a[1], a[2])
        lasp_oracle.bidir_bwd_left(a[0], a[1], a[2], a[3])
        c1 = time.perf_counter()
        cpu = {"value": round(B * n_s / (c1 - c0), 1), "unit": "tokens/s", "cores": os.cpu_count(), "kind": "oracle",
               "sample": f"fp64 oracle, the definition O = (Q K^T) V with its N x N scores (quadratic: the rate falls "
                         f"with N), fwd+bwd, a {n_s}-token sequence of all {B * H} heads, {c1 - c0:.1f} s; numpy "
                         f"matmul on the host's BLAS threads"}

    line = {"metric": "fwd+bwd tokens/sec, bidirectional (unmasked) linear attention O = Q (K^T V)",
            "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
            "config": {"workload": f"{cfg.name}: B={B} H={H} N={N} d={D} {cfg.dtype}, T={T} sub-sequence(s), fwd+bwd, "
                                   f"no mask, no decay",
                       "partial_states_per_head": lasp.bidir_scratch_bytes(seq.shapes[0]) // (B * H * D * D * 4),
                       "hip_graph": not args.eager, "prewarm_seconds": args.prewarm_seconds},
            "roofline": roofline, "whole_step": extra, "copy_reference": copy, "cpu_baseline": cpu}
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
