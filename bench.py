#!/usr/bin/env python3
"""Benchmark of the LASP hot path on one MI355X.

One step = one forward + one backward pass of chunked causal linear attention
over one batch of synthetic input already resident in HBM (config c3:
bf16, B=1, H=16, N=32768, d=128, chunk=128). Prints ONE JSON line:
tokens/s of the whole step, the roofline of the dominant kernel measured with
HIP events inside the timed region, and the CPU oracle timed on a bounded
sample of the same workload.
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

# HBM bytes per launch from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised in
# profiles/<config>_fwd_bwd_kernels.md (read + written MiB, scaled by the plain-copy calibration:
# FETCH_SIZE x 2.000, WRITE_SIZE x 1.000), for the default launch configuration. Other configs: None.
_MIB = 2**20
MEASURED_TRAFFIC_BYTES = {
    "c3": {"fwd_walk": int((416.2 + 258.1) * _MIB), "bwd_walk": int((659.1 + 385.0) * _MIB),
           "fwd_local": int((248.1 + 31.0) * _MIB), "bwd_local": int((240.1 + 15.0) * _MIB)},
    "g3": {"fwd_walk": int((418.2 + 257.4) * _MIB), "bwd_walk": int((659.4 + 387.0) * _MIB),
           "fwd_local": int((250.1 + 31.0) * _MIB), "bwd_local": int((242.0 + 15.0) * _MIB)},
    "n3": {"fwd_walk": int((416.2 + 260.6) * _MIB), "bwd_walk": int((789.1 + 385.0) * _MIB),
           "fwd_local": int((248.1 + 31.0) * _MIB), "bwd_local": int((362.0 + 15.0) * _MIB)},
    "m3": {"fwd_walk": int((288.2 + 256.7) * _MIB), "bwd_walk": int((529.2 + 256.5) * _MIB),
           "fwd_local": int((186.1 + 31.0) * _MIB), "bwd_local": int((180.1 + 15.0) * _MIB)},
    "b3": {"bwd_apply": int((401.8 + 384.0) * _MIB), "fwd_apply": int((136.2 + 128.0) * _MIB),
           "state_reduce": int((256.1 + 16.0) * _MIB)},
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="c3", help="named workload (c3 is the headline; g3 = c3 with a decay per token, n3 = c3 with the fused Norm, b3 = c3 without mask and decay, m3 = c3 with d_k = 64, d_v = 128)")
    ap.add_argument("--segments", type=int, default=0)
    ap.add_argument("--sub-sequences", type=int, default=0,
                    help="process the sequence as this many sub-sequences with the state handed over (0 = the config's T)")
    ap.add_argument("--graph", action="store_true",
                    help="time the step as replays of one HIP graph (pays off when the T-loop is launch-bound); "
                         "per-kernel times then come from a short eager pass before the timed region")
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
    from paper_2404_02882_amd.sequence import LaspSequence

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
    seq = LaspSequence(B, H, N, D, cfg.chunk, dt, T=T, segments=args.segments, device=dev, token_decay=token,
                       norm_eps=cfg.norm_eps, Dv=cfg.Dv)
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

    def step():
        seq.forward(q, k, v, decay, out, rstd=rstd)
        seq.backward(q, k, v, do, decay, dq, dk, dv, dlog_g=dlg, out=out, rstd=rstd)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.graph:
        from paper_2404_02882_amd.sequence import GraphedStep
        lasp.profile_begin(5 * T)          # per-kernel times from an eager pass: events are not captured
        for _ in range(5):
            step()
        torch.cuda.synchronize()
        kernel_ms, nf, nb = lasp.profile_end()
        graphed = GraphedStep(seq, dict(q=q, k=k, v=v, decay=decay, out=out, rstd=rstd),
                              dict(q=q, k=k, v=v, dout=do, decay=decay, dq=dq, dk=dk, dv=dv, dlog_g=dlg, out=out, rstd=rstd))
        for _ in range(args.warmup):
            graphed.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graphed.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    else:
        lasp.profile_begin(args.steps * T)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        kernel_ms, nf, nb = lasp.profile_end()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    graph_ms = None
    if not args.graph:   # for information: the same steps as replays of one HIP graph (not `value`)
        from paper_2404_02882_amd.sequence import GraphedStep
        graphed = GraphedStep(seq, dict(q=q, k=k, v=v, decay=decay, out=out, rstd=rstd),
                              dict(q=q, k=k, v=v, dout=do, decay=decay, dq=dq, dk=dk, dv=dv, dlog_g=dlg, out=out, rstd=rstd))
        for _ in range(args.warmup):
            graphed.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(args.steps):
            graphed.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - g0) * 1e3 / args.steps
    tokens_per_s = B * N / (ms_per_step * 1e-3)

    # ---- roofline of the dominant kernel (largest share of the step) ----
    tok_heads_per_launch = B * H * (N // T)
    esz = 2 if cfg.dtype == "bf16" else 4
    per_launch_ms = {"fwd_local": kernel_ms["fwd"][0] / nf, "fwd_scan": kernel_ms["fwd"][1] / nf,
                     "fwd_walk": kernel_ms["fwd"][2] / nf, "bwd_local": kernel_ms["bwd"][0] / nb,
                     "bwd_scan": kernel_ms["bwd"][1] / nb, "bwd_walk": kernel_ms["bwd"][2] / nb}
    # algorithmic (compulsory) HBM bytes per token-head: forward walk reads q,k,v and
    # writes o; backward walk reads q,k,v,do and writes dq,dk,dv; local passes read two tensors.
    # With a decay per token every kernel also reads log g (4 B per token-head); dlog_g is written by a
    # separate small kernel.
    # With the fused Norm the forward walk also writes rstd (4 B) and both backward kernels also read the
    # normalised output and rstd (dO is rebuilt from dY on the fly).
    gb = 4 if token else 0
    nb = D * esz + 4 if norm else 0
    alg_bytes = {"fwd_walk": (2 * dk_ + 2 * dv_) * esz + gb + (4 if norm else 0),
                 "bwd_walk": (4 * dk_ + 3 * dv_) * esz + gb + nb,
                 "fwd_local": (dk_ + dv_) * esz + gb, "bwd_local": (dk_ + dv_) * esz + gb + nb}
    dominant = max(("fwd_walk", "bwd_walk", "fwd_local", "bwd_local"), key=lambda n: per_launch_ms[n])
    dom_bytes = alg_bytes[dominant] * tok_heads_per_launch
    achieved = dom_bytes / (per_launch_ms[dominant] * 1e-3) / 1e9
    roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": MEASURED_TRAFFIC_BYTES.get(args.config, {}).get(dominant) if args.segments == 0 else None,
                "algorithmic_bytes_per_launch": dom_bytes,
                "avg_launch_ms": round(per_launch_ms[dominant], 4),
                "kernel_ms_per_launch": {n: round(x, 4) for n, x in per_launch_ms.items()}}

    # whole-step figures against both roofs: the chunked algorithm's flops per token-head at the
    # configured chunk length C (intra-chunk 14*C*d, inter-chunk and state updates 12*d*d), not issued
    # flops (the kernels run shorter tiles than C and rebuild half of the cached states)
    flops_step = (cfg.chunk * (8 * dk_ + 6 * dv_) + 12 * dk_ * dv_) * B * H * N   # = 14 C d + 12 d^2 at d_k = d_v = d
    min_bytes_step = ((6 * dk_ + 5 * dv_) * esz + 3 * gb + (D * esz + 8 if norm else 0)) * B * H * N
    step_s = ms_per_step * 1e-3
    extra = {"hip_graph_replay_ms_per_step": round(graph_ms, 4) if graph_ms is not None else None,
             "algorithmic_tflops": round(flops_step / step_s / 1e12, 2),
             "mfma_bf16_peak_frac": round(flops_step / step_s / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
             "min_hbm_bytes_per_step": min_bytes_step,
             "step_hbm_frac_at_min_bytes": round(min_bytes_step / step_s / 1e9 / HBM_PEAK_GBS, 4)}

    copy = copy_reference(args, dev)

    # ---- CPU oracle on a bounded sample of the same workload ----
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import lasp_oracle
        n_s = min(args.cpu_sample_tokens, N)
        n_s -= n_s % cfg.chunk
        sl = slice(0, n_s)
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
        c1 = time.perf_counter()
        cpu = {"value": round(B * n_s / (c1 - c0), 1), "unit": "tokens/s", "cores": lasp_oracle.num_threads(),
               "kind": "oracle",
               "sample": f"chunked fp64 oracle (Alg. 2 + Alg. 3), fwd+bwd, first {n_s} of {N} tokens of all "
                         f"{B * H} heads, {c1 - c0:.1f} s"
                         + (f"; run at d = {max(dk_, dv_)} with zero columns on the narrower side" if dk_ != dv_ else "")}

    line = {"metric": "fwd+bwd tokens/sec, chunked causal linear attention with decay (LASP per-device hot path)"
                      + (", decay per token" if token else "") + (", normalised output" if norm else ""),
            "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
            "config": {"workload": f"{cfg.name}: B={B} H={H} N={N} " + (f"d_k={dk_} d_v={dv_}" if dk_ != dv_ else f"d={D}")
                                   + f" chunk={cfg.chunk} {cfg.dtype}, "
                                   f"T={T} sub-sequence(s), fwd+bwd" + (", decay per token (log_g in, dlog_g out)" if token else "")
                                   + (f", output RMS-normalised per row (eps {cfg.norm_eps})" if norm else ""),
                       "tile_tokens": tile, "segments_per_head": nseg, "hip_graph": bool(args.graph),
                       "state_cache_bytes": seq.cache_bytes()},
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

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    lasp.profile_begin(args.steps * 3 * T)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kernel_ms, nf, nb = lasp.profile_end()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = B * N / (ms_per_step * 1e-3)
    # for information: the same steps as replays of one HIP graph (not `value`)
    from paper_2404_02882_amd.sequence import GraphedStep
    graphed = GraphedStep(seq, dict(q=q, k=k, v=v, out=out), dict(q=q, k=k, v=v, dout=do, dq=dq, dk=dk, dv=dv))
    for _ in range(args.warmup):
        graphed.replay()
    torch.cuda.synchronize()
    g0 = time.perf_counter()
    for _ in range(args.steps):
        graphed.replay()
    torch.cuda.synchronize()
    graph_ms = (time.perf_counter() - g0) * 1e3 / args.steps

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
                "traffic": MEASURED_TRAFFIC_BYTES.get(args.config, {}).get(dominant) if args.segments == 0 else None,
                "algorithmic_bytes_per_launch": dom_bytes,
                "avg_launch_ms": round(per_launch_ms[dominant], 4),
                "kernel_ms_per_launch": {n: round(x, 4) for n, x in per_launch_ms.items()}}
    flops_step = 12 * D * D * B * H * N      # two reductions and four products of 2 d^2 each per token-head
    min_bytes_step = 11 * D * esz * B * H * N
    step_s = ms_per_step * 1e-3
    extra = {"hip_graph_replay_ms_per_step": round(graph_ms, 4),
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
                       "hip_graph": False},
            "roofline": roofline, "whole_step": extra, "copy_reference": copy, "cpu_baseline": cpu}
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
