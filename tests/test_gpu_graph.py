"""The T-loop captured in a HIP graph: every replay must give what the eager loop gives on the
same buffers, also after the inputs were changed in place and with eager work between replays."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_graph_replays_match_eager():
    import torch
    from paper_2404_02882_amd import harness, synth_inputs as si
    from paper_2404_02882_amd.sequence import GraphedStep, LaspSequence

    cfg = si.Config("graph", B=2, H=4, N=2048, D=64, chunk=64, dtype="bf16", T=4, seed=77)
    dev = "cuda"
    T = cfg.T
    seq = LaspSequence(cfg.B, cfg.H, cfg.N, cfg.D, cfg.chunk, torch.bfloat16, T=T, device=dev)
    decay = torch.from_numpy(si.decay_schedule(cfg.H)).to(dev)

    def upload(seed):
        inp = si.make_inputs(cfg, seed=seed)
        return [harness.shards(x, T, cfg.dtype, dev) for x in (inp.q, inp.k, inp.v, inp.dout)]

    q, k, v, do = upload(1)
    out, dq, dk, dv = ([torch.zeros_like(x) for x in q] for _ in range(4))
    step = GraphedStep(seq, dict(q=q, k=k, v=v, decay=decay, out=out),
                       dict(q=q, k=k, v=v, dout=do, decay=decay, dq=dq, dk=dk, dv=dv))

    def eager_reference():
        ref_seq = LaspSequence(cfg.B, cfg.H, cfg.N, cfg.D, cfg.chunk, torch.bfloat16, T=T, device=dev)
        o2, dq2, dk2, dv2 = ([torch.zeros_like(x) for x in q] for _ in range(4))
        kv = ref_seq.forward(q, k, v, decay, o2).clone()
        dkv = ref_seq.backward(q, k, v, do, decay, dq2, dk2, dv2).clone()
        torch.cuda.synchronize()
        return o2, dq2, dk2, dv2, kv, dkv

    for rep, seed in enumerate((1, 2, 3, 2)):
        if rep > 0:   # new data in place: the graph keeps reading the same buffers
            for dst, src in zip((q, k, v, do), upload(seed)):
                for d, s in zip(dst, src):
                    d.copy_(s)
        for t in out + dq + dk + dv:
            t.fill_(float("nan"))
        step.replay()
        torch.cuda.synchronize()
        o2, dq2, dk2, dv2, kv, dkv = eager_reference()   # eager work between replays
        for name, got, ref in (("out", out, o2), ("dq", dq, dq2), ("dk", dk, dk2), ("dv", dv, dv2)):
            for g, r in zip(got, ref):
                assert torch.equal(g, r), (rep, name)
        assert torch.equal(seq.kv[T], kv) and torch.equal(seq.dkv[0], dkv), rep


def test_bidirectional_graph_replays_match_eager():
    import torch
    from paper_2404_02882_amd import harness, synth_inputs as si
    from paper_2404_02882_amd.sequence import BidirSequence, GraphedStep

    cfg = si.Config("bgraph", B=2, H=4, N=1500, D=128, chunk=128, dtype="bf16", seed=78, decay="one", bidirectional=True)
    dev = "cuda"
    lengths = [700, 800]
    edges = [0, 700, 1500]
    seq = BidirSequence(cfg.B, cfg.H, lengths, cfg.D, cfg.chunk, torch.bfloat16, device=dev)

    def upload(seed):
        inp = si.make_inputs(cfg, seed=seed)
        return [[harness.to_device(x[:, :, a:b], cfg.dtype, dev) for a, b in zip(edges[:-1], edges[1:])]
                for x in (inp.q, inp.k, inp.v, inp.dout)]

    q, k, v, do = upload(1)
    out, dq, dk, dv = ([torch.zeros_like(x) for x in q] for _ in range(4))
    step = GraphedStep(seq, dict(q=q, k=k, v=v, out=out), dict(q=q, k=k, v=v, dout=do, dq=dq, dk=dk, dv=dv))

    def eager_reference():
        ref_seq = BidirSequence(cfg.B, cfg.H, lengths, cfg.D, cfg.chunk, torch.bfloat16, device=dev)
        o2, dq2, dk2, dv2 = ([torch.zeros_like(x) for x in q] for _ in range(4))
        kv = ref_seq.forward(q, k, v, o2).clone()
        dkv = ref_seq.backward(q, k, v, do, dq2, dk2, dv2).clone()
        torch.cuda.synchronize()
        return o2, dq2, dk2, dv2, kv, dkv

    for rep, seed in enumerate((1, 2, 3, 2)):
        if rep > 0:
            for dst, src in zip((q, k, v, do), upload(seed)):
                for d, s in zip(dst, src):
                    d.copy_(s)
        for t in out + dq + dk + dv + [seq.kv, seq.dkv]:
            t.fill_(float("nan"))
        step.replay()
        torch.cuda.synchronize()
        o2, dq2, dk2, dv2, kv, dkv = eager_reference()
        for name, got, ref in (("out", out, o2), ("dq", dq, dq2), ("dk", dk, dk2), ("dv", dv, dv2)):
            for g, r in zip(got, ref):
                assert torch.equal(g, r), (rep, name)
        assert torch.equal(seq.kv, kv) and torch.equal(seq.dkv, dkv), rep
