"""Host-side helpers shared by the GPU tests, the smoke check and bench.py:
upload seeded inputs, run the T-loop through the C-ABI, fetch results.
No attention arithmetic happens here."""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from . import lasp
from .sequence import BidirSequence, LaspSequence
from .synth_inputs import Inputs, bf16_bits

TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def to_device(x: np.ndarray, dtype: str, device="cuda") -> torch.Tensor:
    """Upload values already representable in `dtype` without any further rounding."""
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(device)
    bits = bf16_bits(x)  # exact: x is already a bf16 value
    return torch.from_numpy(bits.view(np.int16)).to(device).view(torch.bfloat16)


def shards(x: np.ndarray, T: int, dtype: str, device="cuda"):
    n = x.shape[2] // T
    return [to_device(x[:, :, t * n:(t + 1) * n], dtype, device) for t in range(T)]


def to_host(ts) -> np.ndarray:
    return np.concatenate([t.float().cpu().numpy().astype(np.float64) for t in ts], axis=2)


def rel_errors(x: np.ndarray, ref: np.ndarray):
    """(max|x-ref| / max|ref|, ||x-ref||_F / ||ref||_F)."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    d = x - ref
    return (float(np.max(np.abs(d)) / max(np.max(np.abs(ref)), 1e-300)),
            float(np.linalg.norm(d.ravel()) / max(np.linalg.norm(ref.ravel()), 1e-300)))


def run_gpu(inp: Inputs, T: int = 1, segments: int = 0, backward: bool = True, chunk: Optional[int] = None,
            device="cuda", norm_eps: Optional[float] = None, recompute: bool = False) -> Dict[str, np.ndarray]:
    """Forward (and backward) of the whole sequence as T sub-sequences; returns float64 host arrays.
    With norm_eps the output is the normalised one, `rstd` is returned too and inp.dout is the gradient
    w.r.t. the normalised output. `recompute`: no state cache; the backward calls rebuild the states."""
    cfg = inp.cfg
    B, H, N, D = inp.q.shape
    kv_heads = inp.k.shape[1] if inp.k.shape[1] != H else 0   # grouped K/V heads: k, v are [B,kv_heads,N,D]
    Dv = inp.v.shape[3] if inp.v.shape[3] != D else 0         # value dimension that differs from the key dimension
    dt = TORCH_DTYPE[cfg.dtype]
    token = inp.log_g is not None
    seq = LaspSequence(B, H, N, D, chunk or cfg.chunk, dt, T=T, segments=segments, device=device,
                       need_backward=backward, token_decay=token, norm_eps=norm_eps, kv_heads=kv_heads, Dv=Dv,
                       recompute=recompute)
    q, k, v = (shards(x, T, cfg.dtype, device) for x in (inp.q, inp.k, inp.v))
    if token:
        n = N // T
        decay = [torch.from_numpy(np.ascontiguousarray(inp.log_g[:, :, t * n:(t + 1) * n])).to(device) for t in range(T)]
    else:
        decay = torch.from_numpy(inp.decay).to(device)
    kv_in = torch.from_numpy(inp.kv_in).to(device) if inp.kv_in is not None else None
    out = [torch.full((B, H, x.shape[2], inp.v.shape[3]), float("nan"), dtype=x.dtype, device=device) for x in q]
    rstd = None
    if norm_eps is not None:
        rstd = [torch.full((B, H, N // T), float("nan"), dtype=torch.float32, device=device) for _ in range(T)]
    kv_out = seq.forward(q, k, v, decay, out, kv_in, rstd=rstd)
    res = {"out": to_host(out), "kv_out": kv_out.cpu().numpy().astype(np.float64)}
    if rstd is not None:
        res["rstd"] = to_host(rstd)
    if backward:
        do = shards(inp.dout, T, cfg.dtype, device)
        g = torch.from_numpy(inp.dkv_out).to(device) if inp.dkv_out is not None else None
        dq = [torch.full_like(x, float("nan")) for x in q]
        dk, dv = ([torch.full_like(x, float("nan")) for x in y] for y in (k, v))
        dlg = [torch.full_like(x, float("nan")) for x in decay] if token else None
        dkv_in = seq.backward(q, k, v, do, decay, dq, dk, dv, g, dlog_g=dlg, out=out, rstd=rstd)
        res.update(dq=to_host(dq), dk=to_host(dk), dv=to_host(dv), dkv_in=dkv_in.cpu().numpy().astype(np.float64))
        if token:
            res["dlog_g"] = to_host(dlg)
    torch.cuda.synchronize()
    return res


def run_gpu_bidir(inp: Inputs, lengths=None, segments: int = 0, backward: bool = True, device="cuda") -> Dict[str, np.ndarray]:
    """Bidirectional attention of the whole sequence cut into sub-sequences of the given lengths
    (default: one); uses q, k, v, dout of `inp` only. Returns float64 host arrays."""
    cfg = inp.cfg
    B, H, N, D = inp.q.shape
    lengths = [N] if lengths is None else list(lengths)
    assert sum(lengths) == N
    edges = np.concatenate([[0], np.cumsum(lengths)])
    cut = lambda x: [to_device(x[:, :, a:b], cfg.dtype, device) for a, b in zip(edges[:-1], edges[1:])]
    seq = BidirSequence(B, H, lengths, D, cfg.chunk, TORCH_DTYPE[cfg.dtype], segments=segments, device=device)
    q, k, v = cut(inp.q), cut(inp.k), cut(inp.v)
    out = [torch.full_like(x, float("nan")) for x in q]
    seq.kv.fill_(float("nan"))
    kv = seq.forward(q, k, v, out)
    res = {"out": to_host(out), "kv": kv.cpu().numpy().astype(np.float64)}
    if backward:
        do = cut(inp.dout)
        dq, dk, dv = ([torch.full_like(x, float("nan")) for x in q] for _ in range(3))
        seq.dkv.fill_(float("nan"))
        dkv = seq.backward(q, k, v, do, dq, dk, dv)
        res.update(dq=to_host(dq), dk=to_host(dk), dv=to_host(dv), dkv=dkv.cpu().numpy().astype(np.float64))
    torch.cuda.synchronize()
    return res
