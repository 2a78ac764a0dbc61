"""Outer loop over sub-sequences: the paper's ring of ranks on one GPU.

A sequence of N tokens is held as T shards of N/T tokens, each a contiguous
[B,H,N/T,D] tensor (what one rank of the paper holds). Forward runs the shards
in order and hands kv_out of one to the next as kv_in (Alg. 2: Recv KV from
rank i-1, Send KV to rank i+1); backward runs them in reverse and hands dkv_in
of one to the previous as dkv_out (Alg. 3). Every shard keeps the per-tile
state cache its forward call filled until its backward call has used it.
All buffers are allocated once, up front; the calls only enqueue kernels.
"""
from __future__ import annotations

from typing import List, Optional

import torch

from . import lasp


class LaspSequence:
    def __init__(self, B, H, N, D, chunk, dtype: torch.dtype, T=1, segments=0, device="cuda", need_backward=True,
                 token_decay=False, norm_eps: Optional[float] = None, kv_heads=0, Dv=0, recompute=False):
        if N % T != 0:
            raise ValueError("N must be a multiple of T")
        self.B, self.H, self.N, self.D, self.T = B, H, N, D, T
        self.n_sub = N // T
        self.dtype = dtype
        # kv_heads: k, v, dk, dv shards are [B,kv_heads,N/T,D]; groups of H/kv_heads query heads share them
        # Dv: value dimension when it differs from the key dimension D (v, out, dout, dv shards are [..,Dv],
        # states [B,H,D,Dv])
        self.shape = lasp.make_shape(B, H, self.n_sub, D, chunk, dtype, segments, kv_heads, Dv)
        rc = lasp.check_shape(self.shape)
        if rc != 0:
            raise lasp.LaspError(rc, "LaspSequence")
        # token_decay: `decay` of forward / backward is a list of T log-decay shards [B,H,N/T] (float32)
        # instead of the [H] vector of lambdas, and backward also fills dlog_g shards.
        # norm_eps: outputs are normalised (lasp_fwd_norm / lasp_bwd_norm); forward fills `rstd` shards
        # [B,H,N/T], backward takes them and the forward outputs. Both may be set together.
        self.norm_eps = norm_eps
        self.token_decay = token_decay
        # recompute: no state cache is kept between the passes (Sec. 3.4's alternative to caching); every
        # backward call rebuilds the states of its shard from k, v and the state the shard started from,
        # into the tail of the (then larger) scratch buffer, which all shards share
        self.recompute = bool(recompute)
        if self.recompute and need_backward:
            scratch_bytes = lasp.gated_bwd_recompute_scratch_bytes if token_decay else lasp.bwd_recompute_scratch_bytes
        else:
            scratch_bytes = lasp.gated_scratch_bytes if token_decay else lasp.scratch_bytes
        cache_bytes = lasp.gated_state_cache_bytes if token_decay else lasp.state_cache_bytes
        self.scratch = torch.empty(scratch_bytes(self.shape), dtype=torch.uint8, device=device)
        self.caches = [torch.empty(cache_bytes(self.shape), dtype=torch.uint8, device=device)
                       for _ in range(T)] if need_backward and not self.recompute else [None] * T
        st = dict(dtype=torch.float32, device=device)
        # kv[t] = state entering shard t (kv[T] = final); dkv[t] = gradient w.r.t. kv[t]
        self.kv = [torch.zeros(B, H, D, Dv or D, **st) for _ in range(T + 1)]
        self.dkv = [torch.zeros(B, H, D, Dv or D, **st) for _ in range(T + 1)] if need_backward else None
        self.has_kv_in = False
        self.has_dkv_out = False

    def cache_bytes(self) -> int:
        return sum(c.numel() for c in self.caches if c is not None)

    def workspace_bytes(self) -> int:
        return int(self.scratch.numel())

    def forward(self, q: List[torch.Tensor], k, v, decay, out: List[torch.Tensor],
                kv_in: Optional[torch.Tensor] = None, rstd: Optional[List[torch.Tensor]] = None) -> torch.Tensor:
        self.has_kv_in = kv_in is not None
        if kv_in is not None:
            self.kv[0].copy_(kv_in)
        for t in range(self.T):
            first = None if (t == 0 and not self.has_kv_in) else self.kv[t]
            if self.norm_eps is not None and self.token_decay:
                lasp.lasp_gated_fwd_norm(self.shape, q[t], k[t], v[t], decay[t], first, self.norm_eps, out[t], rstd[t],
                                         self.kv[t + 1], self.caches[t], self.scratch)
            elif self.norm_eps is not None:
                lasp.lasp_fwd_norm(self.shape, q[t], k[t], v[t], first, decay, self.norm_eps, out[t], rstd[t],
                                   self.kv[t + 1], self.caches[t], self.scratch)
            elif self.token_decay:
                lasp.lasp_gated_fwd(self.shape, q[t], k[t], v[t], decay[t], first, out[t], self.kv[t + 1],
                                    self.caches[t], self.scratch)
            else:
                lasp.lasp_fwd(self.shape, q[t], k[t], v[t], first, decay, out[t], self.kv[t + 1], self.caches[t],
                              self.scratch)
        return self.kv[self.T]

    def backward(self, q, k, v, dout, decay, dq, dk, dv, dkv_out: Optional[torch.Tensor] = None,
                 dlog_g: Optional[List[torch.Tensor]] = None, out: Optional[List[torch.Tensor]] = None,
                 rstd: Optional[List[torch.Tensor]] = None) -> torch.Tensor:
        self.has_dkv_out = dkv_out is not None
        if dkv_out is not None:
            self.dkv[self.T].copy_(dkv_out)
        for t in reversed(range(self.T)):
            last = None if (t == self.T - 1 and not self.has_dkv_out) else self.dkv[t + 1]
            first = None if (t == 0 and not self.has_kv_in) else self.kv[t]   # read only without a cache
            if self.norm_eps is not None and self.token_decay:
                lasp.lasp_gated_bwd_norm(self.shape, q[t], k[t], v[t], out[t], rstd[t], dout[t], decay[t], first,
                                         self.kv[t + 1], last, self.caches[t], dq[t], dk[t], dv[t], dlog_g[t],
                                         self.dkv[t], self.scratch)
            elif self.norm_eps is not None:
                lasp.lasp_bwd_norm(self.shape, q[t], k[t], v[t], out[t], rstd[t], dout[t], first, last, decay,
                                   self.caches[t], dq[t], dk[t], dv[t], self.dkv[t], self.scratch)
            elif self.token_decay:
                lasp.lasp_gated_bwd(self.shape, q[t], k[t], v[t], dout[t], decay[t], first, self.kv[t + 1], last,
                                    self.caches[t], dq[t], dk[t], dv[t], dlog_g[t], self.dkv[t], self.scratch)
            else:
                lasp.lasp_bwd(self.shape, q[t], k[t], v[t], dout[t], first, last, decay, self.caches[t], dq[t], dk[t],
                              dv[t], self.dkv[t], self.scratch)
        return self.dkv[0]


class GraphedStep:
    """One forward + backward pass of a LaspSequence captured in a HIP graph and replayed.

    With short sub-sequences the T-loop is launch-bound (six small kernels per call, 2T calls per
    step); a graph replays them with one submission. The library allocates nothing and never
    synchronises, so its calls can be captured as they are. The graph reads and writes the very
    tensors given here: refresh their contents in place between replays. Per-kernel timing
    (lasp_profile_begin) must be off while capturing.
    """

    def __init__(self, seq: LaspSequence, fwd_kwargs: Optional[dict], bwd_kwargs: Optional[dict] = None, warmup: int = 2):
        """fwd_kwargs None: the graph holds the backward pass alone (the state caches must already hold what a
        forward pass over the same inputs wrote); bwd_kwargs None: the forward pass alone."""
        self.seq = seq
        if fwd_kwargs is None and bwd_kwargs is None:
            raise ValueError("nothing to capture")

        def run():
            if fwd_kwargs is not None:
                seq.forward(**fwd_kwargs)
            if bwd_kwargs is not None:
                seq.backward(**bwd_kwargs)

        # eager passes first, on a side stream as graph capture requires: they set the kernels'
        # LDS attributes (a host-side call that must not fall inside the capture)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(max(1, warmup)):
                run()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            run()

    def replay(self) -> None:
        self.graph.replay()


class BidirSequence:
    """Bidirectional (unmasked) attention O = Q (K^T V) over sub-sequences of any lengths.

    The state is a sum over every token, so nothing is handed from shard to shard: a first loop adds
    each shard's K^T V into `kv` (on several devices: their partial states summed across them), a
    second loop computes each shard's output from the complete state. Backward likewise with
    dKV = Q^T dO. All buffers are allocated up front; the calls only enqueue kernels.
    """

    def __init__(self, B, H, lengths, D, chunk, dtype: torch.dtype, segments=0, device="cuda"):
        self.lengths = [int(n) for n in lengths]
        self.shapes = [lasp.make_shape(B, H, n, D, chunk, dtype, segments) for n in self.lengths]
        need = 0
        for shp in self.shapes:
            nbytes = lasp.bidir_scratch_bytes(shp)
            if nbytes == 0:
                raise lasp.LaspError(lasp.check_shape(shp) or 2, "BidirSequence")
            need = max(need, nbytes)
        self.scratch = torch.empty(need, dtype=torch.uint8, device=device)
        st = dict(dtype=torch.float32, device=device)
        self.kv = torch.empty(B, H, D, D, **st)
        self.dkv = torch.empty(B, H, D, D, **st)

    def forward(self, q: List[torch.Tensor], k, v, out: List[torch.Tensor]) -> torch.Tensor:
        for t, shp in enumerate(self.shapes):
            lasp.lasp_bidir_state(shp, k[t], v[t], self.kv, t > 0, self.scratch)
        for t, shp in enumerate(self.shapes):
            lasp.lasp_bidir_fwd(shp, q[t], self.kv, out[t])
        return self.kv

    def backward(self, q, k, v, dout, dq, dk, dv) -> torch.Tensor:
        """Needs the state `kv` of the forward pass."""
        for t, shp in enumerate(self.shapes):
            lasp.lasp_bidir_state(shp, q[t], dout[t], self.dkv, t > 0, self.scratch)
        for t, shp in enumerate(self.shapes):
            lasp.lasp_bidir_bwd(shp, k[t], v[t], dout[t], self.kv, self.dkv, dq[t], dk[t], dv[t])
        return self.dkv
