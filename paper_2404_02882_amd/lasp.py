"""Thin ctypes binding over the C-ABI library (include/lasp.h).

Argument marshalling only: every step of the path runs in the HIP kernels.
PyTorch supplies device memory and the current stream. If the shared library
has not been built, importing this module raises: there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblasp.so")

LASP_F32, LASP_BF16 = 0, 1
STATUS_NAMES = {0: "LASP_OK", 1: "LASP_ERR_NULL", 2: "LASP_ERR_SHAPE", 3: "LASP_ERR_DTYPE", 4: "LASP_ERR_DECAY",
                5: "LASP_ERR_WORKSPACE", 6: "LASP_ERR_ALIAS", 7: "LASP_ERR_HIP", 8: "LASP_ERR_ALIGN"}


class Shape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("N", ctypes.c_int32), ("D", ctypes.c_int32),
                ("chunk", ctypes.c_int32), ("dtype", ctypes.c_int32), ("segments", ctypes.c_int32),
                ("kv_heads", ctypes.c_int32), ("Dv", ctypes.c_int32)]


class LaspError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)} ({status_str(status)})")


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
                      "There is no fallback path.")

_vp, _sz = ctypes.c_void_p, ctypes.c_size_t
_sp = ctypes.POINTER(Shape)


def _bind(handle):
    """Declare the C signatures of include/lasp.h on a loaded library."""
    handle.lasp_version.restype = ctypes.c_int
    handle.lasp_status_str.restype = ctypes.c_char_p
    handle.lasp_status_str.argtypes = [ctypes.c_int]
    handle.lasp_check_shape.argtypes = [_sp]
    handle.lasp_check_decay.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_int32]
    handle.lasp_tile_tokens.argtypes = [_sp]
    handle.lasp_tile_tokens.restype = ctypes.c_int32
    handle.lasp_num_segments.argtypes = [_sp]
    handle.lasp_num_segments.restype = ctypes.c_int32
    handle.lasp_state_cache_bytes.argtypes = [_sp]
    handle.lasp_state_cache_bytes.restype = _sz
    handle.lasp_scratch_bytes.argtypes = [_sp]
    handle.lasp_scratch_bytes.restype = _sz
    handle.lasp_fwd.argtypes = [_sp] + [_vp] * 9 + [_sz, _vp]
    handle.lasp_fwd.restype = ctypes.c_int
    handle.lasp_fwd_noalloc.argtypes = [_sp] + [_vp] * 9
    handle.lasp_fwd_noalloc.restype = ctypes.c_int
    handle.lasp_noalloc_scratch_limit.argtypes = []
    handle.lasp_noalloc_scratch_limit.restype = _sz
    handle.lasp_bwd.argtypes = [_sp] + [_vp] * 13 + [_sz, _vp]
    handle.lasp_bwd_recompute_scratch_bytes.argtypes = [_sp]
    handle.lasp_bwd_recompute_scratch_bytes.restype = _sz
    handle.lasp_gated_bwd_recompute_scratch_bytes.argtypes = [_sp]
    handle.lasp_gated_bwd_recompute_scratch_bytes.restype = _sz
    handle.lasp_bwd.restype = ctypes.c_int
    handle.lasp_check_log_decay.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_int64]
    handle.lasp_gated_state_cache_bytes.argtypes = [_sp]
    handle.lasp_gated_state_cache_bytes.restype = _sz
    handle.lasp_gated_scratch_bytes.argtypes = [_sp]
    handle.lasp_gated_scratch_bytes.restype = _sz
    handle.lasp_gated_fwd.argtypes = [_sp] + [_vp] * 9 + [_sz, _vp]
    handle.lasp_gated_fwd.restype = ctypes.c_int
    handle.lasp_gated_bwd.argtypes = [_sp] + [_vp] * 15 + [_sz, _vp]
    handle.lasp_gated_bwd.restype = ctypes.c_int
    handle.lasp_fwd_norm.argtypes = [_sp] + [_vp] * 5 + [ctypes.c_float] + [_vp] * 5 + [_sz, _vp]
    handle.lasp_fwd_norm.restype = ctypes.c_int
    handle.lasp_bwd_norm.argtypes = [_sp] + [_vp] * 15 + [_sz, _vp]
    handle.lasp_bwd_norm.restype = ctypes.c_int
    handle.lasp_gated_fwd_norm.argtypes = [_sp] + [_vp] * 5 + [ctypes.c_float] + [_vp] * 5 + [_sz, _vp]
    handle.lasp_gated_fwd_norm.restype = ctypes.c_int
    handle.lasp_gated_bwd_norm.argtypes = [_sp] + [_vp] * 17 + [_sz, _vp]
    handle.lasp_gated_bwd_norm.restype = ctypes.c_int
    handle.lasp_bidir_scratch_bytes.argtypes = [_sp]
    handle.lasp_bidir_scratch_bytes.restype = _sz
    handle.lasp_bidir_state.argtypes = [_sp, _vp, _vp, _vp, ctypes.c_int32, _vp, _sz, _vp]
    handle.lasp_bidir_state.restype = ctypes.c_int
    handle.lasp_bidir_fwd.argtypes = [_sp] + [_vp] * 4
    handle.lasp_bidir_fwd.restype = ctypes.c_int
    handle.lasp_bidir_bwd.argtypes = [_sp] + [_vp] * 9
    handle.lasp_bidir_bwd.restype = ctypes.c_int
    handle.lasp_profile_begin.argtypes = [ctypes.c_int32]
    handle.lasp_profile_end.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32),
                                        ctypes.POINTER(ctypes.c_int32)]
    return handle


lib = _bind(ctypes.CDLL(LIB_PATH))


def profile_begin(max_calls: int) -> None:
    rc = lib.lasp_profile_begin(int(max_calls))
    if rc != 0:
        raise LaspError(rc, "lasp_profile_begin")


def profile_end():
    """Returns ({'fwd': (local, scan, walk), 'bwd': (...)} summed milliseconds, fwd_calls, bwd_calls)."""
    ms = (ctypes.c_double * 6)()
    nf, nb = ctypes.c_int32(0), ctypes.c_int32(0)
    rc = lib.lasp_profile_end(ms, ctypes.byref(nf), ctypes.byref(nb))
    if rc != 0:
        raise LaspError(rc, "lasp_profile_end")
    return {"fwd": tuple(ms[0:3]), "bwd": tuple(ms[3:6])}, nf.value, nb.value


def status_str(status: int) -> str:
    return lib.lasp_status_str(int(status)).decode()


def version() -> int:
    return int(lib.lasp_version())


def make_shape(B, H, N, D, chunk, dtype, segments=0, kv_heads=0, Dv=0) -> Shape:
    if isinstance(dtype, torch.dtype):
        dtype = {torch.float32: LASP_F32, torch.bfloat16: LASP_BF16}.get(dtype, -1)
    elif isinstance(dtype, str):
        dtype = {"f32": LASP_F32, "bf16": LASP_BF16}.get(dtype, -1)
    return Shape(int(B), int(H), int(N), int(D), int(chunk), int(dtype), int(segments), int(kv_heads), int(Dv))


def check_shape(shape: Shape) -> int:
    return int(lib.lasp_check_shape(ctypes.byref(shape)))


def check_decay(decay_host) -> int:
    arr = (ctypes.c_float * len(decay_host))(*[float(x) for x in decay_host])
    return int(lib.lasp_check_decay(arr, len(decay_host)))


def tile_tokens(shape: Shape) -> int:
    return int(lib.lasp_tile_tokens(ctypes.byref(shape)))


def num_segments(shape: Shape) -> int:
    return int(lib.lasp_num_segments(ctypes.byref(shape)))


def state_cache_bytes(shape: Shape) -> int:
    return int(lib.lasp_state_cache_bytes(ctypes.byref(shape)))


def scratch_bytes(shape: Shape) -> int:
    return int(lib.lasp_scratch_bytes(ctypes.byref(shape)))


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensors handed to the library must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def lasp_fwd(shape: Shape, q, k, v, kv_in, decay, out, kv_out, state_cache, scratch, stream=None) -> None:
    """Enqueue the forward pass; raises LaspError on a non-zero status."""
    nbytes = scratch.numel() * scratch.element_size() if scratch is not None else 0
    rc = lib.lasp_fwd(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(kv_in), _ptr(decay), _ptr(out),
                      _ptr(kv_out), _ptr(state_cache), _ptr(scratch), nbytes, _stream(stream))
    if rc != 0:
        raise LaspError(rc, "lasp_fwd")


def noalloc_scratch_limit() -> int:
    return int(lib.lasp_noalloc_scratch_limit())


def lasp_fwd_noalloc(shape: Shape, q, k, v, kv_in, decay, out, kv_out, state_cache, stream=None) -> None:
    """lasp_fwd with the library's own fixed scratch (no workspace argument); raises LaspError on a non-zero status."""
    rc = lib.lasp_fwd_noalloc(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(kv_in), _ptr(decay), _ptr(out),
                              _ptr(kv_out), _ptr(state_cache), _stream(stream))
    if rc != 0:
        raise LaspError(rc, "lasp_fwd_noalloc")


def bwd_recompute_scratch_bytes(shape: Shape) -> int:
    return int(lib.lasp_bwd_recompute_scratch_bytes(ctypes.byref(shape)))


def gated_bwd_recompute_scratch_bytes(shape: Shape) -> int:
    return int(lib.lasp_gated_bwd_recompute_scratch_bytes(ctypes.byref(shape)))


def lasp_bwd(shape: Shape, q, k, v, dout, kv_in, dkv_out, decay, state_cache, dq, dk, dv, dkv_in, scratch,
             stream=None) -> None:
    """Enqueue the backward pass (state_cache None = the states are rebuilt from k, v, kv_in); raises LaspError
    on a non-zero status."""
    nbytes = scratch.numel() * scratch.element_size() if scratch is not None else 0
    rc = lib.lasp_bwd(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(dout), _ptr(kv_in), _ptr(dkv_out), _ptr(decay),
                      _ptr(state_cache), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dkv_in), _ptr(scratch), nbytes,
                      _stream(stream))
    if rc != 0:
        raise LaspError(rc, "lasp_bwd")


def check_log_decay(log_g_host) -> int:
    import numpy as np
    a = np.ascontiguousarray(log_g_host, dtype=np.float32).ravel()
    return int(lib.lasp_check_log_decay(a.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), a.size))


def gated_state_cache_bytes(shape: Shape) -> int:
    return int(lib.lasp_gated_state_cache_bytes(ctypes.byref(shape)))


def gated_scratch_bytes(shape: Shape) -> int:
    return int(lib.lasp_gated_scratch_bytes(ctypes.byref(shape)))


def lasp_gated_fwd(shape: Shape, q, k, v, log_g, kv_in, out, kv_out, state_cache, scratch, stream=None) -> None:
    """Forward with a decay per token (log_g: float32 [B,H,N]); raises LaspError on a non-zero status."""
    nbytes = scratch.numel() * scratch.element_size() if scratch is not None else 0
    rc = lib.lasp_gated_fwd(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(log_g), _ptr(kv_in), _ptr(out),
                            _ptr(kv_out), _ptr(state_cache), _ptr(scratch), nbytes, _stream(stream))
    if rc != 0:
        raise LaspError(rc, "lasp_gated_fwd")


def lasp_gated_bwd(shape: Shape, q, k, v, dout, log_g, kv_in, kv_out, dkv_out, state_cache, dq, dk, dv, dlog_g, dkv_in,
                   scratch, stream=None) -> None:
    """Backward with a decay per token; raises LaspError on a non-zero status."""
    nbytes = scratch.numel() * scratch.element_size() if scratch is not None else 0
    rc = lib.lasp_gated_bwd(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(dout), _ptr(log_g), _ptr(kv_in), _ptr(kv_out),
                            _ptr(dkv_out), _ptr(state_cache), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dlog_g),
                            _ptr(dkv_in), _ptr(scratch), nbytes, _stream(stream))
    if rc != 0:
        raise LaspError(rc, "lasp_gated_bwd")


def lasp_fwd_norm(shape: Shape, q, k, v, kv_in, decay, eps, out, rstd, kv_out, state_cache, scratch,
                  stream=None) -> None:
    """Forward with the normalised output (out = Norm(o), rstd: float32 [B,H,N]); raises LaspError."""
    nbytes = scratch.numel() * scratch.element_size() if scratch is not None else 0
    rc = lib.lasp_fwd_norm(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(kv_in), _ptr(decay), float(eps),
                           _ptr(out), _ptr(rstd), _ptr(kv_out), _ptr(state_cache), _ptr(scratch), nbytes,
                           _stream(stream))
    if rc != 0:
        raise LaspError(rc, "lasp_fwd_norm")


def lasp_bwd_norm(shape: Shape, q, k, v, out, rstd, dout, kv_in, dkv_out, decay, state_cache, dq, dk, dv, dkv_in,
                  scratch, stream=None) -> None:
    """Backward of lasp_fwd_norm (dout: gradient w.r.t. the normalised output); raises LaspError."""
    nbytes = scratch.numel() * scratch.element_size() if scratch is not None else 0
    rc = lib.lasp_bwd_norm(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(rstd), _ptr(dout),
                           _ptr(kv_in), _ptr(dkv_out), _ptr(decay), _ptr(state_cache), _ptr(dq), _ptr(dk), _ptr(dv),
                           _ptr(dkv_in), _ptr(scratch), nbytes, _stream(stream))
    if rc != 0:
        raise LaspError(rc, "lasp_bwd_norm")


def lasp_gated_fwd_norm(shape: Shape, q, k, v, log_g, kv_in, eps, out, rstd, kv_out, state_cache, scratch,
                        stream=None) -> None:
    """Per-token decay and normalised output together; raises LaspError on a non-zero status."""
    nbytes = scratch.numel() * scratch.element_size() if scratch is not None else 0
    rc = lib.lasp_gated_fwd_norm(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(log_g), _ptr(kv_in), float(eps),
                                 _ptr(out), _ptr(rstd), _ptr(kv_out), _ptr(state_cache), _ptr(scratch), nbytes,
                                 _stream(stream))
    if rc != 0:
        raise LaspError(rc, "lasp_gated_fwd_norm")


def lasp_gated_bwd_norm(shape: Shape, q, k, v, out, rstd, dout, log_g, kv_in, kv_out, dkv_out, state_cache, dq, dk, dv,
                        dlog_g, dkv_in, scratch, stream=None) -> None:
    """Backward of lasp_gated_fwd_norm; raises LaspError on a non-zero status."""
    nbytes = scratch.numel() * scratch.element_size() if scratch is not None else 0
    rc = lib.lasp_gated_bwd_norm(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(rstd), _ptr(dout),
                                 _ptr(log_g), _ptr(kv_in), _ptr(kv_out), _ptr(dkv_out), _ptr(state_cache), _ptr(dq), _ptr(dk),
                                 _ptr(dv), _ptr(dlog_g), _ptr(dkv_in), _ptr(scratch), nbytes, _stream(stream))
    if rc != 0:
        raise LaspError(rc, "lasp_gated_bwd_norm")


def bidir_scratch_bytes(shape: Shape) -> int:
    return int(lib.lasp_bidir_scratch_bytes(ctypes.byref(shape)))


def lasp_bidir_state(shape: Shape, x, y, state, accumulate, scratch, stream=None) -> None:
    """state (+)= sum over tokens of x_s y_s^T (bidirectional attention); raises LaspError on a non-zero status."""
    nbytes = scratch.numel() * scratch.element_size() if scratch is not None else 0
    rc = lib.lasp_bidir_state(ctypes.byref(shape), _ptr(x), _ptr(y), _ptr(state), int(bool(accumulate)), _ptr(scratch),
                              nbytes, _stream(stream))
    if rc != 0:
        raise LaspError(rc, "lasp_bidir_state")


def lasp_bidir_fwd(shape: Shape, q, kv, out, stream=None) -> None:
    """out = q kv; raises LaspError on a non-zero status."""
    rc = lib.lasp_bidir_fwd(ctypes.byref(shape), _ptr(q), _ptr(kv), _ptr(out), _stream(stream))
    if rc != 0:
        raise LaspError(rc, "lasp_bidir_fwd")


def lasp_bidir_bwd(shape: Shape, k, v, dout, kv, dkv, dq, dk, dv, stream=None) -> None:
    """dq = dout kv^T, dk = v dkv^T, dv = k dkv; raises LaspError on a non-zero status."""
    rc = lib.lasp_bidir_bwd(ctypes.byref(shape), _ptr(k), _ptr(v), _ptr(dout), _ptr(kv), _ptr(dkv), _ptr(dq), _ptr(dk),
                            _ptr(dv), _stream(stream))
    if rc != 0:
        raise LaspError(rc, "lasp_bidir_bwd")


class Workspace:
    """Device buffers one (shape) needs besides the tensors: per-tile state cache and scratch."""

    def __init__(self, shape: Shape, device="cuda", with_cache=True):
        self.shape = shape
        if check_shape(shape) != 0:
            raise LaspError(check_shape(shape), "Workspace")
        self.cache = torch.empty(state_cache_bytes(shape), dtype=torch.uint8, device=device) if with_cache else None
        self.scratch = torch.empty(scratch_bytes(shape), dtype=torch.uint8, device=device)
