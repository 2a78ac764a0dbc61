"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol include/lasp.h declares, and rejects bad arguments before any
launch (no compute call is made here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2404_02882_amd import lasp
    return lasp


def test_exports_every_declared_symbol(L):
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):   # lasp.h (the method) and lasp_profile.h (timing)
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(lasp_[a-z_]+)\s*\(", text))
    assert {"lasp_fwd", "lasp_bwd", "lasp_scratch_bytes", "lasp_state_cache_bytes", "lasp_fwd_noalloc",
            "lasp_bwd_recompute_scratch_bytes", "lasp_profile_begin"} <= names
    for n in names:
        assert hasattr(L.lib, n), n
    assert L.version() >= 1


def test_status_strings(L):
    for s in range(9):
        assert L.status_str(s) and "unknown" not in L.status_str(s)
    assert "unknown" in L.status_str(99)


@pytest.mark.parametrize("kw,expect", [
    (dict(), 0),
    (dict(D=96), 2), (dict(D=256), 2), (dict(chunk=32), 2), (dict(chunk=512), 2),
    (dict(N=1000), 0), (dict(N=1), 0), (dict(N=0), 2), (dict(B=0), 2), (dict(H=-1), 2),
    (dict(dtype=2), 3), (dict(dtype=-1), 3),
    (dict(segments=-1), 2), (dict(segments="tiles+1"), 2), (dict(segments="tiles"), 0),
])
def test_check_shape(L, kw, expect):
    base = dict(B=2, H=4, N=1024, D=128, chunk=128, dtype=1, segments=0)
    base.update(kw)
    if isinstance(base["segments"], str):   # relative to the tile count of this shape
        tiles = base["N"] // L.tile_tokens(L.make_shape(**dict(base, segments=0)))
        base["segments"] = tiles + 1 if base["segments"] == "tiles+1" else tiles
    assert L.check_shape(L.make_shape(**base)) == expect


def test_sizes_and_plan(L):
    s = L.make_shape(1, 16, 32768, 128, 128, "bf16")
    tile = L.tile_tokens(s)
    assert tile in (32, 64, 128) and 128 % tile == 0          # the tile divides the chunk
    nseg = L.num_segments(s)
    assert 1 <= nseg <= 32768 // tile and 16 * nseg >= 256     # enough workgroups to fill 256 CUs
    per_tile = 16 * (32768 // tile) * 128 * 128 * 2
    assert L.state_cache_bytes(s) in (per_tile, per_tile // 2)   # one cached state per tile, or per pair of tiles
    assert L.scratch_bytes(s) == 16 * nseg * 128 * 128 * 4
    f = L.make_shape(1, 2, 256, 64, 64, "f32")
    ft = L.tile_tokens(f)
    assert ft > 0 and 64 % ft == 0
    assert L.state_cache_bytes(f) == 2 * (256 // ft) * 64 * 64 * 4
    # a segment count that does not divide the tiles still covers them all
    r = L.make_shape(1, 1, 64 * 7, 64, 64, "bf16", segments=3)
    assert 1 <= L.num_segments(r) <= 3
    bad = L.make_shape(1, 1, 128, 96, 64, "bf16")
    assert L.tile_tokens(bad) == 0 and L.scratch_bytes(bad) == 0 and L.state_cache_bytes(bad) == 0
    # a length that is not a multiple of the tile: one more (short) tile, and scratch for the synthesised log g
    rag = L.make_shape(1, 2, 64 * 3 + 5, 64, 64, "bf16")
    full = L.make_shape(1, 2, 64 * 4, 64, 64, "bf16")
    assert L.state_cache_bytes(rag) == L.state_cache_bytes(full)
    assert L.scratch_bytes(rag) > L.scratch_bytes(full)
    assert L.gated_scratch_bytes(rag) < L.scratch_bytes(rag)


def test_check_decay(L):
    assert L.check_decay([1.0, 0.5, 0.999]) == 0
    assert L.check_decay([0.0]) == 4
    assert L.check_decay([1.0001]) == 4
    assert L.check_decay([float("nan")]) == 4
    assert L.check_decay([-0.5]) == 4


def _fake(n):
    """Distinct non-null addresses that are never dereferenced (validation fails first)."""
    return ctypes.c_void_p(0x10000000 + n * 0x10000000)


def test_fwd_rejects_before_launch(L):
    s = L.make_shape(1, 1, 64, 64, 64, "bf16")
    sb = L.scratch_bytes(s)
    P = [_fake(i) for i in range(1, 10)]
    q, k, v, kvin, dec, out, kvout, cache, scr = P
    call = lambda *a: L.lib.lasp_fwd(*a)
    assert call(None, q, k, v, kvin, dec, out, kvout, cache, scr, sb, None) == 1
    assert call(ctypes.byref(s), None, k, v, kvin, dec, out, kvout, cache, scr, sb, None) == 1
    assert call(ctypes.byref(s), q, k, v, kvin, None, out, kvout, cache, scr, sb, None) == 1
    assert call(ctypes.byref(s), q, k, v, kvin, dec, None, kvout, cache, scr, sb, None) == 1
    assert call(ctypes.byref(s), q, k, v, kvin, dec, out, None, cache, scr, sb, None) == 1
    assert call(ctypes.byref(s), q, k, v, kvin, dec, out, kvout, cache, None, sb, None) == 5
    assert call(ctypes.byref(s), q, k, v, kvin, dec, out, kvout, cache, scr, sb - 1, None) == 5
    assert call(ctypes.byref(s), q, k, v, kvin, dec, q, kvout, cache, scr, sb, None) == 6      # out aliases q
    assert call(ctypes.byref(s), q, k, v, kvin, dec, out, kvin, cache, scr, sb, None) == 6     # kv_out aliases kv_in
    assert call(ctypes.byref(s), q, k, v, kvin, dec, out, kvout, out, scr, sb, None) == 6      # cache aliases out
    odd = ctypes.c_void_p(q.value + 8)
    assert call(ctypes.byref(s), odd, k, v, kvin, dec, out, kvout, cache, scr, sb, None) == 8   # q not 16-byte aligned
    assert call(ctypes.byref(s), q, k, v, kvin, dec, out, kvout, cache, ctypes.c_void_p(scr.value + 4), sb, None) == 8
    bad = L.make_shape(1, 1, 64, 96, 64, "bf16")
    assert call(ctypes.byref(bad), q, k, v, kvin, dec, out, kvout, cache, scr, sb, None) == 2
    bad = L.make_shape(1, 1, 64, 64, 64, 7)
    assert call(ctypes.byref(bad), q, k, v, kvin, dec, out, kvout, cache, scr, sb, None) == 3


def test_bwd_rejects_before_launch(L):
    s = L.make_shape(1, 1, 64, 64, 64, "f32")
    sb = L.scratch_bytes(s)
    P = [_fake(i) for i in range(1, 15)]
    q, k, v, do, g, dec, cache, dq, dk, dv, gin, scr, kvin, _ = P
    call = lambda *a: L.lib.lasp_bwd(*a)
    ok_args = [ctypes.byref(s), q, k, v, do, kvin, g, dec, cache, dq, dk, dv, gin, scr, sb, None]
    for idx in (1, 2, 3, 4, 7, 9, 10, 11, 12):   # every required pointer (kv_in, dkv_out and the cache are optional)
        a = list(ok_args)
        a[idx] = None
        assert call(*a) == 1, idx
    a = list(ok_args); a[13] = None
    assert call(*a) == 5
    a = list(ok_args); a[14] = 0
    assert call(*a) == 5
    a = list(ok_args); a[9] = q
    assert call(*a) == 6
    a = list(ok_args); a[10] = dq
    assert call(*a) == 6
    a = list(ok_args); a[12] = g
    assert call(*a) == 6
    # no state cache = the states are rebuilt: more scratch, and kv_in becomes an input
    rb = L.bwd_recompute_scratch_bytes(s)
    assert rb >= sb + L.state_cache_bytes(s) and rb % 16 == 0
    a = list(ok_args); a[8] = None                   # scratch of the cached path is too small
    assert call(*a) == 5
    a = list(ok_args); a[8] = None; a[14] = rb; a[12] = kvin   # dkv_in aliases kv_in
    assert call(*a) == 6
    assert L.bwd_recompute_scratch_bytes(L.make_shape(1, 1, 64, 96, 64, "f32")) == 0


# ---------------------------------------------------------------- per-token decay entry points
def test_gated_sizes(L):
    s = L.make_shape(1, 16, 32768, 128, 128, "bf16")
    tile = L.tile_tokens(s)
    per_tile = 16 * (32768 // tile) * 128 * 128 * 2
    assert L.gated_state_cache_bytes(s) in (per_tile, per_tile // 2)
    # segment states + one log-decay per segment + one float per token and head
    assert L.gated_scratch_bytes(s) >= L.scratch_bytes(s) + 16 * 32768 * 4
    bad = L.make_shape(1, 1, 100, 64, 32, "bf16")
    assert L.gated_scratch_bytes(bad) == 0 and L.gated_state_cache_bytes(bad) == 0


def test_check_log_decay(L):
    assert L.check_log_decay([0.0, -0.5, -30.0]) == 0
    assert L.check_log_decay([1e-3]) == 4
    assert L.check_log_decay([float("nan")]) == 4
    assert L.check_log_decay([float("-inf")]) == 4


def test_gated_fwd_rejects_before_launch(L):
    s = L.make_shape(1, 1, 64, 64, 64, "bf16")
    sb = L.gated_scratch_bytes(s)
    q, k, v, lg, kvin, out, kvout, cache, scr = [_fake(i) for i in range(1, 10)]
    call = lambda *a: L.lib.lasp_gated_fwd(*a)
    ok_args = [ctypes.byref(s), q, k, v, lg, kvin, out, kvout, cache, scr, sb, None]
    for idx in (1, 2, 3, 4, 6, 7):
        a = list(ok_args)
        a[idx] = None
        assert call(*a) == 1, idx
    a = list(ok_args); a[9] = None
    assert call(*a) == 5
    a = list(ok_args); a[10] = L.scratch_bytes(s)    # the fixed-decay size is too small
    assert call(*a) == 5
    a = list(ok_args); a[6] = lg                     # out aliases log_g
    assert call(*a) == 6
    a = list(ok_args); a[0] = ctypes.byref(L.make_shape(1, 1, 64, 64, 96, "bf16"))
    assert call(*a) == 2


def test_gated_bwd_rejects_before_launch(L):
    s = L.make_shape(1, 1, 64, 64, 64, "f32")
    sb = L.gated_scratch_bytes(s)
    q, k, v, do, lg, kvout, g, cache, dq, dk, dv, dlg, gin, scr, kvin = [_fake(i) for i in range(1, 16)]
    call = lambda *a: L.lib.lasp_gated_bwd(*a)
    ok_args = [ctypes.byref(s), q, k, v, do, lg, kvin, kvout, g, cache, dq, dk, dv, dlg, gin, scr, sb, None]
    for idx in (1, 2, 3, 4, 5, 10, 11, 12, 13, 14):   # every required pointer
        a = list(ok_args)
        a[idx] = None
        assert call(*a) == 1, idx
    a = list(ok_args); a[7] = None                   # dkv_out given but kv_out missing
    assert call(*a) == 1
    a = list(ok_args); a[15] = None
    assert call(*a) == 5
    a = list(ok_args); a[16] = sb - 1
    assert call(*a) == 5
    a = list(ok_args); a[13] = lg                    # dlog_g aliases log_g
    assert call(*a) == 6
    a = list(ok_args); a[14] = kvout                 # dkv_in aliases kv_out
    assert call(*a) == 6
    a = list(ok_args); a[13] = ctypes.c_void_p(dlg.value + 4)   # dlog_g not 16-byte aligned
    assert call(*a) == 8
    a = list(ok_args); a[9] = None                   # no cache: the cached path's scratch is too small
    assert call(*a) == 5
    assert L.gated_bwd_recompute_scratch_bytes(s) >= sb + L.gated_state_cache_bytes(s)


# ---------------------------------------------------------------- normalised output entry points
def test_norm_rejects_before_launch(L):
    s = L.make_shape(1, 1, 64, 64, 64, "bf16")
    sb = L.scratch_bytes(s)
    q, k, v, kvin, dec, out, rstd, kvout, cache, scr = [_fake(i) for i in range(1, 11)]
    call = lambda *a: L.lib.lasp_fwd_norm(*a)
    ok_args = [ctypes.byref(s), q, k, v, kvin, dec, 1e-6, out, rstd, kvout, cache, scr, sb, None]
    for idx in (1, 2, 3, 5, 7, 8, 9):
        a = list(ok_args)
        a[idx] = None
        assert call(*a) == 1, idx
    a = list(ok_args); a[6] = -1.0
    assert call(*a) == 2
    a = list(ok_args); a[6] = float("nan")
    assert call(*a) == 2
    a = list(ok_args); a[12] = sb - 1
    assert call(*a) == 5
    a = list(ok_args); a[8] = out                    # rstd aliases out
    assert call(*a) == 6
    # a length that is not a multiple of the tile is a valid shape; it needs more scratch (log g is synthesised)
    ragged = L.make_shape(1, 1, 100, 64, 64, "bf16")
    assert L.check_shape(ragged) == 0 and L.scratch_bytes(ragged) > sb
    a = list(ok_args); a[0] = ctypes.byref(ragged)
    assert call(*a) == 5

    do, g, dq, dk, dv, gin = [_fake(i) for i in range(11, 17)]
    call = lambda *a: L.lib.lasp_bwd_norm(*a)
    ok_args = [ctypes.byref(s), q, k, v, out, rstd, do, kvin, g, dec, cache, dq, dk, dv, gin, scr, sb, None]
    for idx in (1, 2, 3, 4, 5, 6, 9, 11, 12, 13, 14):
        a = list(ok_args)
        a[idx] = None
        assert call(*a) == 1, idx
    a = list(ok_args); a[15] = None
    assert call(*a) == 5
    a = list(ok_args); a[11] = out                   # dq aliases the forward output
    assert call(*a) == 6
    a = list(ok_args); a[10] = None                  # no cache: needs the larger scratch
    assert call(*a) == 5


def test_gated_norm_rejects_before_launch(L):
    s = L.make_shape(1, 1, 64, 64, 64, "bf16")
    sb = L.gated_scratch_bytes(s)
    q, k, v, lg, kvin, out, rstd, kvout, cache, scr = [_fake(i) for i in range(1, 11)]
    call = lambda *a: L.lib.lasp_gated_fwd_norm(*a)
    ok_args = [ctypes.byref(s), q, k, v, lg, kvin, 1e-6, out, rstd, kvout, cache, scr, sb, None]
    for idx in (1, 2, 3, 4, 7, 8, 9):
        a = list(ok_args)
        a[idx] = None
        assert call(*a) == 1, idx
    a = list(ok_args); a[12] = L.scratch_bytes(s)
    assert call(*a) == 5
    ragged = L.make_shape(1, 1, 70, 64, 64, "bf16")          # a short last tile is a valid shape
    assert L.check_shape(ragged) == 0
    a = list(ok_args); a[0] = ctypes.byref(ragged); a[12] = L.gated_scratch_bytes(ragged) - 1
    assert call(*a) == 5
    do, g, dq, dk, dv, dlg, gin = [_fake(i) for i in range(11, 18)]
    call = lambda *a: L.lib.lasp_gated_bwd_norm(*a)
    ok_args = [ctypes.byref(s), q, k, v, out, rstd, do, lg, kvin, kvout, g, cache, dq, dk, dv, dlg, gin, scr, sb, None]
    for idx in (1, 2, 3, 4, 5, 6, 7, 12, 13, 14, 15, 16):
        a = list(ok_args)
        a[idx] = None
        assert call(*a) == 1, idx
    a = list(ok_args); a[9] = None      # dkv_out without kv_out
    assert call(*a) == 1
    a = list(ok_args); a[15] = out      # dlog_g aliases the forward output
    assert call(*a) == 6


# ---------------------------------------------------------------- grouped K/V heads
def test_kv_heads_shape_and_sizes(L):
    base = dict(B=2, H=8, N=1024, D=128, chunk=128, dtype=1, segments=0)
    for kvh, expect in ((0, 0), (8, 0), (4, 0), (1, 0), (3, 2), (16, 2), (-1, 2)):
        assert L.check_shape(L.make_shape(**base, kv_heads=kvh)) == expect, kvh
    mha, gqa = L.make_shape(**base), L.make_shape(**base, kv_heads=2)
    assert L.state_cache_bytes(gqa) == L.state_cache_bytes(mha)                 # states stay per query head
    tensor = 2 * 8 * 1024 * 128 * 2
    assert L.scratch_bytes(gqa) == L.scratch_bytes(mha) + 2 * tensor            # dK, dV per query head
    assert L.gated_scratch_bytes(gqa) == L.gated_scratch_bytes(mha) + 2 * tensor


def test_kv_heads_alias_check_uses_group_sizes(L):
    """k of a grouped call is [B, kv_heads, N, D]: an output overlapping its last bytes is an alias.
    (Every call here stops at validation; nothing is launched.)"""
    s = L.make_shape(1, 4, 64, 64, 64, "bf16", kv_heads=1)
    sb = L.scratch_bytes(s)
    one_head = 64 * 64 * 2
    q, kvin, dec, kvout, cache, scr = [_fake(i) for i in range(1, 7)]
    k, v = _fake(8), _fake(9)
    out_inside_k = ctypes.c_void_p(k.value + one_head - 16)
    assert L.lib.lasp_fwd(ctypes.byref(s), q, k, v, kvin, dec, out_inside_k, kvout, cache, scr, sb, None) == 6


# ---------------------------------------------------------------- bidirectional entry points
def test_bidir_sizes(L):
    s = L.make_shape(1, 16, 32768, 128, 128, "bf16")
    sb = L.bidir_scratch_bytes(s)
    assert sb > 0 and sb % (16 * 128 * 128 * 4) == 0            # whole partial states per head
    assert 16 * (sb // (16 * 128 * 128 * 4)) >= 256              # enough workgroups to fill 256 CUs
    one = L.make_shape(1, 16, 32768, 128, 128, "bf16", segments=1)
    assert L.bidir_scratch_bytes(one) == 16 * 128 * 128 * 4
    assert L.bidir_scratch_bytes(L.make_shape(2, 3, 1, 64, 64, "f32")) == 2 * 3 * 64 * 64 * 4   # N = 1: one partial
    assert L.bidir_scratch_bytes(L.make_shape(1, 4, 100, 64, 64, "bf16", kv_heads=2)) == 0      # no grouped heads here
    assert L.bidir_scratch_bytes(L.make_shape(1, 4, 100, 64, 64, "bf16", kv_heads=4)) > 0
    assert L.bidir_scratch_bytes(L.make_shape(1, 4, 100, 96, 64, "bf16")) == 0
    assert L.bidir_scratch_bytes(L.make_shape(1, 4, 100, 64, 64, "bf16", segments=3)) == 0      # > ceil(100 / 64) tiles


def test_bidir_rejects_before_launch(L):
    s = L.make_shape(1, 2, 100, 64, 64, "bf16")
    sb = L.bidir_scratch_bytes(s)
    x, y, st, scr, q, kv, out, k, v, do, dkv, dq, dk, dv = [_fake(i) for i in range(1, 15)]
    state = lambda *a: L.lib.lasp_bidir_state(*a)
    ok = [ctypes.byref(s), x, y, st, 0, scr, sb, None]
    for idx in (0, 1, 2, 3):
        a = list(ok); a[idx] = None
        assert state(*a) == 1, idx
    a = list(ok); a[5] = None
    assert state(*a) == 5
    a = list(ok); a[6] = sb - 1
    assert state(*a) == 5
    a = list(ok); a[3] = scr
    assert state(*a) == 6                                          # state aliases the scratch
    a = list(ok); a[1] = ctypes.c_void_p(x.value + 2)
    assert state(*a) == 8
    grouped = L.make_shape(1, 2, 100, 64, 64, "bf16", kv_heads=1)
    a = list(ok); a[0] = ctypes.byref(grouped)
    assert state(*a) == 2
    a = list(ok); a[0] = ctypes.byref(L.make_shape(1, 2, 100, 64, 64, 5))
    assert state(*a) == 3

    fwd = lambda *a: L.lib.lasp_bidir_fwd(*a)
    ok = [ctypes.byref(s), q, kv, out, None]
    for idx in (0, 1, 2, 3):
        a = list(ok); a[idx] = None
        assert fwd(*a) == 1, idx
    a = list(ok); a[3] = q
    assert fwd(*a) == 6
    a = list(ok); a[2] = ctypes.c_void_p(kv.value + 4)
    assert fwd(*a) == 8

    bwd = lambda *a: L.lib.lasp_bidir_bwd(*a)
    ok = [ctypes.byref(s), k, v, do, kv, dkv, dq, dk, dv, None]
    for idx in range(9):
        a = list(ok); a[idx] = None
        assert bwd(*a) == 1, idx
    a = list(ok); a[6] = do
    assert bwd(*a) == 6                                            # dq aliases dout
    a = list(ok); a[8] = dk
    assert bwd(*a) == 6                                            # dv aliases dk
    a = list(ok); a[0] = ctypes.byref(L.make_shape(1, 2, 0, 64, 64, "bf16"))
    assert bwd(*a) == 2


# ---------------------------------------------------------------- key and value dimensions that differ
def test_value_dimension_shapes_and_sizes(L):
    base = dict(B=1, H=2, N=256, D=64, chunk=64, dtype="bf16")
    assert L.check_shape(L.make_shape(**base, Dv=0)) == 0
    assert L.check_shape(L.make_shape(**base, Dv=64)) == 0
    assert L.check_shape(L.make_shape(**base, Dv=128)) == 0
    assert L.check_shape(L.make_shape(**base, Dv=96)) == 2
    assert L.check_shape(L.make_shape(**base, Dv=-64)) == 2
    mixed, wide = L.make_shape(**base, Dv=128), L.make_shape(**dict(base, D=128))
    # scratch and the state cache hold [D][Dv] states (the real rows and columns): half of the 128 x 128 shape's
    narrow = L.make_shape(**base)
    assert L.scratch_bytes(wide) == 2 * L.scratch_bytes(mixed) == 4 * L.scratch_bytes(narrow) > 0
    assert L.state_cache_bytes(wide) == 2 * L.state_cache_bytes(mixed) == 4 * L.state_cache_bytes(narrow) > 0
    assert L.tile_tokens(mixed) == L.tile_tokens(wide)


def test_value_dimension_sizes_enter_the_alias_check(L):
    s = L.make_shape(1, 1, 64, 64, 64, "bf16", Dv=128)       # q: 8192 bytes, out: 16384 bytes
    sb = L.scratch_bytes(s)
    q, k, v, kvin, dec, out, kvout, cache, scr = [_fake(i) for i in range(1, 10)]
    inside_out = ctypes.c_void_p(out.value + 16384 - 16)
    assert L.lib.lasp_fwd(ctypes.byref(s), q, k, v, kvin, dec, out, inside_out, cache, scr, sb, None) == 6
    s2 = L.make_shape(1, 1, 64, 128, 64, "bf16", Dv=64)      # q: 16384 bytes
    inside_q = ctypes.c_void_p(q.value + 16384 - 16)
    assert L.lib.lasp_fwd(ctypes.byref(s2), q, k, v, kvin, dec, inside_q, kvout, cache, scr, L.scratch_bytes(s2), None) == 6
    rstd = _fake(11)                                          # the fused Norm accepts the shape: out is still 16384 bytes
    assert L.lib.lasp_fwd_norm(ctypes.byref(s), q, k, v, kvin, dec, ctypes.c_float(1e-5), out, rstd, inside_out, cache,
                               scr, sb, None) == 6
