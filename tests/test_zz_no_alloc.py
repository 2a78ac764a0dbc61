"""The entry point that allocates nothing, lasp_fwd_noalloc (for callers that cannot call hipMalloc
or bring a workspace), against lasp_fwd through the C-ABI: same kernels, so every output must be
bit-identical. Two calls in a row share the library's fixed scratch array; the second is smaller,
so stale contents of the first would show. Collected last: a failure here must not hide other tests."""
import sys

import pytest

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "needs a GPU"
    from paper_2404_02882_amd import harness, lasp, synth_inputs
    return harness, lasp, synth_inputs


def run_pair(gpu, B, H, N, D, chunk, dtype, seed, segments=0):
    import torch
    harness, lasp, si = gpu
    cfg = si.Config("noalloc", B=B, H=H, N=N, D=D, chunk=chunk, dtype=dtype, T=1, seed=seed)
    inp = si.make_inputs(cfg, with_states=True)
    dev = "cuda"
    q, k, v = (harness.to_device(x, dtype, dev) for x in (inp.q, inp.k, inp.v))
    decay = torch.from_numpy(inp.decay).to(dev)
    kv_in = torch.from_numpy(inp.kv_in).to(dev)
    shape = lasp.make_shape(B, H, N, D, chunk, dtype, segments)
    assert lasp.scratch_bytes(shape) <= lasp.noalloc_scratch_limit()
    res = []
    for variant in ("workspace", "noalloc"):
        out = torch.full_like(v, float("nan"))
        kv_out = torch.full((B, H, D, D), float("nan"), dtype=torch.float32, device=dev)
        cache = torch.full((lasp.state_cache_bytes(shape),), 0x7f, dtype=torch.uint8, device=dev)
        if variant == "workspace":
            scratch = torch.full((lasp.scratch_bytes(shape),), 0x7f, dtype=torch.uint8, device=dev)
            lasp.lasp_fwd(shape, q, k, v, kv_in, decay, out, kv_out, cache, scratch)
        else:
            lasp.lasp_fwd_noalloc(shape, q, k, v, kv_in, decay, out, kv_out, cache)
        torch.cuda.synchronize()
        res.append((out, kv_out, cache))
    for name, a, b in zip(("out", "kv_out", "state_cache"), res[0], res[1]):
        same = torch.equal(a.view(torch.uint8).flatten(), b.view(torch.uint8).flatten())
        say(f"  noalloc {dtype} B{B} H{H} N{N} D{D} seg{segments} {name}: {'bit-identical' if same else 'DIFFERS'}")
        assert same, name
    assert not torch.isnan(res[1][0].float()).any() and not torch.isnan(res[1][1]).any()


def test_two_calls_in_a_row_second_smaller(gpu):
    # several segments per head (so the scratch is really used), then a smaller problem on the same array
    run_pair(gpu, 2, 4, 64 * 24, 128, 128, "bf16", seed=4101, segments=6)
    run_pair(gpu, 1, 2, 64 * 6, 64, 64, "bf16", seed=4102, segments=3)
    run_pair(gpu, 1, 2, 32 * 9, 64, 64, "f32", seed=4103, segments=0)
    # a length that is not a multiple of the tile (scratch then also holds the synthesised log decay)
    run_pair(gpu, 1, 3, 64 * 5 + 17, 128, 128, "bf16", seed=4104, segments=2)


def test_rejects_more_scratch_than_the_library_holds(gpu):
    import torch
    harness, lasp, si = gpu
    # 64 heads x 16 segments x 64 KiB = 64 MiB of segment states: over the 32 MiB limit
    shape = lasp.make_shape(4, 16, 64 * 32, 128, 128, "bf16", 16)
    assert lasp.scratch_bytes(shape) > lasp.noalloc_scratch_limit()
    t = torch.zeros(4, 16, 64 * 32, 128, dtype=torch.bfloat16, device="cuda")
    st = torch.zeros(4, 16, 128, 128, dtype=torch.float32, device="cuda")
    decay = torch.ones(16, dtype=torch.float32, device="cuda")
    with pytest.raises(lasp.LaspError) as e:
        lasp.lasp_fwd_noalloc(shape, t, t, t, None, decay, torch.empty_like(t), st, None)
    assert e.value.status == 5   # LASP_ERR_WORKSPACE, before anything was launched
