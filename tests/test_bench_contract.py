"""bench.py without a GPU: more than one GPU is refused with a message (this build runs on one device); the flop
counts, the traffic parser and the head-groups adapter."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_world_size_above_one_is_refused():
    env = dict(os.environ, WORLD_SIZE="2", RANK="0")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, timeout=120,
                       env=env)
    assert r.returncode == 2 and "one GPU" in r.stderr


def test_flop_conventions():
    """The three flop counts bench.py reports: the printed algorithm at chunk C (14 C d + 12 d^2 per token-head),
    the causal minimum (10 of 16 blocks of a 128-token chunk), and what the 64-token kernels issue."""
    sys.path.insert(0, ROOT)
    import bench
    f = bench.flop_counts(1, 16, 32768, 128, 128, 128, 64)
    th = 16 * 32768
    assert f["algorithmic"] == th * (14 * 128 * 128 + 12 * 128 * 128)
    assert f["causal_minimal"] == th * (14 * 128 * 128 * 10 / 16 + 12 * 128 * 128)
    assert f["causal_minimal"] < f["issued"] < f["algorithmic"]
    g = bench.flop_counts(2, 8, 4096, 64, 64, 64, 64)     # chunk = tile: 3 of 4 blocks in both counts
    assert g["causal_minimal"] == 2 * 8 * 4096 * (14 * 64 * 64 * 3 / 4 + 12 * 64 * 64)


def test_traffic_is_read_from_the_committed_profiles():
    """roofline.traffic comes from profiles/<config>_fwd_bwd_kernels.md, not from a constant in bench.py."""
    sys.path.insert(0, ROOT)
    import bench
    got, src = bench.traffic_from_profile("c3", "bwd_walk")
    assert src == os.path.join("profiles", "c3_fwd_bwd_kernels.md")
    text = open(os.path.join(ROOT, src)).read()
    table = text[text.index("## HBM traffic per launch"):]
    row = [l for l in table.splitlines() if l.startswith("| `lasp::k_bwd")][0].split("|")
    assert got == int((float(row[3]) + float(row[5])) * 2**20)
    # the backward walk of c3 moves its algorithmic bytes (1792 B per token-head) plus the state cache and start states
    assert 1792 * 16 * 32768 < got < 1.3 * 1792 * 16 * 32768
    assert bench.traffic_from_profile("c3", "fwd_local")[0] != bench.traffic_from_profile("c3", "bwd_local")[0]
    assert bench.traffic_from_profile("no_such_config", "bwd_walk") == (None, None)


def test_head_groups_slice_every_tensor_with_a_head_axis():
    """bench.py --head-groups: the adapter hands each group the head slice of every tensor argument (CPU: a recording
    stand-in for the sequence object, no library call)."""
    import torch
    sys.path.insert(0, ROOT)
    import bench

    class Recorder:
        shape = "shape of a group"

        def __init__(self):
            self.calls = []

        def forward(self, **kw):
            self.calls.append(("fwd", kw))

        def backward(self, **kw):
            self.calls.append(("bwd", kw))

        def cache_bytes(self):
            return 3

        def workspace_bytes(self):
            return 5

    H, made = 6, []
    groups = bench.HeadGroups(3, lambda heads: made.append(heads) or Recorder(), H)
    assert made == [2, 2, 2] and groups.cache_bytes() == 9 and groups.workspace_bytes() == 15
    q = [torch.arange(H * 4.0).reshape(1, H, 4, 1)]
    decay = torch.arange(float(H))
    groups.forward(q=q, decay=decay, rstd=None)
    groups.backward(q=q, decay=decay, dlog_g=None)
    for g, seq in enumerate(groups.seqs):
        (kind_f, f), (kind_b, b) = seq.calls
        assert (kind_f, kind_b) == ("fwd", "bwd")
        assert torch.equal(f["q"][0], q[0][:, 2 * g:2 * g + 2]) and f["q"][0].is_contiguous()
        assert torch.equal(f["decay"], decay[2 * g:2 * g + 2]) and f["rstd"] is None and b["dlog_g"] is None
