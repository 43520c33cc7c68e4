"""bench.py's host-side pieces (no GPU): the refusal of more than one GPU, the source digest that marks a committed
counter summary as stale, and the summary that is committed."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)


def test_committed_counter_summary_belongs_to_the_committed_sources():
    import bench
    value, src = bench.committed_traffic("resnet50_bf16_b32", "conv_wgrad_bf16_128x128")
    assert value and value > 1e6                                  # bytes per launch of the dominant family
    assert src["kernel_sources_now"] == bench.kernel_sources_digest()
    # a summary taken from other sources than the ones in the tree makes roofline.traffic a stale figure, which
    # bench.py then says in its line; here it is a reason to profile again, not a failure of the library
    if src["stale"]:
        pytest.skip("profiles/resnet50_bf16_b32_hbm_traffic.txt predates a change of the kernel sources: profile again")


def test_a_changed_source_marks_the_summary_stale(tmp_path, monkeypatch):
    import bench
    monkeypatch.setattr(bench, "kernel_sources_digest", lambda: "0" * 16)
    _, src = bench.committed_traffic("resnet50_bf16_b32", "conv_wgrad_bf16_128x128")
    assert src["stale"] is True and src["kernel_sources_now"] == "0" * 16
    at = src["kernel_sources_at_profile"]
    assert len(at) == 16 and all(c in "0123456789abcdef" for c in at)
