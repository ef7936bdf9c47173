"""Host-side behaviour of the benchmark driver and of the hooks' shape logic (no GPU needed)."""
from __future__ import annotations

import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode == 2
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_bench_refuses_a_multi_rank_launch():
    env = dict(os.environ, WORLD_SIZE="2", RANK="0")
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, env=env,
                         timeout=120)
    assert res.returncode == 2 and "ONE GPU" in res.stderr


def test_channel_wise_hooks_view_a_tensor_as_outer_channels_inner():
    torch = pytest.importorskip("torch")
    from paper_2510_11400_amd import hooks
    h = hooks.SavedActivations(channel_dim=1)
    assert h._split(torch.empty(8, 32, 7, 7)) == (8, 32, 49, 2)
    assert h._split(torch.empty(40, 96)) == (40, 96, 1, 6)
    assert h._split(torch.empty(5, 8)) == (5, 8, 1, 1)                 # at least one raw-store row
    h = hooks.SavedActivations(channel_dim=-1, raw_share=0.5)
    assert h._split(torch.empty(6, 200, 768)) == (1200, 768, 1, 384)
    assert h._split(torch.empty(4, 20000)) is None                      # more channels than the slot table serves
    assert hooks.SavedActivations()._split(torch.empty(8, 32)) is None  # plain path unless a dimension is named
    h = hooks.SavedActivations(channel_dim=0)
    assert h._split(torch.empty(16, 10, 10)) == (1, 16, 100, 1)
