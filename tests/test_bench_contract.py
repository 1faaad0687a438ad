"""Host-side contract of bench.py that needs no GPU: more than one GPU is refused with a message, and the
algorithmic byte counts it prices the roofline with follow from the workload's shape."""
import os
import subprocess
import sys

import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout) or "single" in (r.stderr + r.stdout).lower()


def test_algorithmic_bytes_of_the_draft_head():
    sys.path.insert(0, ROOT)
    import bench
    cfg = workloads.get_config(1)
    head, attn, total = bench.algorithmic_bytes(cfg, [2048] * cfg.B, [cfg.max_nodes] * cfg.B)
    # the weights dominate: (V+1) x D bf16 read once
    assert head >= cfg.Vp1 * cfg.D * 2 and head < cfg.Vp1 * cfg.D * 2 * 1.01
    assert attn >= 2 * 2048 * cfg.H * cfg.dh * 2 * cfg.B and total >= head + attn
