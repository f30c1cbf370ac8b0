"""Host-side logic of bench.py that needs no GPU: the one-GPU rule, the byte accounting of a
step, and the guard that ties the stored HBM-counter figure to the kernel sources."""
import os
import subprocess
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode == 2
    assert "one GPU" in p.stderr and p.stdout.strip() == ""


def test_algorithmic_bytes_of_a_step():
    # 3 sessions, gamma = 2, V = 1000, bf16 logits: 9 logits rows, 6 draft rows
    inputs = dict(V=1000, B=3, R_L=9, R_Q=6, logits=torch.zeros((9, 1000), dtype=torch.bfloat16))
    ab = bench.algorithmic_bytes(inputs, 2, C_bonus_fraction=0.25)      # two of the three sessions rejected
    assert ab["row_stats"] == 9 * 1000 * 2                 # every logits row once
    assert ab["residual"] == 2 * 1000 * (2 + 4)            # P row again + Q row, per rejected session
    assert ab["bonus"] == 1 * 1000 * 2 * 0.25              # one chunk of the bonus row
    assert ab["gathers"] == 6 * (4 + 4 + 2) and ab["records"] == 36
    assert ab["total"] == sum(ab[k] for k in ("row_stats", "residual", "bonus", "gathers", "records"))
    half = bench.algorithmic_bytes(inputs, 1.5, C_bonus_fraction=0.25)  # a mean over steps need not be whole
    assert half["residual"] == 1.5 * 1000 * 6 and half["bonus"] == 1.5 * 1000 * 2 * 0.25


def test_traffic_figure_is_tied_to_the_kernel_sources():
    digest = bench.kernel_sources_digest()
    assert len(digest) == 64
    # a stored figure counts only while the sources hash to what it was taken with; otherwise
    # bench.py reports null, which is a legal state, so a mismatch is not a failure here
    for v in bench.PMC_TRAFFIC.values():
        assert len(v["sources_sha256"]) == 64
        assert 0.99 < v["bytes_per_launch"] / (9705 * 256000 * 2) < 1.05
