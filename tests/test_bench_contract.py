"""Host-side contract of bench.py that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one-GPU" in r.stderr or "must be 1" in r.stderr
    assert r.stdout.strip() == ""                      # no JSON line is printed for a refused run


def test_algorithmic_work_figures():
    """FLOPs per role at config 4 as the scope table derives them (7B target ~32.4 T, 1.5B draft ~7.8 T) and bytes a
    generation position streams (7B: 14.14 GB of bf16 weights)."""
    sys.path.insert(0, ROOT)
    import bench
    import workload as W
    wl = W.get_config("c4_7b")
    M = wl.B * wl.n * wl.L
    ctx = float(sum(int(l) * wl.n * wl.L for l in wl.prefix_lens()))
    f = {r: bench.role_flops(m, M, ctx, wl.n, wl.L, wl.B) / 1e12 for r, m in wl.models().items()}
    assert abs(f["target"] - 32.4) < 0.2 and abs(f["draft"] - 7.8) < 0.1
    assert 28.5 < f["prm"] < 30.2                      # no vocabulary head, last layer for the last tokens only
    assert abs(bench.model_bytes(wl.target) / 1e9 - 14.14) < 0.02
