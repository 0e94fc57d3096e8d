"""Host-side pieces of bench.py that need no GPU: the one-GPU contract, the flop accounting of a
denoising step, and the rule that the committed HBM counter figure is reported only while the kernel
source it was taken on is unchanged."""
import hashlib
import os
import subprocess
import sys

import bench
from paper_2509_25188_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and not r.stdout.strip()


def test_step_flops_of_the_benched_workload():
    # 32 layers x 512 rows x (4 d^2 + 3 d F) multiply-adds, attention 4 T^2 d per layer, LM head on the block's 32 rows
    w = synth.WORKLOADS["8b_g256"]
    lin, attn, head = bench.step_flops(w)
    d, F, T, L, V = 4096, 12288, 512, 32, 126464
    assert lin == 2.0 * T * L * (4 * d * d + 3 * d * F)
    assert attn == 4.0 * T * T * d * L
    assert head == 2.0 * 32 * d * V
    assert abs((lin + attn + head) / 1e12 - 7.317) < 1e-3        # the figure the bench line reports as step_tflop


def test_hbm_counter_figure_follows_the_kernel_source(tmp_path, monkeypatch):
    with open(bench.GEMM_SOURCE, "rb") as fh:
        sha = hashlib.sha256(fh.read()).hexdigest()
    good = tmp_path / "traffic.txt"
    good.write_text(f"# comment: ignored\nhbm_bytes_per_launch: 247700000\nkernel_source_sha256: {sha}\n")
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(good))
    assert bench.measured_traffic() == 247700000.0
    stale = tmp_path / "stale.txt"
    stale.write_text("hbm_bytes_per_launch: 1\nkernel_source_sha256: 0000\n")
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(stale))
    assert bench.measured_traffic() is None
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(tmp_path / "missing.txt"))
    assert bench.measured_traffic() is None

