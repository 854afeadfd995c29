"""bench.py without a GPU: the one-GPU rule and the algorithmic byte counts behind the roofline."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench    # noqa: E402
import synth    # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""           # no JSON line that a reader could mistake for a measurement


def test_algorithmic_bytes_of_the_workloads():
    # one-token draft call: k int4 experts (codes + fp16 scale and zero per group of g inputs) + router + x + y
    phi = synth.config_by_name("phi")
    P = 3 * 4096 * 6400
    int4_expert = P // 2 + (P // 128) * 4
    assert int4_expert == 41_779_200
    nb = bench.algorithmic_bytes(phi, 5, 5.9)
    assert nb["draft_fused_kernel"] == 2 * int4_expert + 16 * 4096 * 2 + 4096 * 2 + 4096 * 4 == 83_714_048
    assert nb["draft_call"] == nb["draft_fused_kernel"]                       # no shared experts
    # verify: |U| distinct bf16 experts once, gate/up two thirds of it
    assert nb["bf16_gateup_kernel"] == 5.9 * (2 * 4096 * 6400 * 2) + 5 * 4096 * 2
    assert nb["bf16_down_kernel"] == 5.9 * (4096 * 6400 * 2) + 5 * 2 * 6400 * 2
    ds = synth.config_by_name("dsv2lite")
    nd = bench.algorithmic_bytes(ds, 6, 28.5)
    Pd = 3 * 2048 * 1408
    assert nd["draft_call"] - nd["draft_fused_kernel"] == 2 * 2 * Pd             # the two bf16 shared experts
    assert abs(nd["draft_call"] / 1e6 - 62.4) < 0.3
    # the symmetric format drops the zeros
    ns = bench.algorithmic_bytes(phi, 5, 5.9, symmetric=True)
    assert nb["draft_fused_kernel"] - ns["draft_fused_kernel"] == 2 * (P // 128) * 2
