"""Host-side contract of bench.py that needs no GPU."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_of_the_update_workload():
    sys.path.insert(0, ROOT)
    import bench
    n, n_pad = 8, 36_500_480
    # (8a)+(8b): read grad, y, x, v_y, z and write y, v_y, z = 32 bytes per element and replica
    assert bench.INNER_B == 32
    assert n * n_pad * bench.INNER_B == 9_344_122_880
    one_inner = bench.algorithmic_bytes(n, n_pad, 1, 0, True)
    assert one_inner == n * n_pad * 32
    # fused outer step: x, z, v_x read, x, v_x, y, z, v_y written per replica, the reference written once
    fused = bench.algorithmic_bytes(n, n_pad, 0, 1, True)
    unfused = bench.algorithmic_bytes(n, n_pad, 0, 1, False)
    assert fused == n * n_pad * 32 + n_pad * 4
    assert unfused - fused == n * n_pad * 4 + n_pad * 4      # the separate mean pass reads x again, (8c) reads x_ref
    assert set(bench.MODEL_WORKLOADS) == {"mlp_n3_fp32", "lenet_n6_fp32", "allcnn_c_n3_bf16", "wrn16_4_n3_bf16",
                                          "wrn28_10_n3_bf16"}
