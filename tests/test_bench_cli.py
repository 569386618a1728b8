"""bench.py's contract that can be checked without a GPU: it runs on one GPU only and says so, and its
byte accounting is the per-element figures times the configuration's element counts."""
import os
import subprocess
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    for argv, env in ((["--gpus", "2"], {}), ([], {"WORLD_SIZE": "2"})):
        r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + argv, capture_output=True, text=True,
                           env={**os.environ, **env}, timeout=300)
        assert r.returncode == 2, (argv, env, r.returncode, r.stderr[-300:])
        assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_of_the_headline_configuration():
    sys.path.insert(0, ROOT)
    import bench
    import mesa_workloads as W
    spec = W.CONFIGS[2]
    b = bench.algorithmic_bytes(spec)
    n_attn = 128 * 6 * 197 * 197
    n_gelu = 128 * 197 * 1536
    n_ln = n_lin = 128 * 197 * 384
    assert spec.dtype == torch.float16
    assert b["update_attn"] == 2 * n_attn and b["quantize_attn"] == 3 * n_attn
    assert b["softmax_bwd_q"] == 5 * n_attn and b["gelu_bwd_q"] == 5 * n_gelu
    assert b["update_ln"] == 2 * n_ln and b["quantize_lin"] == 3 * n_lin
    assert b["dequantize_lin"] == 3 * n_lin
    assert abs(sum(b.values()) - 949.4e6) < 0.1e6
