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


def test_algorithmic_bytes_of_the_benchmark_configurations():
    sys.path.insert(0, ROOT)
    import bench
    import mesa_workloads as W
    spec = W.CONFIGS[2]
    b = bench.algorithmic_bytes(spec, 2)
    n_attn = 128 * 6 * 197 * 197
    n_gelu = 128 * 197 * 1536
    n_ln = n_lin = 128 * 197 * 384
    assert spec.dtype == torch.float16
    assert b["update_attn"] == 2 * n_attn and b["quantize_attn"] == 3 * n_attn
    assert b["softmax_bwd_q"] == 5 * n_attn and b["gelu_bwd_q"] == 5 * n_gelu
    assert b["update_ln0"] == 2 * n_ln and b["quantize_lin0"] == 3 * n_lin
    assert b["dequantize_lin0"] == 3 * n_lin
    assert abs(sum(b.values()) - 949.4e6) < 0.1e6
    # the headline: one DeiT-B-shaped block of the twelve -- two LayerNorms, four Linear layers
    spec = W.CONFIGS[bench.HEADLINE_CONFIG]
    b = bench.algorithmic_bytes(spec, bench.HEADLINE_CONFIG)
    M = 256 * 197
    assert bench.BLOCKS[bench.HEADLINE_CONFIG] == 12 and spec.linears == ((768, 2304), (768, 768), (768, 3072), (3072, 768))
    assert b["softmax_bwd_q"] == 5 * 256 * 12 * 197 * 197 and b["gelu_bwd_q"] == 5 * M * 3072
    assert b["layernorm_bwd_q_ln0"] == b["layernorm_bwd_q_ln1"] == 5 * M * 768 + 8 * M + 10 * 768
    assert b["linear_dw_q_lin2"] == M * 768 + 2 * M * 3072 + 4 * 3072 * 768 + 4 * 3072
    assert b["linear_dw_q_lin3"] == M * 3072 + 2 * M * 768 + 4 * 3072 * 768 + 4 * 768
    assert b["update_lin3"] == 2 * M * 3072 and b["quantize_ln1"] == 3 * M * 768
    assert len(b) == 2 * 8 + 1 + 1 + 2 + 4 + 1
