"""bench.py's byte and flop accounting against figures that can be worked out by hand from the geometries
(the per-step bytes are what the roofline fraction is computed from), and its refusal to run on several GPUs."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench                                    # noqa: E402
from paper_2506_24119_amd import inputs as si   # noqa: E402


def test_step_bytes_of_the_4b_shape():
    g = si.WORKLOADS["C3"].geometry
    # per layer: q/k/v (32 + 2 * 8 heads of 128) x 2560, o 2560 x 4096, gate + up + down 3 x 2560 x 9728
    per_layer = 2560 * 48 * 128 + 2560 * 4096 + 3 * 2560 * 9728
    assert g.params_per_layer() == per_layer == 100_925_440          # the matrices; the 5,376 norm gains are not counted
    weights = (36 * per_layer + 151936 * 2560) * 2
    assert abs(weights - 8.045e9) < 1e6                                   # 8.045 GB of weights per step
    lens = np.full(128, 896, dtype=np.int64)                              # the mean context of the run
    total, kv_launch = bench.algorithmic_bytes(g, lens, 128, fused=False)
    kv_token_layer = 2 * 8 * 128 * 2                                      # K and V, 8 kv heads of 128, 2 bytes
    assert kv_launch == 128 * 896 * kv_token_layer == 469_762_048        # 0.47 GB per attention launch
    want = weights + 36 * kv_launch + 36 * 128 * kv_token_layer + 2 * 128 * 151936 * 4
    assert total == want and abs(total - 25.1e9) < 0.1e9                  # ~25.1 GB, 3.14 ms at 8 TB/s
    fused, _ = bench.algorithmic_bytes(g, lens, 128, fused=True)
    assert total - fused == 2 * 128 * 151936 * 4                          # the logits written and read back


def test_prefill_flops_formula():
    g = si.WORKLOADS["C3"].geometry
    prompts = [np.zeros(3, dtype=np.int32), np.zeros(5, dtype=np.int32)]
    rep = bench.prefill_report(g, prompts, seconds=2.0, score=False)
    mm = 2.0 * 36 * g.params_per_layer() * 8 + 2.0 * 151936 * 2560 * 2   # matmuls on 8 tokens, LM head on 2 rows
    att = 4.0 * 128 * 32 * 36 * (3 * 4 / 2 + 5 * 6 / 2)                   # q.k and p.v over the causal triangle
    assert rep["tokens"] == 8 and abs(rep["tflops"] * 2.0e12 - (mm + att)) < 1e-6 * (mm + att)


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE,
                       stderr=subprocess.STDOUT, text=True, timeout=300)
    assert r.returncode != 0 and "single-GPU" in r.stdout
