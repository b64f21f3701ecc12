"""Host-side checks of the benchmark: the multi-GPU refusal and the algorithmic work it prices the roofline with."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench
from paper_2511_10676_amd import configs


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0
    assert "one GPU" in res.stderr and not res.stdout.strip()


def test_algorithmic_work_per_token_and_layer():
    # flops per token and layer F = 2 r (d + E); weight bytes per layer W = 2 r (d + E) in bf16;
    # bytes per layer call B(T) = W + 2 T d + 8 T k (+ 2 E with an output bias)
    want_F = {"deepseek_v2_lite": 8_650_752, "qwen3_30b_a3b": 8_912_896, "phi_mini_moe": 8_421_376, "stress": 18_874_368}
    for name, F in want_F.items():
        w = configs.get(name)
        flops, nbytes = bench.algorithmic_work(w, 1)
        assert flops == F
        assert nbytes == F + 2 * w.d + 8 * w.k + (2 * w.E if w.zipf_bias else 0)
        flops64, nbytes64 = bench.algorithmic_work(w, 64)
        assert flops64 == 64 * F and nbytes64 == F + 64 * (2 * w.d + 8 * w.k) + (2 * w.E if w.zipf_bias else 0)
    ds = configs.get("deepseek_v2_lite")
    assert bench.algorithmic_work(ds, 1)[1] == 8_654_896            # 8.655 MB per layer call at T = 1
    assert bench.algorithmic_work(ds, 8, k=10)[1] == 8_650_752 + 8 * (4096 + 80)


def test_traffic_figures_are_keyed_by_kernel_code():
    assert bench._code_hash("prefill") is not None and bench._code_hash("decode") is not None
    assert bench._code_hash("no_such_kernel") is None
    # a figure is either absent (kernel changed since the counters were read, or never measured) or a byte count
    for path, T in (("prefill", 4096), ("decode", 1), ("decode", 64)):
        v = bench.measured_traffic(path, "deepseek_v2_lite", T)
        assert v is None or v > 1e8
    assert bench.measured_traffic("decode", "deepseek_v2_lite", 2) is None
