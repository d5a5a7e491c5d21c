"""No-GPU checks of bench.py's contract pieces that do not need a device."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_byte_and_flop_counts():
    sys.path.insert(0, ROOT)
    import bench
    # config 5 of the workloads: 469.76 + 121.63 + 15.20 MB for the quantizer, 3985.7 GFLOP for the GEMM
    assert bench.quantizer_bytes(8192, 28672, 1024) == 8192 * (2 * 28672 + 29696 // 2 + 29696 // 16) == 606601216
    assert abs(bench.gemm_flops(8192, 8192, 29696) - 3.9857e12) < 1e9
    assert bench.gemm_bytes(16, 4096, 14592) == (16 + 4096) * (7296 + 912) + 16 * 4096 * 2


def test_traffic_comes_from_the_committed_counter_summary():
    sys.path.insert(0, ROOT)
    import bench
    traffic = bench.load_traffic()
    assert os.path.exists(os.path.join(ROOT, bench.TRAFFIC_FILE))
    assert {"c2_llama8b_q", "c3a_llama8b_up", "c3b_llama8b_down", "c4_qwen32b_mlp", "c5_llama70b_down"} <= set(traffic)
    for wl, d in traffic.items():
        assert {"arcq_gemm", "arcq_quantize_act"} <= set(d) and all(v > 0 for v in d.values())
    # the quantizer moves its algorithmic bytes once: the counters must agree with the byte count within a few per cent
    q = traffic["c5_llama70b_down"]["arcq_quantize_act"]
    assert 0.95 < q / bench.quantizer_bytes(8192, 28672, 1024) < 1.10


def test_verification_sample_touches_every_tile_and_both_ends():
    sys.path.insert(0, ROOT)
    import numpy as np
    import bench
    rng = np.random.default_rng(0)
    idx = bench.sample_indices(8192, 256, 48, rng)
    assert idx[0] == 0 and idx[-1] == 8191 and len(idx) <= 34
    assert {i // 256 for i in idx} == set(range(32))
    idx = bench.sample_indices(27648, 256, 96, rng)
    assert idx[0] == 0 and idx[-1] == 27647 and len(idx) <= 98 and len({i // 256 for i in idx}) >= 96
    assert bench.sample_indices(16, 256, 48, rng)[0] == 0 and bench.sample_indices(1, 256, 48, rng) == [0]


def test_profiles_name_their_commands():
    prof = os.path.join(ROOT, "profiles")
    files = [f for f in os.listdir(prof) if f.endswith((".md", ".txt"))]
    assert files
    for f in files:
        text = open(os.path.join(prof, f)).read()
        assert "rocprofv3" in text and "bench.py" in text, f
