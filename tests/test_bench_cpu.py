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
    for wl, d in bench.MEASURED_TRAFFIC.items():
        assert {"arcq_gemm", "arcq_quantize_act"} <= set(d) and all(v > 0 for v in d.values())


def test_profiles_name_their_commands():
    prof = os.path.join(ROOT, "profiles")
    files = [f for f in os.listdir(prof) if f.endswith((".md", ".txt"))]
    assert files
    for f in files:
        text = open(os.path.join(prof, f)).read()
        assert "rocprofv3" in text and "bench.py" in text, f
