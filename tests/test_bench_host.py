"""Host-side behaviour of bench.py: the one-GPU contract, the byte accounting behind the roofline figures,
and the parsing of the counter summaries it reads from profiles/."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_per_parameter():
    # Table 1's layout: BF16 weight + INT8 correction, 8-bit states with one FP16 scale per 32 elements,
    # BF16 gradient read once; the ablation variants keep FP32 arrays for the half that is switched off
    assert bench.variant_bytes("adamw", "flash") == 12.25 == bench.BYTES_PER_PARAM["adamw"]
    assert bench.variant_bytes("sgd", "flash") == 10.125 == bench.BYTES_PER_PARAM["sgd"]
    assert bench.variant_bytes("lion", "flash") == 10.125
    assert bench.variant_bytes("adamw", "wsplit") == 6 + 16 + 2
    assert bench.variant_bytes("adamw", "oquant") == 8 + 4.25 + 2
    assert bench.variant_bytes("adamw", "ref") == 8 + 16 + 2
    assert bench.variant_bytes("sgd", "ref") == 8 + 8 + 2


def test_counter_summaries_under_profiles_parse():
    n = 8030261248
    traffic = bench.read_traffic("adamw", "llama31_8b_adamw")
    assert traffic is not None and 0.98 < traffic / (12.25 * n) < 1.05      # no re-reads
    for kind in ("sgd", "lion"):
        t = bench.read_traffic(kind, f"llama31_8b_{kind}")
        assert t is not None and 0.98 < t / (10.125 * n) < 1.05
    assert bench.read_traffic("adamw", "no_such_workload") is None


@pytest.mark.skipif(os.path.exists("/dev/kfd"), reason="a GPU is present")
def test_without_a_gpu_bench_exits_instead_of_falling_back():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True)
    assert r.returncode == 3 and "no CPU fallback" in r.stderr and r.stdout.strip() == ""
