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


def test_counter_summaries_under_profiles_are_current():
    # the recorded HBM traffic is reported only for the device code it was measured on: a summary whose
    # KERNEL_SOURCE_SHA differs from the tree's is stale and fails here (re-run the counters, then commit)
    n = 8030261248
    traffic, src = bench.read_traffic("adamw", "llama31_8b_adamw", "exact")
    assert src is not None and not src.get("stale"), "profiles/adamw_step_exact_llama31_8b_adamw_pmc.txt is stale"
    assert src["kernel_source_sha"] == bench.kernel_source_sha() and src["recorded_not_measured_in_this_run"]
    assert 0.98 < traffic / (12.25 * n) < 1.05      # no re-reads
    for kind in ("sgd", "lion"):
        t, src = bench.read_traffic(kind, f"llama31_8b_{kind}")
        assert src is not None and not src.get("stale"), f"profiles/{kind}_step_llama31_8b_{kind}_pmc.txt is stale"
        assert 0.98 < t / (10.125 * n) < 1.05
    assert bench.read_traffic("adamw", "no_such_workload") == (None, None)


def test_kernel_label_names_the_real_template_arguments():
    # <KIND, VEC, THREADS, DIRECT, SPLIT, QUANT, EXACT>, as rocprofv3 prints the kernel
    assert bench.kernel_label("adamw", False, True) == "fo::step_kernel<0, 8, 256, false, true, true, true>"
    assert bench.kernel_label("adamw", True, False) == "fo::step_kernel<0, 8, 256, true, true, true, false>"
    assert bench.kernel_label("lion", False, False) == "fo::step_kernel<2, 8, 512, false, true, true, true>"
    assert bench.kernel_label("adamw", False, True, ckpt=True) == "fo::copy_kernel"


@pytest.mark.skipif(os.path.exists("/dev/kfd"), reason="a GPU is present")
def test_without_a_gpu_bench_exits_instead_of_falling_back():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True)
    assert r.returncode == 3 and "no CPU fallback" in r.stderr and r.stdout.strip() == ""
