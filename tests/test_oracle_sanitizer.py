"""The oracle under the undefined-behaviour sanitizer: a copy built with -fsanitize=undefined (aborting on
the first finding) must pass its own pins.  Host code only; nothing here touches a GPU."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["tests/test_oracle_formats.py", "tests/test_oracle_split.py", "tests/test_oracle_quant.py",
             "tests/test_oracle_steps.py"]


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_pins_pass_on_a_ubsan_build(tmp_path):
    lib = str(tmp_path / "liboracle_ubsan.so")
    subprocess.run(["g++", "-O1", "-g", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared",
                    "-fPIC", "-fsanitize=undefined", "-fno-sanitize-recover=undefined",
                    os.path.join(ROOT, "oracle", "flashoptim_oracle.cpp"), "-o", lib], check=True)
    env = dict(os.environ, FLASHOPTIM_ORACLE_LIB=lib, OMP_NUM_THREADS="4")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        "-k", "not exhaustive and not constant_across"] + PIN_FILES,
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-3000:]
