"""The oracle's pins must notice a plausible mistake anywhere in it: each case below plants ONE mistake in
a copy of the oracle's source (on the CPU, in a temporary directory), builds it, and runs the pin tests
against that build in a child process; at least one pin has to fail.  The real oracle is not touched."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

from oracle import build as oracle_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["tests/test_oracle_formats.py", "tests/test_oracle_split.py", "tests/test_oracle_quant.py",
             "tests/test_oracle_steps.py"]

# (what is planted, text in the source, replacement)
MUTANTS = [
    ("bf16 rounding: ties away instead of ties to even", "u += 0x7fffu + lsb;", "u += 0x8000u;"),
    ("half-ULP exponent off by one", "return (E - 127 - 7) - 1;", "return (E - 127 - 7);"),
    ("BF16 has 7 mantissa bits, not 8", "return (E - 127 - 7) - 1;", "return (E - 127 - 8) - 1;"),
    ("sign of the split residual", "float e = theta - bf16_to_f32(thp);", "float e = bf16_to_f32(thp) - theta;"),
    ("scale saturation dropped", "if (a > 65504.0f) a = 65504.0f;", ""),
    ("momentum compander: sign lost in the denominator", "float den = 1.0f + std::fabs(m1);", "float den = 1.0f + m1;"),
    ("momentum expander: wrong sign in the denominator", "float m1 = m2 / (2.0f - std::fabs(m2));",
     "float m1 = m2 / (2.0f + std::fabs(m2));"),
    ("momentum code: round half up instead of half to even", "float y = std::rint(m2 * 127.0f);",
     "float y = std::floor(m2 * 127.0f + 0.5f);"),
    ("variance code: round half up instead of half to even", "float y = std::rint((vr[i] * r) * 255.0f);",
     "float y = std::floor((vr[i] * r) * 255.0f + 0.5f);"),
    ("correction: scaled by N + 1", "*rho_out = (int)std::rint(c * (float)N);", "*rho_out = (int)std::rint(c * (float)(N + 1));"),
    ("reconstruction: correction subtracted", "    return base + e;\n}", "    return base - e;\n}"),
    ("reconstruction: divides by N + 1", "float q = (float)rho / (float)N;", "float q = (float)rho / (float)(N + 1);"),
    ("variance: square root dropped in the encoder", "vr[i] = std::sqrt(v[i]);", "vr[i] = v[i];"),
    ("variance: square dropped in the decoder", "return v1 * v1;", "return v1;"),
    ("directional reading: spacing doubled instead of halved below a power of two",
     "    if (e != 0.0f && below_power_of_two(thp, e < 0.0f)) l -= 1;", "    if (e != 0.0f && below_power_of_two(thp, e < 0.0f)) l += 1;"),
    ("directional reading: decoder ignores the side", "    if (rho != 0 && below_power_of_two(thp, rho < 0)) l -= 1;", ""),
    ("directional reading: side test ignores the sign of theta'", "(error_is_negative != negative);", "error_is_negative;"),
    ("AdamW: beta1 and 1 - beta1 swapped", "float mt = (beta1 * m) + (omb1 * gr);          // m_t",
     "float mt = (omb1 * m) + (beta1 * gr);          // m_t"),
    ("AdamW: gradient not squared", "float gg = gr * gr;", "float gg = gr;"),
    ("AdamW: first bias correction dropped", "float mhat = mt * rbc1;", "float mhat = mt;"),
    ("AdamW: second bias correction dropped", "float vhat = vt * rbc2;", "float vhat = vt;"),
    ("AdamW: epsilon inside the root", "float den = std::sqrt(vhat) + eps;", "float den = std::sqrt(vhat + eps);"),
    ("AdamW: sign of the weight decay", "float upd = (mhat / den) + (wd * th);", "float upd = (mhat / den) - (wd * th);"),
    ("SGD: dampened momentum", "float mt = (momentum * m) + gr;", "float mt = (momentum * m) + (1.0f - momentum) * gr;"),
    ("SGD: weight decay not multiplied by the learning rate", "float tht = th - (lr * (mt + (wd * th)));",
     "float tht = th - (lr * mt + (wd * th));"),
    ("Lion: update direction from the wrong interpolation", "float c = (beta1 * m) + (omb1 * gr);           // b1",
     "float c = (beta2 * m) + (omb2 * gr);           // b1"),
    ("Lion: ascent instead of descent", "float tht = th - (lr * (u + (wd * th)));", "float tht = th + (lr * (u + (wd * th)));"),
]


def _pins_fail_for(case, tmp):
    idx, (what, old, new) = case
    src = open(os.path.join(ROOT, "oracle", "flashoptim_oracle.cpp")).read()
    assert src.count(old) >= 1, f"mutant {idx} ({what}): the text to replace is no longer in the oracle"
    msrc, mlib = os.path.join(tmp, f"mutant{idx}.cpp"), os.path.join(tmp, f"libmutant{idx}.so")
    with open(msrc, "w") as f:
        f.write(src.replace(old, new, 1))
    oracle_build.build(force=True, src=msrc, out=mlib)
    env = dict(os.environ, FLASHOPTIM_ORACLE_LIB=mlib, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        "-k", "not exhaustive and not constant_across"] + PIN_FILES,
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    return what, r.returncode != 0


def test_every_planted_mistake_fails_a_pin(tmp_path):
    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(lambda c: _pins_fail_for(c, str(tmp_path)), enumerate(MUTANTS)))
    survivors = [what for what, failed in results if not failed]
    assert not survivors, f"no pin noticed: {survivors}"
