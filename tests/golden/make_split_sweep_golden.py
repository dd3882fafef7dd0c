#!/usr/bin/env python3
"""Writes tests/golden/split_sweep_oracle.txt: the statistics of the exhaustive FP32 split/reconstruct
experiment (paper Section 4.4) as computed by the CPU oracle over EVERY FP32 bit pattern, for the 8-bit
and the 16-bit correction, under the literal and the directional reading of ULP(theta').  Calls only oracle/.
Takes a few minutes on 8 cores."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402

out = os.path.join(ROOT, "tests", "golden", "split_sweep_oracle.txt")
with open(out, "w") as f:
    f.write("# CPU-oracle statistics of C then C^-1 over all 2^32 FP32 bit patterns (Section 4.4 experiment).\n")
    f.write("# Written by tests/golden/make_split_sweep_golden.py (oracle only).  Per correction width N and per\n")
    f.write("# reading of ULP(theta') (literal = Algorithm 1 as printed; directional = spacing on the side of theta'\n")
    f.write("# where theta lies): scalars, then one line per FP32 exponent field E: mean relative error of the normal\n")
    f.write("# values, then one line per E: bit-exact reconstructions and values measured.\n")
    for reading in ("literal", "directional"):
        for N in (127, 32767):
            d = oracle.split_sweep(0, 1, N, directional=(reading == "directional"))
            f.write(f"N {N} {reading}\n")
            for k in ("measured", "skipped", "interval_violations", "bit_exact", "rho_out_of_range"):
                f.write(f"{k} {int(d[k])}\n")
            f.write(f"max_err_over_bound {d['max_err_over_bound']!r}\n")
            f.write(f"max_rel_err {d['max_rel_err']!r}\n")
            for E, v in enumerate(d["mean_rel_by_exponent"]):
                f.write(f"mean_rel {E} {float(v)!r}\n")
            for E in range(256):
                f.write(f"exact {E} {int(d['bit_exact_by_exponent'][E])} {int(d['count_by_exponent'][E])}\n")
print("wrote", out)
