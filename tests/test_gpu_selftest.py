"""The library's device self-test: the hardware provisions behind the short instruction sequences."""
import pytest

import paper_2602_23349_amd as fo

pytestmark = pytest.mark.gpu


def test_device_selftest_passes():
    status, checked, failed = fo.selftest()
    print("self-test sections (checked / failed):", list(zip(checked, failed)))
    assert status == 0 and sum(failed) == 0
    assert checked[0] == 0x7BFF                      # every positive finite FP16 scale
    assert checked[1] == 1 << 24                     # every d in [1, 4)
    assert checked[2] == 0x7f800000 - 0x0f800000      # every FP32 value in [2^-96, FLT_MAX]
    # code sections: all candidates minus the few inside the tie window
    assert checked[3] > 0.99 * 2 * 14 * (1 << 23)
    # variance codes: 4 values of beta2 x 34 steps (1..20, then log-spaced to 10^6) x 3 group scales
    assert checked[4] > 0.95 * (4 * 34 * 3) * 4 * (1 << 23)
    assert checked[5] == (1 << 30) + (1 << 24)       # short division against IEEE division
    assert checked[6] == checked[5]                  # faithful division on the same operand pairs


def test_faithful_division_is_rarely_inexact():
    # the default AdamW step's division: never more than one ulp off (checked by the self-test), and
    # different from the exactly rounded quotient for about one operand pair in 10^9 (bound asserted here: 1e-7)
    n_div, bad_div = fo.faithful_rounding_stats()
    print(f"faithful division: {bad_div} of {n_div} quotients not exactly rounded ({bad_div / n_div:.2e})")
    assert n_div == (1 << 30) + (1 << 24)
    assert bad_div <= 1e-7 * n_div
