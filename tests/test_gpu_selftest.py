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
    assert checked[2] > (1 << 25)                    # spread values + two full binades
    # code sections: all candidates minus the few inside the tie window
    assert checked[3] > 0.99 * 2 * 14 * (1 << 23)
    assert checked[4] > 0.95 * 15 * 4 * (1 << 23)
    assert checked[5] == (1 << 26) + (1 << 24)       # short division against IEEE division
