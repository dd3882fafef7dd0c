"""Pins for the oracle's number-format conversions (BF16 and FP16 rounding)."""
import numpy as np
import torch

import oracle


def _all_upper16_with_low(low):
    """Every FP32 pattern whose low 16 bits equal `low` (65536 values)."""
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    return (hi | np.uint32(low)).view(np.float32)


def test_bf16_paper_example(golden_dir):
    # Section 3.1: 1e-5 is representable in BF16 only as 1.0014e-5 (round to nearest);
    # truncation would give 9.9540e-6 instead.
    rows = [l.split() for l in open(f"{golden_dir}/bf16_example.txt") if not l.startswith("#")]
    x, printed, bound = float(rows[0][0]), rows[0][1], float(rows[0][2])
    b = oracle.bf16_rne(np.array([x], np.float32))
    y = float(oracle.bf16_to_f32(b)[0])
    assert f"{y:.4e}" == f"{float(printed):.4e}"
    trunc = (np.array([x], np.float32).view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)[0]
    assert f"{float(trunc):.4e}" != f"{float(printed):.4e}"
    assert abs(y - x) / x <= bound


def test_bf16_relative_error_bound():
    # Section 3.1: 7 mantissa bits guarantee relative error <= 1/256 (normal range).
    rng = np.random.default_rng(0)
    bits = rng.integers(0x00800000, 0x7F000000, size=2_000_000, dtype=np.uint32)
    bits |= rng.integers(0, 2, size=bits.size, dtype=np.uint32) << 31
    x = bits.view(np.float32)
    y = oracle.bf16_to_f32(oracle.bf16_rne(x)).astype(np.float64)
    rel = np.abs(y - x.astype(np.float64)) / np.abs(x.astype(np.float64))
    assert rel.max() <= 1.0 / 256
    assert rel.max() > 1.0 / 600  # round-to-nearest actually reaches close to 2^-9


def test_bf16_matches_library_rounding():
    # Library special case: torch's float32 -> bfloat16 cast is round-to-nearest-even.
    pats = [_all_upper16_with_low(l) for l in (0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x1234, 0xC000)]
    rng = np.random.default_rng(1)
    pats.append(rng.integers(0, 1 << 32, size=4_000_000, dtype=np.uint64).astype(np.uint32).view(np.float32))
    x = np.concatenate(pats)
    x = x[~np.isnan(x)]
    ours = oracle.bf16_rne(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)


def test_bf16_nan_inf():
    x = np.array([np.inf, -np.inf, np.nan, 3.4e38, -3.4e38], np.float32)
    b = oracle.bf16_rne(x)
    assert b[0] == 0x7F80 and b[1] == 0xFF80
    assert (b[2] & 0x7F80) == 0x7F80 and (b[2] & 0x7F) != 0
    assert b[3] == 0x7F80 and b[4] == 0xFF80  # max float rounds up to infinity


def test_fp16_decode_matches_numpy_exhaustively():
    h = np.arange(1 << 16, dtype=np.uint16)
    ours = oracle.fp16_to_f32(h)
    ref = h.view(np.float16).astype(np.float32)
    assert np.array_equal(ours.view(np.uint32)[~np.isnan(ref)], ref.view(np.uint32)[~np.isnan(ref)])
    assert np.isnan(ours[np.isnan(ref)]).all()


def test_fp16_encode_matches_numpy():
    # Library special case: numpy's float32 -> float16 cast is IEEE round-to-nearest-even.
    pats = [_all_upper16_with_low(l) for l in (0x0000, 0x0001, 0x0FFF, 0x1000, 0x1001, 0x2000, 0x3000, 0xFFFF)]
    # every FP32 value that is an FP16 value, a midpoint between two, or one FP32 ulp off either
    h = np.arange(0x7C00, dtype=np.uint16).view(np.float16).astype(np.float64)
    mids = (h[:-1] + h[1:]) / 2
    cand = np.concatenate([h, mids]).astype(np.float32)
    cb = cand.view(np.uint32)
    pats += [cand, (cb + 1).view(np.float32), (cb - 1).view(np.float32), -cand]
    rng = np.random.default_rng(2)
    e = rng.integers(127 - 30, 127 + 18, size=3_000_000, dtype=np.uint32)
    m = rng.integers(0, 1 << 23, size=e.size, dtype=np.uint32)
    pats.append(((e << 23) | m).view(np.float32))
    x = np.concatenate(pats)
    x = x[~np.isnan(x)]
    ours = oracle.fp16_rne(x)
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(ours, ref)
