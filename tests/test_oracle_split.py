"""Pins for the oracle's weight splitting C / C^-1 (Section 3.1, Eq. 1-2, Algorithm 1)."""
from fractions import Fraction

import numpy as np
import pytest

import oracle

N8 = 127


def _frac(x):
    return Fraction(float(x))


def _ulp_bf16(thp_bits):
    """ULP of a finite BF16 value as an exact Fraction (7 explicit mantissa bits, subnormal
    spacing 2^-133 shared by zero and the lowest binade)."""
    E = (int(thp_bits) >> 7) & 0xFF
    return Fraction(2) ** (max(E, 1) - 134)


def _round_half_even(fr):
    fl = fr.numerator // fr.denominator
    rem = fr - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        return fl + 1
    return fl


@pytest.fixture(scope="module")
def sweep8():
    # every finite FP32 value: the data-independent experiment of Section 4.4
    return oracle.split_sweep(0, 1, N8)


def test_exhaustive_interval_claim(sweep8):
    # Section 3.1: under round-to-nearest theta lies within [theta' - u/2, theta' + u/2].
    assert sweep8["measured"] + sweep8["skipped"] == 2.0 ** 32
    assert sweep8["skipped"] == 2 * (2 ** 23 + 2 ** 15)  # inf/NaN inputs + finite inputs that round to +-inf
    assert sweep8["interval_violations"] == 0
    assert sweep8["not_nearest"] == 0


def test_exhaustive_error_bound(sweep8):
    # Eq. 1-2: [-u/2, u/2] is cut into 2N steps of u/(2N); rounding rho to the nearest step
    # leaves at most half a step, u/(4N), for EVERY finite FP32 value.
    assert sweep8["max_err_over_bound"] <= 1.0
    assert sweep8["max_err_over_bound"] > 0.99      # and the bound is tight
    # relative form: u <= 2^-7 |theta'|, and theta >= theta' (1 - 2^-9) at a power of two
    assert sweep8["max_rel_err"] <= (2.0 ** -9 / 127) / (1 - 2.0 ** -9) * (1 + 1e-9)
    assert sweep8["rho_out_of_range"] == 0


def test_exhaustive_tie_rule_is_immaterial(sweep8):
    # For N = 127 half-to-even and half-away-from-zero give the same rho for every FP32 value.
    assert sweep8["tie_rule_differs"] == 0


def test_error_is_constant_across_normal_range(sweep8):
    # Section 4.4: the 24-bit format has constant error across the normal range, at a level
    # above 1e-6 (comparable to BF16+BF16).
    mr = sweep8["mean_rel_by_exponent"][1:254]
    assert mr.min() > 1e-6
    assert (mr.max() - mr.min()) / mr.mean() < 1e-3
    assert mr.max() < 2.0 ** -9 / 127


def test_int16_variant_level():
    # Section 4.4: with a 16-bit correction the mean relative error is < 1e-9 and reconstruction is
    # bit-exact for almost all values.  (The paper prints 99.92 %; the literal ULP reading used
    # here gives ~99.5 % over all finite FP32 values: the difference is the handling of
    # theta' = 2^k with theta below it, which Algorithm 1 does not distinguish.)
    d = oracle.split_sweep(5, 97, 32767)
    mr = d["mean_rel_by_exponent"][30:254]
    assert mr.max() < 1e-9
    assert d["bit_exact"] / d["measured"] > 0.99
    # u/(4N) is about 2^-17 u here, the same size as half an FP32 ulp (2^-17 u) added by the
    # final rounding of theta_hat, so the total stays below two bound units
    assert d["max_err_over_bound"] <= 2.0
    assert d["rho_out_of_range"] == 0


def _sample_values(rng, n):
    e = rng.integers(1, 254, size=n, dtype=np.uint32)
    m = rng.integers(0, 1 << 23, size=n, dtype=np.uint32)
    s = rng.integers(0, 2, size=n, dtype=np.uint32)
    return ((s << 31) | (e << 23) | m).view(np.float32)


def test_rho_equals_exact_rational_eq1():
    # Eq. 1 evaluated in exact rational arithmetic: rho = round((theta - theta') / (u/2) * N).
    rng = np.random.default_rng(3)
    x = np.concatenate([_sample_values(rng, 3000),
                        np.array([0.0, 1.0, -1.0, 0.02, 1e-30, 1e-38, 1e-40, 1e-45, 3e38, 0.99999994, 1.0000001],
                                 np.float32),
                        (rng.standard_normal(2000) * 0.02).astype(np.float32)])
    thp, rho = oracle.split(x)
    for xi, bi, ri in zip(x, thp, rho):
        tp = _frac(oracle.bf16_to_f32(np.array([bi], np.uint16))[0])
        u = _ulp_bf16(bi)
        assert abs(_frac(xi) - tp) <= u / 2
        want = _round_half_even((_frac(xi) - tp) / (u / 2) * N8)
        assert want == int(ri), (xi, bi, ri, want)


def test_reconstruct_equals_exact_rational_eq2():
    # Eq. 2 in exact arithmetic vs the FP32 evaluation: they differ only by the rounding of
    # rho/N (relative 2^-24 of a term <= u/2) and of the final sum (half an FP32 ulp).
    rng = np.random.default_rng(4)
    thp = rng.integers(0, 0x7F80, size=4000, dtype=np.uint16) | (rng.integers(0, 2, size=4000, dtype=np.uint16) << 15)
    thp = np.concatenate([thp, np.array([0x0000, 0x8000, 0x0001, 0x007F, 0x0080, 0x3F80, 0x7F7F], np.uint16)])
    rho = rng.integers(-127, 128, size=thp.size).astype(np.int8)
    hat = oracle.reconstruct(thp, rho)
    base = oracle.bf16_to_f32(thp)
    for bi, ri, hi, b32 in zip(thp, rho, hat, base):
        u = _ulp_bf16(bi)
        exact = _frac(b32) + Fraction(int(ri), N8) * u / 2
        e32 = (int(np.array([hi], np.float32).view(np.uint32)[0]) >> 23) & 0xFF
        ulp32 = Fraction(2) ** (max(e32, 1) - 150)
        e_exact = abs(Fraction(int(ri), N8) * u / 2)
        e_round = max(e_exact * Fraction(2) ** -23, Fraction(2) ** -150)  # e itself may be subnormal
        assert abs(_frac(hi) - exact) <= ulp32 / 2 + e_round, (bi, ri, hi)


def test_roundtrip_sign_and_order():
    # rho carries the sign of the rounding error: the reconstruction moves from theta' TOWARDS theta.
    rng = np.random.default_rng(5)
    x = _sample_values(rng, 200000)
    thp, rho = oracle.split(x)
    base = oracle.bf16_to_f32(thp).astype(np.float64)
    hat = oracle.reconstruct(thp, rho).astype(np.float64)
    x64 = x.astype(np.float64)
    assert np.all(np.abs(hat - x64) <= np.abs(base - x64))
    moved = rho != 0
    assert np.all(np.sign(hat - base)[moved] == np.sign(x64 - base)[moved])
    assert np.all(np.sign(rho.astype(np.int32))[moved] == np.sign(x64 - base)[moved])
    # average precision gain over plain BF16 is close to 2N = 254
    gain = np.abs(base - x64).mean() / np.abs(hat - x64).mean()
    assert 200 < gain < 300


def test_power_of_two_and_subnormal_cases():
    # theta just below a power of two rounds up to it; its error is at most a quarter of the
    # upper binade's ULP, so the literal ULP reading uses only rho in [-64, 0] there.
    one_minus = np.nextafter(np.float32(1.0), np.float32(0.0))
    thp, rho = oracle.split(np.array([one_minus, 1.0 - 2.0 ** -9, 1.0 + 2.0 ** -8], np.float32))
    assert thp[0] == 0x3F80 and thp[1] in (0x3F80, 0x3F7F)
    assert -64 <= rho[0] <= 0
    # 1 + 2^-8 is the midpoint between 1 and 1 + 2^-7: ties-to-even keeps 1.0 and rho = +127
    assert thp[2] == 0x3F80 and rho[2] == 127
    # the smallest FP32 subnormal: theta' = 0, u = 2^-133, e/(u/2) = 2^-149 / 2^-134 = 2^-15 -> rho = 0
    tiny = np.array([1e-45], np.float32)
    thp, rho = oracle.split(tiny)
    assert thp[0] == 0 and rho[0] == 0
    # half a BF16-subnormal step: e = 2^-134 = u/2 -> tie to even (theta' = 0), rho = +127, exact recovery
    x = np.array([2.0 ** -134], np.float32)
    thp, rho = oracle.split(x)
    assert thp[0] == 0 and rho[0] == 127
    assert oracle.reconstruct(thp, rho)[0] == x[0]
    assert oracle.half_ulp_log2(0x0000) == -134 and oracle.half_ulp_log2(0x0080) == -134
    assert oracle.half_ulp_log2(0x3F80) == -8 and oracle.half_ulp_log2(0x7F7F) == 119


def test_non_finite_inputs():
    x = np.array([np.inf, -np.inf, np.nan, 3.4e38], np.float32)
    thp, rho = oracle.split(x)
    assert np.all(rho == 0)
    hat = oracle.reconstruct(thp, rho)
    assert hat[0] == np.inf and hat[1] == -np.inf and np.isnan(hat[2]) and hat[3] == np.inf
    # rho is ignored for a non-finite theta'
    assert oracle.reconstruct(np.array([0x7F80], np.uint16), np.array([55], np.int8))[0] == np.inf


# ---- the directional reading of ULP(theta') (Section 4.4 experiment only) ----------------------------

def _spacing_on_the_side_of(theta_frac, thp_bits):
    """Distance from theta' to its BF16 neighbour on the side where theta lies, as an exact Fraction,
    found from the BF16 bit patterns themselves (next pattern up or down in magnitude)."""
    b = int(thp_bits)
    tp = _frac(oracle.bf16_to_f32(np.array([b], np.uint16))[0])
    mag = b & 0x7FFF
    away = (theta_frac > tp) == (tp > 0) if tp != 0 else True
    other = mag + 1 if away else mag - 1
    nb = _frac(oracle.bf16_to_f32(np.array([(b & 0x8000) | other], np.uint16))[0])
    return abs(nb - tp)


def test_directional_reading_reaches_the_printed_bit_exact_fraction():
    # Section 4.4 prints 99.92 % bit-exact reconstructions for the 16-bit correction.  Over the
    # mid-range binades the directional reading gives exactly that figure; the literal reading of
    # Algorithm 1 gives 99.73 %.  (Binades near the bottom of the range lose exactness in both
    # readings because the error term itself becomes subnormal.)
    lit = oracle.split_sweep(5, 97, 32767)
    dire = oracle.split_sweep(5, 97, 32767, directional=True)
    mid = slice(40, 250)
    f_lit = lit["bit_exact_by_exponent"][mid].sum() / lit["count_by_exponent"][mid].sum()
    f_dir = dire["bit_exact_by_exponent"][mid].sum() / dire["count_by_exponent"][mid].sum()
    assert round(100 * f_dir, 2) == 99.92
    assert round(100 * f_lit, 2) == 99.73
    assert dire["interval_violations"] == 0 and dire["rho_out_of_range"] == 0
    assert dire["max_err_over_bound"] <= 2.0
    assert (dire["mean_rel_by_exponent"][30:254] <= lit["mean_rel_by_exponent"][30:254] * (1 + 1e-12)).all()


def test_directional_rho_equals_exact_rational_with_the_spacing_of_that_side():
    # rho = round(e / (d/2) * N) with d the BF16 spacing on the side of theta' where theta lies
    rng = np.random.default_rng(13)
    pow2 = (np.float32(2.0) ** rng.integers(-100, 100, size=600)).astype(np.float32)
    near = (pow2 * (1 - rng.uniform(0, 2.0 ** -9, size=600))).astype(np.float32) * rng.choice([-1, 1], size=600)
    x = np.concatenate([_sample_values(rng, 2000), near.astype(np.float32), pow2, -pow2,
                        np.array([0.0, 1e-40, 2.0 ** -126, -(2.0 ** -126) * (1 - 2.0 ** -10), 0.99999994, 1.0000001],
                                 np.float32)])
    for N in (127, 32767):
        thp, rho = oracle.split(x, N=N, directional=True)
        thp_lit, rho_lit = oracle.split(x, N=N)
        assert np.array_equal(thp, thp_lit)
        n_differ = 0
        for xi, bi, ri, rl in zip(x, thp, rho, rho_lit):
            tp = _frac(oracle.bf16_to_f32(np.array([bi], np.uint16))[0])
            e = _frac(xi) - tp
            if e == 0:
                assert int(ri) == 0
                continue
            d = _spacing_on_the_side_of(_frac(xi), bi)
            assert abs(e) <= d / 2
            want = _round_half_even(e / (d / 2) * N)
            # N = 127: the FP32 product e_norm * N is exact; N = 32767: it is rounded (17 x 15 bits), so the
            # code may sit one step beside the exactly rounded one
            assert want == int(ri) if N == 127 else abs(want - int(ri)) <= 1, (xi, bi, ri, want)
            if d != _ulp_bf16(bi):
                n_differ += 1
                assert (int(bi) & 0x7F) == 0                        # only just below a power of two
            else:
                assert int(ri) == int(rl)
        assert n_differ > 300


def test_directional_worked_example_and_round_trip():
    # theta = 1 - 2^-10 rounds to theta' = 1.0 (BF16 spacing 2^-8 below 1, 2^-7 above).  Literal reading:
    # e / (u/2) = -2^-10 / 2^-8 = -1/4, rho = round(-31.75) = -32.  Directional: -2^-10 / 2^-9 = -1/2,
    # rho = round(-63.5) = -64 (half to even); the decoder undoes it with the same spacing.
    x = np.array([1.0 - 2.0 ** -10], np.float32)
    thp, rho = oracle.split(x)
    assert thp[0] == 0x3F80 and rho[0] == -32
    thp, rho = oracle.split(x, directional=True)
    assert thp[0] == 0x3F80 and rho[0] == -64
    hat = oracle.reconstruct(thp, rho, directional=True)
    assert hat[0] == np.float32(1.0) + np.float32(-64.0 / 127.0) * np.float32(2.0 ** -9)
    # round trip error: at most spacing / (4N) plus the two FP32 roundings, for both widths
    rng = np.random.default_rng(14)
    xs = np.concatenate([_sample_values(rng, 20000), (1.0 - rng.uniform(0, 2.0 ** -9, 2000)).astype(np.float32)])
    for N in (127, 32767):
        thp, rho = oracle.split(xs, N=N, directional=True)
        hat = oracle.reconstruct(thp, rho, N=N, directional=True).astype(np.float64)
        E = np.maximum((thp.astype(np.int64) >> 7) & 0xFF, 1)
        u = np.ldexp(1.0, (E - 134).astype(np.int64))
        bound = u / (4 * N) + np.abs(xs.astype(np.float64)) * 2.0 ** -23
        assert (np.abs(hat - xs.astype(np.float64)) <= bound).all()
