"""Pins for the oracle's companded 8-bit state quantizers (Section 3.2, Eq. 3-4, Algorithms 2-3)."""
import numpy as np

import oracle

G = 32


def _f16(x):
    with np.errstate(over="ignore"):
        return np.asarray(x, np.float32).astype(np.float16)


def _groups(rng, n_groups, scale_lo=-9.0, scale_hi=2.0, heavy=False):
    """Random groups with per-group magnitudes spread log-uniformly."""
    mag = 10.0 ** rng.uniform(scale_lo, scale_hi, size=(n_groups, 1))
    z = rng.standard_t(3, size=(n_groups, G)) if heavy else rng.standard_normal((n_groups, G))
    return (z * mag).astype(np.float32)


# ------------------------------------------------------------------ momentum --

def test_momentum_codes_match_real_number_formula():
    # Eq. 3 / Algorithm 2 in float64 real-number arithmetic: code = round(127 * phi_m(m / s)),
    # phi_m(x) = 2x / (1 + |x|), s = group absmax as stored in FP16.  The FP32 oracle must agree
    # wherever the real value is not within rounding noise of a tie.
    rng = np.random.default_rng(10)
    m = np.concatenate([_groups(rng, 4000), _groups(rng, 4000, heavy=True)])
    q, s_bits = oracle.quantize_momentum(m.ravel())
    q = q.reshape(m.shape).astype(np.int64)
    a = np.abs(m).max(axis=1)
    s = _f16(np.minimum(a, 65504)).astype(np.float64)[:, None]
    assert np.array_equal(s_bits, _f16(np.minimum(a, 65504)).view(np.uint16))
    ok = s[:, 0] > 0
    x = m[ok].astype(np.float64) / s[ok]
    c = 127.0 * (2 * x / (1 + np.abs(x)))
    want = np.clip(np.rint(c), -127, 127)
    safe = np.abs(np.abs(c - np.floor(c)) - 0.5) > 1e-4
    assert safe.mean() > 0.999
    assert np.array_equal(q[ok][safe], want[safe].astype(np.int64))
    assert np.all(np.abs(q[ok] - want) <= 1)
    assert np.all(q[~ok] == 0)


def test_momentum_roundtrip_error_bound():
    # phi_m^-1(z) = z / (2 - |z|) has slope 2 / (2 - |z|)^2; a code is off by at most half a step
    # (1/254 in z), so |m_hat - m| <= s * (1/254) * 2 / (2 - z_hi)^2, which is 2s/255 at |m| = s
    # and s/508 near zero.
    rng = np.random.default_rng(11)
    m = np.concatenate([_groups(rng, 6000, -6, 1), _groups(rng, 2000, -6, 1, heavy=True)])
    q, s_bits = oracle.quantize_momentum(m.ravel())
    back = oracle.dequantize_momentum(q, s_bits).reshape(m.shape).astype(np.float64)
    s = oracle.fp16_to_f32(s_bits).astype(np.float64)[:, None]
    x = np.abs(m.astype(np.float64)) / s
    z = 2 * x / (1 + x)
    z_hi = np.minimum(z + 1 / 254, 1.0)
    bound = s * (1 / 254) * 2 / (2 - z_hi) ** 2
    # the stored scale s is the FP16 rounding of the absmax a: elements above s clamp to code 127
    # and lose up to a - s (<= 2^-11 a for a normal FP16 scale, more for a subnormal one)
    a = np.abs(m.astype(np.float64)).max(axis=1, keepdims=True)
    slack = np.maximum(a - s, 0) + s * 2.0 ** -20 + 1e-30
    err = np.abs(back - m)
    assert np.all(err <= bound + slack)
    assert np.all(err <= (2 / 255) * s * (1 + 2.0 ** -9) + slack)
    # the bound is reached to within 15 %: the codec is not secretly finer or coarser than 8 bits
    assert (err / bound).max() > 0.85
    small = x < 0.02
    assert np.all(err[small] <= (s / 508 * 1.05 + slack)[np.nonzero(small)[0]][:, 0])


def test_momentum_monotone_symmetric_and_extremes():
    rng = np.random.default_rng(12)
    m = _groups(rng, 3000, -8, 3)
    q, s_bits = oracle.quantize_momentum(m.ravel())
    q = q.reshape(m.shape)
    order = np.argsort(m, axis=1, kind="stable")
    assert np.all(np.diff(np.take_along_axis(q.astype(np.int32), order, axis=1), axis=1) >= 0)
    qn, sn = oracle.quantize_momentum((-m).ravel())
    assert np.array_equal(qn.reshape(m.shape), -q) and np.array_equal(sn, s_bits)
    # the absmax element takes code +-127 whenever the scale is a normal FP16 number
    normal = (s_bits >= 0x0400)
    am = np.abs(m).argmax(axis=1)
    top = np.take_along_axis(q, am[:, None], axis=1)[:, 0]
    assert np.all(np.abs(top[normal]) == 127)
    assert q.min() >= -127  # -128 is never produced


def test_momentum_zero_group_and_partial_group():
    q, s = oracle.quantize_momentum(np.zeros(64, np.float32))
    assert not q.any() and not s.any()
    assert not oracle.dequantize_momentum(q, s).any()
    # zero codes with a non-zero scale also decode to exactly zero
    assert not oracle.dequantize_momentum(np.zeros(32, np.int8), np.array([0x3C00], np.uint16)).any()
    # a short last group uses the absmax of its own elements only
    rng = np.random.default_rng(13)
    m = rng.standard_normal(40).astype(np.float32)
    m[35] = 50.0
    q, s = oracle.quantize_momentum(m)
    q0, s0 = oracle.quantize_momentum(m[:32])
    q1, s1 = oracle.quantize_momentum(m[32:])
    assert np.array_equal(q, np.concatenate([q0, q1])) and np.array_equal(s, np.concatenate([s0, s1]))
    assert s.size == 2 and q[35] == 127
    # scale below half the smallest FP16 subnormal flushes the group to zero
    q, s = oracle.quantize_momentum(np.full(32, 2.0 ** -26, np.float32))
    assert not q.any() and s[0] == 0
    # absmax beyond the FP16 range saturates the scale at 65504 and the codes at +-127
    q, s = oracle.quantize_momentum(np.array([1e6, -1e6, 65504.0, 1.0] + [0.0] * 28, np.float32))
    assert s[0] == 0x7BFF and q[0] == 127 and q[1] == -127 and q[2] == 127


def _all_positive_fp16():
    return np.arange(1, 0x7C00, dtype=np.uint16)


def test_momentum_requantize_is_identity_for_every_code_and_scale():
    # Q_m(Q_m^-1(q, s)) = (q, s) for every code and every positive finite FP16 scale, provided
    # the group contains the code 127 (so that its absmax decodes to s itself).
    scales = _all_positive_fp16()
    codes = np.arange(-127, 128, dtype=np.int16)           # 255 codes -> 9 groups of 32 with 127 first
    per = []
    for k in range(9):
        chunk = codes[k * 31:(k + 1) * 31]
        g = np.full(G, 127, np.int16)
        g[1:1 + chunk.size] = chunk
        per.append(g)
    per = np.stack(per).astype(np.int8)                    # (9, 32)
    q = np.tile(per, (scales.size, 1)).ravel()
    s = np.repeat(scales, 9)
    m = oracle.dequantize_momentum(q, s)
    q2, s2 = oracle.quantize_momentum(m)
    assert np.array_equal(s2, s)
    assert np.array_equal(q2, q)


def test_momentum_decode_formula():
    # Algorithm 2, inverse: m = phi_m^-1(q / 127) * s, checked against float64 for all codes.
    q = np.arange(-127, 128).astype(np.int8)
    q = np.concatenate([q, np.zeros(1, np.int8)])
    s_bits = np.repeat(_f16([0.37]).view(np.uint16), 8)
    m = oracle.dequantize_momentum(q, s_bits).astype(np.float64)
    z = q.astype(np.float64) / 127
    want = z / (2 - np.abs(z)) * float(_f16([0.37])[0])
    assert np.allclose(m, want, rtol=3e-7, atol=0)
    assert m[0] == -float(_f16([0.37])[0]) and m[254] == float(_f16([0.37])[0])


# ------------------------------------------------------------------ variance --

def test_variance_codes_match_real_number_formula():
    # Eq. 4 / Algorithm 3 in float64: code = round(255 * sqrt(v) / s), s = FP16(max sqrt(v)).
    rng = np.random.default_rng(20)
    v = np.concatenate([_groups(rng, 4000, -9, 1) ** 2, _groups(rng, 4000, -9, 1, heavy=True) ** 2]).astype(np.float32)
    q, s_bits = oracle.quantize_variance(v.ravel())
    q = q.reshape(v.shape).astype(np.int64)
    r = np.sqrt(v.astype(np.float64))
    a32 = np.sqrt(v).max(axis=1)    # numpy float32 sqrt is correctly rounded
    assert np.array_equal(s_bits, _f16(np.minimum(a32, 65504)).view(np.uint16))
    s = oracle.fp16_to_f32(s_bits).astype(np.float64)[:, None]
    ok = s[:, 0] > 0
    c = 255.0 * r[ok] / s[ok]
    want = np.clip(np.rint(c), 0, 255)
    safe = np.abs(np.abs(c - np.floor(c)) - 0.5) > 1e-4
    assert safe.mean() > 0.999
    assert np.array_equal(q[ok][safe], want[safe].astype(np.int64))
    assert np.all(np.abs(q[ok] - want) <= 1)


def test_variance_roundtrip_error_bound_and_monotone():
    # Linear in sqrt(v): |sqrt(v_hat) - sqrt(v)| <= s / 510.
    rng = np.random.default_rng(21)
    v = (_groups(rng, 6000, -8, 1, heavy=True) ** 2).astype(np.float32)
    q, s_bits = oracle.quantize_variance(v.ravel())
    back = oracle.dequantize_variance(q, s_bits).reshape(v.shape).astype(np.float64)
    s = oracle.fp16_to_f32(s_bits).astype(np.float64)[:, None]
    err = np.abs(np.sqrt(back) - np.sqrt(v.astype(np.float64)))
    a = np.sqrt(v.astype(np.float64)).max(axis=1, keepdims=True)
    slack = np.maximum(a - s, 0) + s * 2.0 ** -20 + 1e-30     # clamp loss above the FP16-rounded scale
    assert np.all(err <= s / 510 * (1 + 1e-3) + slack)
    normal_scale = (s_bits >= 0x0400)
    assert (err[normal_scale] / (s[normal_scale] / 510)).max() > 0.95
    q = q.reshape(v.shape).astype(np.int32)
    order = np.argsort(v, axis=1, kind="stable")
    assert np.all(np.diff(np.take_along_axis(q, order, axis=1), axis=1) >= 0)
    normal = s_bits >= 0x0400
    assert np.all(q.max(axis=1)[normal] == 255)
    # companding keeps small entries alive: an entry is flushed to code 0 only below s/510 in
    # sqrt(v), i.e. below (1/510)^2 of the group maximum in v (a linear code would flush below 1/510)
    vv = v.astype(np.float64)
    flushed = (q == 0) & (vv > 0)
    assert np.all(np.sqrt(vv[flushed]) <= (s / 510 * (1 + 1e-3) + slack + np.zeros_like(vv))[flushed])


def test_variance_requantize_is_identity_for_every_code_and_scale():
    scales = _all_positive_fp16()
    per = np.arange(256, dtype=np.int16).reshape(8, 32)
    per[:, 0] = 255
    per = per.astype(np.uint8)
    # codes 0, 32, 64, ... were overwritten by 255 above; cover them in a ninth group
    extra = np.full(G, 255, np.uint8)
    extra[1:9] = np.arange(0, 256, 32, dtype=np.int16).astype(np.uint8)
    per = np.concatenate([per, extra[None]])
    q = np.tile(per, (scales.size, 1)).ravel()
    s = np.repeat(scales, 9)
    v = oracle.dequantize_variance(q, s)
    q2, s2 = oracle.quantize_variance(v)
    assert np.array_equal(s2, s)
    assert np.array_equal(q2, q)


def test_variance_zero_saturation_and_decode():
    q, s = oracle.quantize_variance(np.zeros(32, np.float32))
    assert not q.any() and s[0] == 0 and not oracle.dequantize_variance(q, s).any()
    q, s = oracle.quantize_variance(np.array([1e12, 65504.0 ** 2, 1.0] + [0.0] * 29, np.float32))
    assert s[0] == 0x7BFF and q[0] == 255 and q[1] == 255 and q[3] == 0
    # Algorithm 3, inverse: v = ((q/255) * s)^2 against float64 for all codes
    codes = np.arange(256, dtype=np.int16).astype(np.uint8)
    s_bits = np.repeat(_f16([0.0123]).view(np.uint16), 8)
    v = oracle.dequantize_variance(codes, s_bits).astype(np.float64)
    want = (codes.astype(np.float64) / 255 * float(_f16([0.0123])[0])) ** 2
    assert np.allclose(v, want, rtol=5e-7, atol=0)


def test_companders_are_inverse_pairs():
    # Section 3.2: both transformations are exactly invertible (checked through the codec:
    # decoding code c then encoding returns c, for a unit scale; and phi_m^-1(phi_m(x)) = x in float64
    # for the function pair the codec was checked against above).
    x = np.linspace(-1, 1, 2001)
    z = 2 * x / (1 + np.abs(x))
    assert np.allclose(z / (2 - np.abs(z)), x, atol=1e-15)
    assert np.abs(z).max() <= 1.0 and np.all(np.diff(z) > 0)


# ------------------------------------------------ linear (no compander) baseline --

def test_linear_quantizers_are_textbook_absmax_quantisation():
    # Section 3.2 / 4.5: the baseline is group-wise absmax scaling to INT8 / UINT8.  Without the
    # compander the code is round(127 m / s) (round(255 v / s)), so |m_hat - m| <= s/254 (s/510).
    rng = np.random.default_rng(30)
    m = _groups(rng, 5000, -6, 1)
    q, s_bits = oracle.quantize_momentum(m.ravel(), linear=True)
    s = oracle.fp16_to_f32(s_bits).astype(np.float64)[:, None]
    a = np.abs(m.astype(np.float64)).max(axis=1, keepdims=True)
    assert np.array_equal(s_bits, _f16(np.minimum(a[:, 0], 65504)).view(np.uint16))
    ok = s[:, 0] > 0
    c = 127.0 * m[ok].astype(np.float64) / s[ok]
    safe = np.abs(np.abs(c - np.floor(c)) - 0.5) > 1e-4
    assert np.array_equal(q.reshape(m.shape)[ok][safe], np.clip(np.rint(c), -127, 127)[safe].astype(np.int8))
    back = oracle.dequantize_momentum(q, s_bits, linear=True).reshape(m.shape).astype(np.float64)
    slack = np.maximum(a - s, 0) + s * 2.0 ** -20 + 1e-30
    assert np.all(np.abs(back - m) <= s / 254 * (1 + 1e-3) + slack)
    v = (_groups(rng, 5000, -8, 1, heavy=True) ** 2).astype(np.float32)
    q, s_bits = oracle.quantize_variance(v.ravel(), linear=True)
    s = oracle.fp16_to_f32(s_bits).astype(np.float64)[:, None]
    a = v.astype(np.float64).max(axis=1, keepdims=True)
    back = oracle.dequantize_variance(q, s_bits, linear=True).reshape(v.shape).astype(np.float64)
    slack = np.maximum(a - s, 0) + s * 2.0 ** -20 + 1e-30
    assert np.all(np.abs(back - v) <= s / 510 * (1 + 1e-3) + slack)
    ok = s[:, 0] > 0
    c = 255.0 * v[ok].astype(np.float64) / s[ok]
    safe = np.abs(np.abs(c - np.floor(c)) - 0.5) > 1e-4
    assert np.array_equal(q.reshape(v.shape)[ok][safe], np.clip(np.rint(c), 0, 255)[safe].astype(np.uint8))


def test_companding_lowers_variance_quantisation_error():
    # Section 4.5: companding gives a large NMSE improvement for variance buffers (heavy-tailed,
    # large dynamic range), measured as sum((x_hat - x)^2) / sum(x^2).  Synthetic stand-in for the
    # paper's training trajectories: v = EMA of squared heavy-tailed gradients.  Linear codes flush
    # everything below 1/510 of the group maximum, which the relative (per-element) error shows.
    rng = np.random.default_rng(31)
    g = rng.standard_t(3, size=(4000, G)) * 1e-3
    v = (0.001 * g * g).astype(np.float32)
    cq, cs = oracle.quantize_variance(v.ravel())
    lq, ls = oracle.quantize_variance(v.ravel(), linear=True)
    cb = oracle.dequantize_variance(cq, cs).astype(np.float64)
    lb = oracle.dequantize_variance(lq, ls, linear=True).astype(np.float64)
    vv = v.ravel().astype(np.float64)
    rel_c = np.abs(cb - vv) / vv
    rel_l = np.abs(lb - vv) / vv
    assert np.median(rel_c) < 0.25 * np.median(rel_l)
    assert (lq == 0).mean() > 3 * (cq == 0).mean()       # linear codes lose far more entries entirely


def test_codes_round_exact_ties_to_even():
    # Reading Q4: when the FP32 value handed to Round() is exactly k + 1/2, the code is the even neighbour.
    # The inputs are found by evaluating the printed operations in numpy FP32 (scale 1.0, so m' = m and
    # v' = sqrt(v)); what is asserted is the tie rule alone.
    from helpers import tie_inputs_momentum, tie_inputs_variance
    ms, want_m = tie_inputs_momentum()
    assert len(ms) >= 60 and any(w % 4 == 0 for w in want_m) and any(w % 4 == 2 for w in want_m)
    for i in range(0, len(ms), 31):                       # groups of 31 ties plus the element 1.0 that fixes the scale
        grp = np.array([1.0] + ms[i:i + 31], np.float32)
        q, s = oracle.quantize_momentum(grp)
        assert s[0] == 0x3C00 and q[0] == 127
        assert list(q[1:]) == want_m[i:i + 31]
    vs, want_v = tie_inputs_variance()
    assert len(vs) >= 60 and any(w % 4 == 0 for w in want_v) and any(w % 4 == 2 for w in want_v)
    for i in range(0, len(vs), 31):
        grp = np.array([1.0] + vs[i:i + 31], np.float32)
        q, s = oracle.quantize_variance(grp)
        assert s[0] == 0x3C00 and q[0] == 255
        assert list(q[1:]) == want_v[i:i + 31]


def test_reciprocal_reading_against_literal_division():
    # Reading Q6: a division by a per-group scale s (Algorithms 2 and 3) or by a bias correction 1 - beta^t
    # (Algorithm 4) is taken as a multiplication by the correctly rounded FP32 reciprocal.  Both the oracle and the
    # GPU follow it, so their comparison cannot see how far it is from the literal division.  This test measures
    # that: the literal form is evaluated here in FP32 (numpy, one rounded operation at a time) for every positive
    # FP16 scale and a sweep of values per scale, and its 8-bit codes are compared with the oracle's.
    f = np.float32
    scales = oracle.fp16_to_f32(_all_positive_fp16())
    scales = scales[scales >= 2.0 ** -24 * 8]                  # at least 3 significant bits in the scale
    rng = np.random.default_rng(5)
    n_codes = n_m_diff = n_v_diff = 0
    max_m = max_v = 0
    for chunk in np.array_split(np.tile(scales, 8), 128):
        # a group per scale (eight different groups for every scale in all): the scale itself (so that the group's stored scale is exactly s) plus 31 fractions of it
        u = rng.uniform(-1.0, 1.0, size=(chunk.size, 32)).astype(np.float32)
        u[:, 0] = 1.0
        m = (u * chunk[:, None]).astype(np.float32)
        q_m, s_m = oracle.quantize_momentum(m.ravel())
        assert np.array_equal(oracle.fp16_to_f32(s_m), chunk)
        m1 = (m / chunk[:, None]).astype(np.float32)                                   # literal m / s
        m2 = ((f(2.0) * m1).astype(np.float32) / (f(1.0) + np.abs(m1)).astype(np.float32)).astype(np.float32)
        lit_m = np.clip(np.rint((m2 * f(127.0)).astype(np.float32)), -127, 127).astype(np.int8)
        d = np.abs(lit_m.astype(np.int32).ravel() - q_m.astype(np.int32))
        n_m_diff += int((d != 0).sum()); max_m = max(max_m, int(d.max()))
        v = (m * m).astype(np.float32)                          # sqrt(v) = |m| up to rounding: group maximum close to s
        q_v, s_v = oracle.quantize_variance(v.ravel())
        sv = oracle.fp16_to_f32(s_v)[:, None]
        ok = sv[:, 0] > 0
        vr = np.sqrt(v, dtype=np.float32)
        with np.errstate(divide="ignore", invalid="ignore"):
            lit_v = np.clip(np.rint(((vr / sv).astype(np.float32) * f(255.0)).astype(np.float32)), 0, 255)
        lit_v = np.where(ok[:, None], lit_v, 0).astype(np.uint8)
        d = np.abs(lit_v.astype(np.int32).ravel() - q_v.astype(np.int32))
        n_v_diff += int((d != 0).sum()); max_v = max(max_v, int(d.max()))
        n_codes += m.size
    rate_m, rate_v = n_m_diff / n_codes, n_v_diff / n_codes
    print(f"literal division vs reciprocal reading over {n_codes} values (256 for each of {scales.size} FP16 scales): "
          f"momentum codes differ on {n_m_diff} ({rate_m:.2e}), variance codes on {n_v_diff} ({rate_v:.2e})")
    # the two forms differ by at most one ulp of m', far below a code step: a code can change only where the
    # argument of Round() sits on a tie to within that ulp, and then by one unit
    assert max_m <= 1 and max_v <= 1
    assert rate_m < 2e-4 and rate_v < 2e-4
    # bias correction: x / bc against x * (1 / bc) in FP32 - how often the quotient itself differs (by one ulp)
    x = rng.standard_normal(1 << 22).astype(np.float32) * f(1e-4)
    worst = 0.0
    for beta, t in ((0.9, 1), (0.9, 7), (0.999, 1), (0.999, 10), (0.999, 1000), (0.99, 100)):
        bc = f(1.0 - beta ** t)
        lit = (x / bc).astype(np.float32)
        rec = (x * (f(1.0) / bc)).astype(np.float32)
        ulps = np.abs(lit.view(np.int32).astype(np.int64) - rec.view(np.int32).astype(np.int64))
        assert ulps.max() <= 1
        worst = max(worst, float((ulps != 0).mean()))
    print(f"bias correction, literal division vs reciprocal: quotients differ (by one ulp) on up to {worst:.1%} of values")
    assert worst < 0.5
