"""GPU parity of the standalone codec entry points against the CPU oracle (bit-exact)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_23349_amd as fo
from helpers import bits16, to_dev_u16

pytestmark = pytest.mark.gpu


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def test_reconstruct_every_bf16_and_correction_value():
    # all 65536 BF16 patterns x all 256 correction bytes (incl. the never-produced -128)
    thp = np.repeat(np.arange(1 << 16, dtype=np.uint16), 256)
    rho = np.tile(np.arange(-128, 128, dtype=np.int16).astype(np.int8), 1 << 16)
    out = torch.empty(thp.size, dtype=torch.float32, device="cuda")
    fo.reconstruct_weights(to_dev_u16(thp, torch.bfloat16), _dev(rho), out)
    got = out.cpu().numpy()
    want = oracle.reconstruct(thp, rho)
    fin = np.isfinite(want)
    assert np.array_equal(got.view(np.uint32)[fin], want.view(np.uint32)[fin])
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(got[np.isinf(want)], want[np.isinf(want)])


def _split_inputs():
    rng = np.random.default_rng(100)
    pats = [np.arange(0, 1 << 32, 257, dtype=np.uint64).astype(np.uint32)]
    hi = (np.arange(1 << 16, dtype=np.uint32) << 16)
    for low in (0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x4000, 0xC000):
        pats.append(hi | np.uint32(low))
    pats.append((rng.standard_normal(1 << 20) * 0.02).astype(np.float32).view(np.uint32))
    x = np.concatenate(pats).view(np.float32)
    return x[:x.size - x.size % 4 + 3]     # an odd length: the last block is ragged


def test_split_matches_oracle():
    x = _split_inputs()
    p = torch.empty(x.size, dtype=torch.bfloat16, device="cuda")
    r = torch.empty(x.size, dtype=torch.int8, device="cuda")
    fo.split_weights(_dev(x), p, r)
    thp, rho = oracle.split(x)
    gp, gr = bits16(p), r.cpu().numpy()
    ok = ~np.isnan(x)
    assert np.array_equal(gp[ok], thp[ok])
    assert np.array_equal(gr[ok], rho[ok])      # incl. +-inf and values that round to +-inf: rho = 0
    assert np.all(rho[np.isinf(oracle.bf16_to_f32(thp))] == 0)
    # NaN weights: theta' is a NaN; the correction byte of a NaN is unspecified
    nan_p = gp[~ok]
    assert np.all((nan_p & 0x7F80) == 0x7F80) and np.all((nan_p & 0x7F) != 0)


def _state_inputs(n, seed, heavy):
    rng = np.random.default_rng(seed)
    ng = (n + 31) // 32
    mag = np.repeat(10.0 ** rng.uniform(-9, 2, ng), 32)[:n]
    z = rng.standard_t(3, n) if heavy else rng.standard_normal(n)
    x = (z * mag).astype(np.float32)
    x[:64] = 0.0                      # an all-zero group
    x[64:96] = 2.0 ** -26             # scale underflows FP16: group flushes to zero
    x[96] = 1e7                       # scale saturates at 65504
    x[200:232] = 2.0 ** -20           # FP16-subnormal scale
    return x


@pytest.mark.parametrize("n", [1, 31, 32, 33, 1000, 4096 * 3 + 17, 1 << 20])
def test_quantize_dequantize_momentum(n):
    x = _state_inputs(max(n, 256), 101, heavy=(n % 2 == 0))[:n]
    ng = (n + 31) // 32
    q = torch.empty(n, dtype=torch.int8, device="cuda")
    s = torch.empty(ng, dtype=torch.float16, device="cuda")
    fo.quantize_momentum(_dev(x), q, s)
    wq, ws = oracle.quantize_momentum(x)
    assert np.array_equal(bits16(s), ws)
    assert np.array_equal(q.cpu().numpy(), wq)
    back = torch.empty(n, dtype=torch.float32, device="cuda")
    fo.dequantize_momentum(q, s, back)
    assert np.array_equal(back.cpu().numpy().view(np.uint32), oracle.dequantize_momentum(wq, ws).view(np.uint32))


@pytest.mark.parametrize("n", [1, 31, 32, 33, 1000, 4096 * 3 + 17, 1 << 20])
def test_quantize_dequantize_variance(n):
    x = _state_inputs(max(n, 256), 102, heavy=True)[:n] ** 2
    x = x.astype(np.float32)
    ng = (n + 31) // 32
    q = torch.empty(n, dtype=torch.uint8, device="cuda")
    s = torch.empty(ng, dtype=torch.float16, device="cuda")
    fo.quantize_variance(_dev(x), q, s)
    wq, ws = oracle.quantize_variance(x)
    assert np.array_equal(bits16(s), ws)
    assert np.array_equal(q.cpu().numpy(), wq)
    back = torch.empty(n, dtype=torch.float32, device="cuda")
    fo.dequantize_variance(q, s, back)
    assert np.array_equal(back.cpu().numpy().view(np.uint32), oracle.dequantize_variance(wq, ws).view(np.uint32))


def test_dequantize_every_code_and_scale():
    scales = np.arange(0, 0x7C00, 7, dtype=np.uint16)
    q = np.tile(np.arange(256, dtype=np.int16), scales.size)
    s = np.repeat(scales, 256 // 32)
    out = torch.empty(q.size, dtype=torch.float32, device="cuda")
    fo.dequantize_momentum(_dev(q.astype(np.int8)), to_dev_u16(s, torch.float16), out)
    assert np.array_equal(out.cpu().numpy().view(np.uint32),
                          oracle.dequantize_momentum(q.astype(np.int8), s).view(np.uint32))
    fo.dequantize_variance(_dev(q.astype(np.uint8)), to_dev_u16(s, torch.float16), out)
    assert np.array_equal(out.cpu().numpy().view(np.uint32),
                          oracle.dequantize_variance(q.astype(np.uint8), s).view(np.uint32))


@pytest.mark.parametrize("n", [1, 7, 9, 33, 2047, 2049, 4096 * 3 + 17])
def test_ragged_ends_write_nothing_past_the_end(n):
    # every output buffer carries 64 sentinel elements behind the n the call is given
    pad = 64
    rng = np.random.default_rng(300 + n)
    x = (rng.standard_normal(n) * 0.02).astype(np.float32)
    xd = _dev(x)

    def guarded(dtype, fill):
        return torch.full((n + pad,), fill, dtype=dtype, device="cuda")

    def tail_intact(t, fill):
        return bool((t[n:] == fill).all().item())

    p = guarded(torch.bfloat16, 3.0); r = guarded(torch.int8, 77); r16 = guarded(torch.int16, 7777)
    fo.split_weights(xd, p[:n], r[:n])
    thp, rho = oracle.split(x)
    assert np.array_equal(bits16(p[:n]), thp) and np.array_equal(r[:n].cpu().numpy(), rho)
    assert tail_intact(p, 3.0) and tail_intact(r, 77)
    p2 = guarded(torch.bfloat16, 3.0)
    fo.split_weights_i16(xd, p2[:n], r16[:n])
    thp16, rho16 = oracle.split(x, 32767)
    assert np.array_equal(bits16(p2[:n]), thp16) and np.array_equal(r16[:n].cpu().numpy(), rho16)
    assert tail_intact(p2, 3.0) and tail_intact(r16, 7777)
    th = guarded(torch.float32, 5.0)
    fo.reconstruct_weights(p[:n], r[:n], th[:n])
    assert np.array_equal(th[:n].cpu().numpy().view(np.uint32), oracle.reconstruct(thp, rho).view(np.uint32))
    assert tail_intact(th, 5.0)
    fo.reconstruct_weights_i16(p2[:n], r16[:n], th[:n])
    assert np.array_equal(th[:n].cpu().numpy().view(np.uint32), oracle.reconstruct(thp16, rho16, 32767).view(np.uint32))
    assert tail_intact(th, 5.0)

    ng = (n + 31) // 32
    q = guarded(torch.int8, 55); s = torch.full((ng + pad,), 9.0, dtype=torch.float16, device="cuda")
    fo.quantize_momentum(xd, q[:n], s[:ng])
    wq, ws = oracle.quantize_momentum(x)
    assert np.array_equal(q[:n].cpu().numpy(), wq) and np.array_equal(bits16(s[:ng]), ws)
    assert tail_intact(q, 55) and bool((s[ng:] == 9.0).all().item())
    fo.dequantize_momentum(q[:n], s[:ng], th[:n])
    assert np.array_equal(th[:n].cpu().numpy().view(np.uint32), oracle.dequantize_momentum(wq, ws).view(np.uint32))
    assert tail_intact(th, 5.0)
    v = (x * x).astype(np.float32)
    qu = guarded(torch.uint8, 200)
    fo.quantize_variance(_dev(v), qu[:n], s[:ng])
    wq, ws = oracle.quantize_variance(v)
    assert np.array_equal(qu[:n].cpu().numpy(), wq) and np.array_equal(bits16(s[:ng]), ws)
    assert tail_intact(qu, 200) and bool((s[ng:] == 9.0).all().item())
    fo.dequantize_variance(qu[:n], s[:ng], th[:n])
    assert np.array_equal(th[:n].cpu().numpy().view(np.uint32), oracle.dequantize_variance(wq, ws).view(np.uint32))
    assert tail_intact(th, 5.0)


def test_exact_rounding_ties_take_the_even_code():
    # inputs whose FP32 value before Round() is exactly k + 1/2 (scale 1.0): the device rounds them as the
    # oracle does, in the standalone quantisers
    from helpers import tie_inputs_momentum, tie_inputs_variance
    ms, _ = tie_inputs_momentum()
    vs, _ = tie_inputs_variance()
    for vals, quant_gpu, quant_cpu, dt in ((ms, fo.quantize_momentum, oracle.quantize_momentum, torch.int8),
                                           (vs, fo.quantize_variance, oracle.quantize_variance, torch.uint8)):
        x = np.concatenate([np.array([1.0] + vals[i:i + 31], np.float32) for i in range(0, len(vals), 31)])
        x = np.concatenate([x, np.zeros((-x.size) % 32, np.float32)])
        q = torch.empty(x.size, dtype=dt, device="cuda")
        s = torch.empty(x.size // 32, dtype=torch.float16, device="cuda")
        quant_gpu(_dev(x), q, s)
        wq, ws = quant_cpu(x)
        assert np.array_equal(bits16(s), ws) and np.array_equal(q.cpu().numpy(), wq)


def test_empty_inputs_are_noops():
    e32 = torch.empty(0, dtype=torch.float32, device="cuda")
    fo.split_weights(e32, torch.empty(0, dtype=torch.bfloat16, device="cuda"), torch.empty(0, dtype=torch.int8, device="cuda"))
    fo.quantize_momentum(e32, torch.empty(0, dtype=torch.int8, device="cuda"), torch.empty(0, dtype=torch.float16, device="cuda"))
    torch.cuda.synchronize()
