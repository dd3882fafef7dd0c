"""Seeded value generators for the synthetic workloads (torch RNG, CPU or GPU).

Every draw is keyed by (seed, tensor index, step, stream) so that any tensor of
any step can be regenerated on its own.  Values drawn on the CPU and on a GPU
differ (different torch generators); a test picks one device and copies.
"""
import math

import torch

_MASK = (1 << 64) - 1


def _mix(x: int) -> int:
    x = (x + 0x9E3779B97F4A7C15) & _MASK
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _MASK
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _MASK
    return x ^ (x >> 31)


def seed_for(seed: int, tensor_index: int, step: int, stream: int) -> int:
    h = _mix(seed & _MASK)
    for v in (tensor_index, step, stream):
        h = _mix(h ^ (v & _MASK))
    return h & ((1 << 62) - 1)


def _gen(device, seed, tensor_index, step, stream):
    g = torch.Generator(device=device)
    g.manual_seed(seed_for(seed, tensor_index, step, stream))
    return g


def to_bits_u16(t: torch.Tensor) -> torch.Tensor:
    """Reinterpret a bf16/fp16 tensor as its 16-bit patterns (int16 storage, same bits)."""
    return t.view(torch.int16)


def from_bits_bf16(t: torch.Tensor) -> torch.Tensor:
    return t.view(torch.bfloat16)


def theta0(spec, tensor_index: int, seed: int = 0, device="cpu", std: float = 0.02) -> torch.Tensor:
    """Initial FP32 master weight of one tensor, flattened."""
    n = spec.numel
    if spec.role == "gain":
        return torch.ones(n, dtype=torch.float32, device=device)
    if spec.role == "bias":
        return torch.zeros(n, dtype=torch.float32, device=device)
    g = _gen(device, seed, tensor_index, 0, 1)
    return torch.randn(n, dtype=torch.float32, device=device, generator=g) * std


def tensor_sigma(tensor_index: int, seed: int = 0, lo: float = 1e-5, hi: float = 1e-2) -> float:
    """Per-tensor gradient scale, log-uniform in [lo, hi]."""
    u = (seed_for(seed, tensor_index, 0, 7) >> 9) / float(1 << 53)
    return 10.0 ** (math.log10(lo) + u * (math.log10(hi) - math.log10(lo)))


def grad_bf16(spec, tensor_index: int, step: int, seed: int = 0, device="cpu",
              dist: str = "normal", scale: float = 1e-3) -> torch.Tensor:
    """BF16 gradient of one tensor at one step, flattened.

    dist = "normal":   scale * N(0,1)
    dist = "student3": scale * Z / sqrt(chi2_3 / 3)   (Student-t, nu = 3: heavy tails)
    """
    n = spec.numel
    g = _gen(device, seed, tensor_index, step, 2)
    z = torch.randn(n, dtype=torch.float32, device=device, generator=g)
    if dist == "normal":
        x = z * scale
    elif dist == "student3":
        c = torch.randn(3, n, dtype=torch.float32, device=device, generator=g)
        x = z / torch.sqrt((c * c).sum(0) / 3.0) * scale
    else:
        raise ValueError(dist)
    return x.to(torch.bfloat16)


def random_state(n: int, tensor_index: int, seed: int = 0, device="cpu", with_variance=True):
    """An arbitrary but valid compressed state for an n-element tensor, drawn directly as
    codes: BF16 weights ~N(0,0.02), rho uniform in [-127,127], momentum codes uniform in
    [-127,127], variance codes uniform in [0,255], FP16 scales log-uniform (momentum around
    1e-4, sqrt-variance around 1e-4).  Useful where a state is needed that neither the oracle
    nor the library produced."""
    g = _gen(device, seed, tensor_index, 0, 3)
    ng = (n + 31) // 32
    thp = (torch.randn(n, dtype=torch.float32, device=device, generator=g) * 0.02).to(torch.bfloat16)
    rho = torch.randint(-127, 128, (n,), dtype=torch.int8, device=device, generator=g)
    mq = torch.randint(-127, 128, (n,), dtype=torch.int8, device=device, generator=g)
    ms = (10.0 ** (torch.rand(ng, device=device, generator=g) * 3.0 - 5.5)).to(torch.float16)
    out = dict(thp=thp, rho=rho, mq=mq, ms=ms)
    if with_variance:
        out["vq"] = torch.randint(0, 256, (n,), dtype=torch.int16, device=device, generator=g).to(torch.uint8)
        out["vs"] = (10.0 ** (torch.rand(ng, device=device, generator=g) * 3.0 - 5.5)).to(torch.float16)
    return out
