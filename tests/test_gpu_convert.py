"""GPU parity of the layout conversion (a standard FP32 optimizer state <-> the compressed layout) against
the oracle's separately pinned codecs: compress = C, Q_m, Q_v; decompress = their inverses."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_23349_amd as fo
import workloads as W
from helpers import bits16, to_dev_u16

pytestmark = pytest.mark.gpu


class _Both:
    """Buffers of both layouts for one tensor."""

    def __init__(self, n, kind):
        c = fo.ParamBuffers(n, kind, with_grad=False)
        f = fo.ParamBuffers(n, kind, with_grad=False, split_weights=False, quantize_states=False)
        for k in ("param", "rho", "m_q", "m_scale", "v_q", "v_scale"):
            setattr(self, k, getattr(c, k))
        self.theta, self.m, self.v = f.theta, f.m, f.v
        self.grad, self.numel, self.kind, self.lr, self.weight_decay, self.flags = None, n, kind, 0.0, 0.0, 3


@pytest.mark.parametrize("kind", ["adamw", "sgd"])
def test_compress_and_decompress_match_oracle(kind):
    specs = W.odd_sizes()
    rng = np.random.default_rng(400)
    bufs, refs = [], []
    for i, sp in enumerate(specs):
        n = sp.numel
        theta = W.theta0(sp, i, seed=31).numpy()
        mag = np.repeat(10.0 ** rng.uniform(-8, -2, (n + 31) // 32), 32)[:n]
        m = (rng.standard_normal(n) * mag).astype(np.float32)
        v = ((rng.standard_t(3, n) * mag) ** 2).astype(np.float32)
        b = _Both(n, kind)
        b.theta.copy_(torch.from_numpy(theta)); b.m.copy_(torch.from_numpy(m))
        if kind == "adamw":
            b.v.copy_(torch.from_numpy(v))
        bufs.append(b); refs.append((theta, m, v))
    fo.compress_state(kind, bufs)
    for b, (theta, m, v), sp in zip(bufs, refs, specs):
        thp, rho = oracle.split(theta)
        mq, ms = oracle.quantize_momentum(m)
        assert np.array_equal(bits16(b.param), thp) and np.array_equal(b.rho.cpu().numpy(), rho), sp.name
        assert np.array_equal(b.m_q.cpu().numpy(), mq) and np.array_equal(bits16(b.m_scale), ms), sp.name
        if kind == "adamw":
            vq, vs = oracle.quantize_variance(v)
            assert np.array_equal(b.v_q.cpu().numpy(), vq) and np.array_equal(bits16(b.v_scale), vs), sp.name
    # and back: overwrite the FP32 side, decompress, compare with the oracle's decoders
    for b in bufs:
        b.theta.fill_(7.0); b.m.fill_(7.0)
        if kind == "adamw":
            b.v.fill_(7.0)
    fo.decompress_state(kind, bufs)
    for b, (theta, m, v) in zip(bufs, refs):
        thp, rho = oracle.split(theta)
        want = oracle.reconstruct(thp, rho)
        assert np.array_equal(b.theta.cpu().numpy().view(np.uint32), want.view(np.uint32))
        mq, ms = oracle.quantize_momentum(m)
        assert np.array_equal(b.m.cpu().numpy().view(np.uint32), oracle.dequantize_momentum(mq, ms).view(np.uint32))
        if kind == "adamw":
            vq, vs = oracle.quantize_variance(v)
            assert np.array_equal(b.v.cpu().numpy().view(np.uint32), oracle.dequantize_variance(vq, vs).view(np.uint32))


def test_compress_then_step_equals_oracle_from_fp32_start():
    # adopt the compressed layout from an FP32 AdamW state mid-training, then keep stepping
    spec = W.ParamSpec("w", (50000,), "matrix")
    ref = oracle.TensorState(W.theta0(spec, 0, seed=32).numpy(), "adamw", split_weights=False, quantize_states=False)
    for t in (1, 2, 3):
        g = W.grad_bf16(spec, 0, t, seed=32)
        oracle.adamw_step(ref, g.view(torch.int16).numpy().view(np.uint16), 1e-3, 0.01, 0.9, 0.999, 1e-8, t)
    b = _Both(spec.numel, "adamw")
    b.theta.copy_(torch.from_numpy(ref.theta32)); b.m.copy_(torch.from_numpy(ref.m32)); b.v.copy_(torch.from_numpy(ref.v32))
    fo.compress_state("adamw", [b])
    st = oracle.TensorState(ref.theta32, "adamw")
    st.mq, st.ms = oracle.quantize_momentum(ref.m32)
    st.vq, st.vs = oracle.quantize_variance(ref.v32)
    b.grad = torch.empty(spec.numel, dtype=torch.bfloat16, device="cuda")
    b.lr, b.weight_decay = 1e-3, 0.01
    for t in (4, 5):
        g = W.grad_bf16(spec, 0, t, seed=32)
        b.grad.copy_(g.cuda())
        fo.adamw_step_exact([b], 0.9, 0.999, 1e-8, t)
        oracle.adamw_step(st, g.view(torch.int16).numpy().view(np.uint16), 1e-3, 0.01, 0.9, 0.999, 1e-8, t)
    assert np.array_equal(bits16(b.param), st.thp) and np.array_equal(b.rho.cpu().numpy(), st.rho)
    assert np.array_equal(b.m_q.cpu().numpy(), st.mq) and np.array_equal(b.v_q.cpu().numpy(), st.vq)
    assert np.array_equal(bits16(b.m_scale), st.ms) and np.array_equal(bits16(b.v_scale), st.vs)
