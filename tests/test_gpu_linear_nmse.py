"""GPU parity of the linear (no compander) baseline codecs and of the quantisation-error measurement
(paper Section 4.5) against the oracle, on synthetic optimizer-state trajectories that stand in for the
paper's training runs: m and v of an uncompressed AdamW driven by the flat-tensor workload's Gaussian
gradients and by the ResNet-50 workload's heavy-tailed (Student-t) gradients."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_23349_amd as fo
import workloads as W
from helpers import bits16, to_dev_u16

pytestmark = pytest.mark.gpu


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("state", ["momentum", "variance"])
@pytest.mark.parametrize("linear", [False, True])
@pytest.mark.parametrize("n", [1, 33, 1000, 4096 * 5 + 7])
def test_quantize_state_matches_oracle(state, linear, n):
    rng = np.random.default_rng(300 + n)
    mag = np.repeat(10.0 ** rng.uniform(-9, 2, (n + 31) // 32), 32)[:n]
    x = (rng.standard_t(3, n) * mag).astype(np.float32)
    if state == "variance":
        x = (x * x).astype(np.float32)
    x[: min(n, 32)] = 0.0
    qf = oracle.quantize_momentum if state == "momentum" else oracle.quantize_variance
    df = oracle.dequantize_momentum if state == "momentum" else oracle.dequantize_variance
    wq, ws = qf(x, linear=linear)
    q = torch.empty(n, dtype=torch.int8 if state == "momentum" else torch.uint8, device="cuda")
    s = torch.empty((n + 31) // 32, dtype=torch.float16, device="cuda")
    fo.quantize_state(state, linear, _dev(x), q, s)
    assert np.array_equal(bits16(s), ws) and np.array_equal(q.cpu().numpy(), wq)
    back = torch.empty(n, dtype=torch.float32, device="cuda")
    fo.dequantize_state(state, linear, q, s, back)
    assert np.array_equal(back.cpu().numpy().view(np.uint32), df(wq, ws, linear=linear).view(np.uint32))


@pytest.mark.parametrize("dist", ["normal", "student3"])
def test_quantisation_error_on_synthetic_trajectories(dist):
    spec = W.flat_tensor((1 << 18) + 13)[0]
    st = oracle.TensorState(W.theta0(spec, 0, seed=5).numpy(), "adamw", split_weights=False, quantize_states=False)
    rows = []
    for t in range(1, 21):
        g = W.grad_bf16(spec, 0, t, seed=5, dist=dist, scale=1e-3)
        oracle.adamw_step(st, g.view(torch.int16).numpy().view(np.uint16), 1e-3, 0.01, 0.9, 0.999, 1e-8, t)
        if t not in (1, 5, 20):
            continue
        res = {}
        for state, x, qf, df in (("momentum", st.m32, oracle.quantize_momentum, oracle.dequantize_momentum),
                                 ("variance", st.v32, oracle.quantize_variance, oracle.dequantize_variance)):
            xd = _dev(x)
            for linear in (False, True):
                err, ref = fo.quantization_nmse(state, linear, xd)
                q, s = qf(x, linear=linear)
                want = oracle.nmse(x, df(q, s, linear=linear))
                x64 = x.astype(np.float64)
                assert ref == pytest.approx(float(np.dot(x64, x64)), rel=1e-12)
                assert err / ref == pytest.approx(want, rel=1e-9)
                res[(state, linear)] = err / ref
        rows.append((t, res))
        # Section 4.5: companding reduces the error of momentum buffers and greatly reduces that of
        # variance buffers
        assert res[("momentum", False)] < res[("momentum", True)]
        assert res[("variance", False)] < 0.05 * res[("variance", True)]
    for t, r in rows:
        print(f"{dist} t={t}: NMSE momentum companded {r[('momentum', False)]:.3e} linear {r[('momentum', True)]:.3e}; "
              f"variance companded {r[('variance', False)]:.3e} linear {r[('variance', True)]:.3e}")


def test_nmse_of_a_buffer_larger_than_one_pass_of_the_grid():
    # 2048 workgroups x 2048 elements is one pass; this buffer needs three passes and has a ragged end
    n = 2 * 2048 * 2048 + 2048 * 700 + 5
    rng = np.random.default_rng(77)
    x = (rng.standard_normal(n) * np.repeat(10.0 ** rng.uniform(-6, -2, (n + 31) // 32), 32)[:n]).astype(np.float32)
    err, ref = fo.quantization_nmse("momentum", False, _dev(x))
    q, s = oracle.quantize_momentum(x)
    want = oracle.nmse(x, oracle.dequantize_momentum(q, s))
    x64 = x.astype(np.float64)
    assert ref == pytest.approx(float(np.dot(x64, x64)), rel=1e-12)
    assert err / ref == pytest.approx(want, rel=1e-9)


def test_nmse_argument_validation_and_empty():
    assert fo.quantization_nmse("momentum", False, torch.empty(0, dtype=torch.float32, device="cuda")) == (0.0, 0.0)
    L = fo.load_library()
    import ctypes as C
    sums = (C.c_double * 2)()
    assert L.flashoptim_quantization_nmse(2, 0, None, 0, sums, None) == -1
    assert L.flashoptim_quantize_state(0, 3, None, None, None, 0, None) == -1
