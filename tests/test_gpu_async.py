"""The enqueue-only convention of the boundary: flashoptim_checkpoint_pack (header, table and sections) and the
first step call on a new list (which creates and uploads its device tables) return while earlier work on the
stream is still running."""
import time

import numpy as np
import pytest
import torch

import oracle
import paper_2602_23349_amd as fo
import workloads as W
from helpers import bits16

pytestmark = pytest.mark.gpu


def _busy_stream(seconds):
    """A stream kept busy for `seconds` by the library's one-wavefront clock monitor (it ends by itself)."""
    mon = fo.ClockMonitor(n_samples=int(seconds * 1000), seconds_per_sample=1e-3)
    mon.start()
    return mon


def _state(specs, seed):
    bufs, states = [], []
    for i, sp in enumerate(specs):
        rs = W.random_state(sp.numel, i, seed=seed, device="cuda")
        b = fo.ParamBuffers(sp.numel, "adamw", with_grad=True)
        b.param.copy_(rs["thp"]); b.rho.copy_(rs["rho"]); b.m_q.copy_(rs["mq"]); b.m_scale.copy_(rs["ms"])
        b.v_q.copy_(rs["vq"]); b.v_scale.copy_(rs["vs"])
        b.grad.copy_(W.grad_bf16(sp, i, 1, seed=seed, device="cuda"))
        b.lr, b.weight_decay = 1e-3, 0.01
        st = oracle.TensorState(np.zeros(1, np.float32), "adamw")
        st.n = sp.numel
        st.thp = bits16(rs["thp"]); st.rho = rs["rho"].cpu().numpy(); st.mq = rs["mq"].cpu().numpy()
        st.ms = bits16(rs["ms"]); st.vq = rs["vq"].cpu().numpy(); st.vs = bits16(rs["vs"])
        bufs.append(b); states.append(st)
    torch.cuda.synchronize()
    return bufs, states


def test_checkpoint_pack_does_not_wait_for_the_stream():
    specs = W.odd_sizes() + [W.ParamSpec("big", (3_000_000,), "matrix")]
    bufs, states = _state(specs, seed=21)
    size = fo.checkpoint_size("adamw", [s.numel for s in specs])
    blob = torch.full((size,), 0x5A, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    mon = _busy_stream(0.4)
    t0 = time.perf_counter()
    fo.checkpoint_pack("adamw", bufs, 5, blob, stream=mon.stream)          # first call on this list: creates its plan
    fo.checkpoint_pack("adamw", bufs, 6, blob, stream=mon.stream)          # and a second one through the cached plan
    dt = time.perf_counter() - t0
    still_busy = not mon.stream.query()
    mon.stream.synchronize()
    assert still_busy and dt < 0.3, f"pack took {dt:.3f} s on the host; stream busy afterwards: {still_busy}"
    want = oracle.checkpoint_pack("adamw", states, 6)
    assert np.array_equal(blob.cpu().numpy(), want)
    fresh = [fo.ParamBuffers(s.numel, "adamw", with_grad=False) for s in specs]
    assert fo.checkpoint_unpack("adamw", blob, fresh) == 6
    for a, b in zip(bufs, fresh):
        assert torch.equal(a.param.view(torch.int16), b.param.view(torch.int16)) and torch.equal(a.v_q, b.v_q)


def test_first_step_on_a_new_list_does_not_wait_for_the_stream():
    specs = W.odd_sizes()
    bufs, _ = _state(specs, seed=22)
    ref, _ = _state(specs, seed=22)
    fo.sgd_step([fo.ParamBuffers(64, "sgd")], 0.9)          # library start-up out of the way
    fo.adamw_step_exact(ref, 0.9, 0.999, 1e-8, 3)           # (also runs the once-per-device square-root check)
    torch.cuda.synchronize()
    mon = _busy_stream(0.4)
    t0 = time.perf_counter()
    fo.adamw_step_exact(bufs, 0.9, 0.999, 1e-8, 3, stream=mon.stream)      # new list: new device tables
    dt = time.perf_counter() - t0
    still_busy = not mon.stream.query()
    mon.stream.synchronize()
    assert still_busy and dt < 0.3, f"step call took {dt:.3f} s on the host; stream busy afterwards: {still_busy}"
    for a, b in zip(ref, bufs):
        assert torch.equal(a.rho, b.rho) and torch.equal(a.m_q, b.m_q) and torch.equal(a.v_q, b.v_q)
        assert torch.equal(a.param.view(torch.int16), b.param.view(torch.int16))
