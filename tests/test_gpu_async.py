"""The enqueue-only convention of the boundary: flashoptim_checkpoint_pack (header, table and sections), the
first step call on a new list (which creates and uploads its device tables) and the first AdamW call of a
process (which puts the check of the short square root on the stream) return while earlier work on the stream
is still running."""
import os
import subprocess
import sys
import time

import numpy as np
import pytest
import torch

import oracle
import paper_2602_23349_amd as fo
import workloads as W
from helpers import bits16, compare_state, download

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


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


def test_first_adamw_call_of_a_process_does_not_wait_for_the_stream():
    # runs in a process of its own: the check of the short square root happens once per process and device
    if os.environ.get("FLASHOPTIM_TEST_FRESH_PROCESS") != "1":
        env = dict(os.environ, FLASHOPTIM_TEST_FRESH_PROCESS="1")
        env.pop("FLASHOPTIM_FORCE_GENERAL_SQRT", None)
        r = subprocess.run([sys.executable, "-u", "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "gpu",
                            os.path.abspath(__file__), "--timeout", "200", "--timeout-method", "thread",
                            "-k", "first_adamw_call_of_a_process"],
                           cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
        assert r.returncode == 0, r.stdout[-3000:]
        assert "1 passed" in r.stdout
        return
    specs = W.odd_sizes()
    hp = dict(beta1=0.9, beta2=0.999, eps=1e-8)
    first, first_states = _state(specs, seed=23)
    other, other_states = _state(specs, seed=24)
    fo.sgd_step([fo.ParamBuffers(64, "sgd")], 0.9)          # library start-up out of the way
    torch.cuda.synchronize()
    assert fo.short_sqrt_state() == 0
    side = torch.cuda.Stream()
    mon = _busy_stream(0.4)
    t0 = time.perf_counter()
    fo.adamw_step_exact(first, hp["beta1"], hp["beta2"], hp["eps"], 2, stream=mon.stream)      # the check goes on the busy stream, then the step
    dt = time.perf_counter() - t0
    # a second stream steps at once: its kernels run before the verdict and take the general square root
    fo.adamw_step_exact(other, hp["beta1"], hp["beta2"], hp["eps"], 2, stream=side)
    side.synchronize()
    still_busy = not mon.stream.query()
    assert still_busy and dt < 0.3, f"step call took {dt:.3f} s on the host; stream busy afterwards: {still_busy}"
    assert fo.short_sqrt_state() == 1                       # waits for the verdict
    mon.stream.synchronize()
    for bufs, states in ((first, first_states), (other, other_states)):
        for i, (b, st, sp) in enumerate(zip(bufs, states, specs)):
            oracle.adamw_step(st, bits16(b.grad), float(np.float32(b.lr)), float(np.float32(b.weight_decay)), hp["beta1"],
                              hp["beta2"], hp["eps"], 2)
            rep = compare_state(download(b), st, where=f"fresh process {sp.name}")
            assert sum(r[1] for r in rep) == 0
