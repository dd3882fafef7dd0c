"""Full-extent GPU parity of the FlashSGD and FlashLion steps on the Llama-3.1-8B parameter list: EVERY one
of the 8,030,261,248 elements of all 291 tensors is compared with the oracle at steps 1 and 2, one fused call
per step (the configuration of the benchmark's SGD and Lion lines).

Same scheme as the AdamW test next to this one: the oracle's state of both optimizers (4.06 B/param each)
lives in host memory and follows its own trajectory from theta_0; per step the gradients and the GPU's new
state are streamed to the host tensor by tensor through pinned buffers, the oracle steps that tensor on all
host cores, and the four arrays are compared byte for byte.  Asserted: zero differing elements.
"""
import time

import numpy as np
import torch
import pytest

import oracle
import paper_2602_23349_amd as fo
import workloads as W
from test_gpu_llama_full import _Pinned, _count_diff, _np, _threaded

pytestmark = pytest.mark.gpu

HP = {"sgd": dict(lr=1e-2, wd=5e-4, momentum=0.9), "lion": dict(lr=1e-4, wd=0.1, beta1=0.9, beta2=0.99)}
SEED = 5
GRAD_SCALE = 1e-4
ARRAYS = ("param", "rho", "m_q", "m_scale")
ORACLE_FIELD = dict(param="thp", rho="rho", m_q="mq", m_scale="ms")


def _initial_state(theta, kind):
    """theta'_0, rho_0 <- C(theta_0) by the oracle (its scalar routine, on slices from several host threads),
    momentum at Q(0)."""
    n = theta.size
    st = oracle.TensorState(np.zeros(1, np.float32), kind)
    st.n = n
    st.thp, st.rho = np.empty(n, np.uint16), np.empty(n, np.int8)

    def work(lo, hi):
        st.thp[lo:hi], st.rho[lo:hi] = oracle.split(theta[lo:hi])

    _threaded(work, n)
    st.mq, st.ms = np.zeros(n, np.int8), np.zeros((n + 31) // 32, np.uint16)
    return st


def _copy_state(st, kind):
    out = oracle.TensorState(np.zeros(1, np.float32), kind)
    out.n = st.n
    out.thp, out.rho, out.mq, out.ms = st.thp.copy(), st.rho.copy(), st.mq.copy(), st.ms.copy()
    return out


def test_llama_sgd_and_lion_every_element_against_the_oracle():
    t_start = time.perf_counter()
    specs = W.llama31_8b()
    n_total = sum(s.numel for s in specs)
    assert n_total == 8_030_261_248 and len(specs) == 291
    pin = _Pinned(max(s.numel for s in specs))
    bufs = {"sgd": [], "lion": []}
    states = {"sgd": [], "lion": []}
    for i, sp in enumerate(specs):
        th = W.theta0(sp, i, seed=SEED, device="cuda")
        a = fo.ParamBuffers(sp.numel, "sgd", with_grad=True)
        fo.split_weights(th, a.param, a.rho)
        host = [pin.fetch("theta", th), pin.fetch("param", a.param), pin.fetch("rho", a.rho)]
        torch.cuda.synchronize()
        st = _initial_state(host[0].numpy(), "sgd")
        assert _count_diff(_np("param", host[1]), st.thp) == 0, f"split {sp.name}: theta' differs"
        assert _count_diff(_np("rho", host[2]), st.rho) == 0, f"split {sp.name}: rho differs"
        del th
        b = fo.ParamBuffers(sp.numel, "lion", with_grad=False)
        b.param.copy_(a.param)
        b.rho.copy_(a.rho)
        for kind, x in (("sgd", a), ("lion", b)):
            x.lr, x.weight_decay = HP[kind]["lr"], (HP[kind]["wd"] if sp.role == "matrix" else 0.0)
            bufs[kind].append(x)
        states["sgd"].append(st)
        states["lion"].append(_copy_state(st, "lion"))
    lists = {k: fo.TensorList(v) for k, v in bufs.items()}
    for i, a in enumerate(bufs["sgd"]):
        lists["lion"].set_grad(i, a.grad)                     # both optimizers see the same gradients
    print(f"\n[full] initial split of {n_total} weights equal on both sides  ({time.perf_counter() - t_start:.0f} s)")

    for t in (1, 2):
        for i, (sp, a) in enumerate(zip(specs, bufs["sgd"])):
            a.grad.copy_(W.grad_bf16(sp, i, t, seed=SEED, device="cuda", dist="normal", scale=GRAD_SCALE))
        fo.sgd_step(lists["sgd"], HP["sgd"]["momentum"])                       # ONE call, 291 tensors, 30 launches
        fo.lion_step(lists["lion"], HP["lion"]["beta1"], HP["lion"]["beta2"])
        torch.cuda.synchronize()
        differing = {kind: {k: 0 for k in ARRAYS} for kind in bufs}
        for i, sp in enumerate(specs):
            grad = pin.fetch("grad", bufs["sgd"][i].grad)
            for kind in ("sgd", "lion"):
                x, st, hp = bufs[kind][i], states[kind][i], HP[kind]
                host = {k: pin.fetch(k, getattr(x, k)) for k in ARRAYS}
                torch.cuda.synchronize()
                if kind == "sgd":
                    oracle.sgd_step(st, _np("grad", grad), hp["lr"], x.weight_decay, hp["momentum"])
                else:
                    oracle.lion_step(st, _np("grad", grad), hp["lr"], x.weight_decay, hp["beta1"], hp["beta2"])
                for k in ARRAYS:
                    differing[kind][k] += _count_diff(_np(k, host[k]), getattr(st, ORACLE_FIELD[k]))
        for kind in ("sgd", "lion"):
            print(f"[full] t={t}: flashoptim_{kind}_step vs oracle, differing elements of {n_total}: {differing[kind]}"
                  f"  ({time.perf_counter() - t_start:.0f} s)")
        assert not any(v for d in differing.values() for v in d.values()), f"t={t}: {differing}"
    # the states became non-trivial
    for kind in bufs:
        assert all(bool(x.m_q.any()) for x in bufs[kind][:12])
    del bufs, lists, states
    fo.release_cache()
    torch.cuda.empty_cache()
