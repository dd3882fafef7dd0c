"""Randomised GPU parity: random hyper-parameters (incl. extreme betas, step counts, learning rates),
random tensor sizes, and states drawn directly as codes over the whole code range, so that the
estimate-then-certify code paths see every region of their domain."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_23349_amd as fo
import workloads as W
from helpers import ADAMW_MODES, adamw_step_fn, assert_parity, bits16, compare_state, download, upload_state

pytestmark = pytest.mark.gpu


def _random_state(kind, n, idx, seed):
    rs = W.random_state(n, idx, seed=seed, with_variance=(kind == "adamw"))
    st = oracle.TensorState(np.zeros(n, np.float32), kind)
    st.thp = bits16(rs["thp"]); st.rho = rs["rho"].numpy().copy(); st.mq = rs["mq"].numpy().copy()
    st.ms = bits16(rs["ms"])
    if kind == "adamw":
        st.vq = rs["vq"].numpy().copy(); st.vs = bits16(rs["vs"])
    return st


def _cases(n_cases, kinds):
    """(case, mode) pairs: AdamW cases run through both entry points, SGD and Lion have one."""
    return [(c, m) for c in range(n_cases) for m in ADAMW_MODES if kinds[c % 4] == "adamw" or m == "exact"]


_KINDS_SINGLE = ("adamw", "adamw", "sgd", "lion")
_KINDS_LIST = ("adamw", "sgd", "lion", "adamw")


@pytest.mark.parametrize("case,mode", _cases(16, _KINDS_SINGLE))
def test_random_hyperparameters_and_states(case, mode):
    rng = np.random.default_rng(1000 + case)
    kind = _KINDS_SINGLE[case % 4]
    n = int(rng.integers(1, 300000))
    f = lambda v: float(np.float32(v))
    lr = f(10.0 ** rng.uniform(-6, -0.5))
    wd = f(rng.choice([0.0, 10.0 ** rng.uniform(-4, -0.3)]))
    b1 = f(rng.choice([0.0, 0.5, 0.9, 0.99, rng.uniform(0, 0.999)]))
    b2 = f(rng.choice([0.0, 0.9, 0.95, 0.999, 0.9999, rng.uniform(0.5, 0.9999)]))
    eps = f(10.0 ** rng.uniform(-12, -3))
    t0 = int(rng.choice([1, 2, 7, 100, 12345, 10 ** 6]))
    gscale = 10.0 ** rng.uniform(-7, -1)
    st = _random_state(kind, n, case, seed=77)
    buf = upload_state(st)
    buf.lr, buf.weight_decay = lr, wd
    spec = W.ParamSpec("r", (n,), "matrix")
    tl = fo.TensorList([buf])
    report = []
    for t in range(t0, t0 + 3):
        g = W.grad_bf16(spec, case, t, seed=77, dist=("student3" if case % 3 == 0 else "normal"), scale=gscale)
        buf.grad.copy_(g.cuda())
        gb = g.view(torch.int16).numpy().view(np.uint16)
        if kind == "adamw":
            adamw_step_fn(mode)(tl, b1, b2, eps, t)
            oracle.adamw_step(st, gb, lr, wd, b1, b2, eps, t)
        elif kind == "sgd":
            fo.sgd_step(tl, b1)
            oracle.sgd_step(st, gb, lr, wd, b1)
        else:
            fo.lion_step(tl, b1, b2)
            oracle.lion_step(st, gb, lr, wd, b1, b2)
        compare_state(download(buf), st, where=f"case {case} {kind} n={n} t={t}", report=report)
    assert_parity(report, mode, f"{(kind, n, lr, wd, b1, b2, eps, t0, gscale)}")


@pytest.mark.parametrize("case,mode", _cases(8, _KINDS_LIST))
def test_random_lists(case, mode):
    # random lists (2..40 tensors, sizes log-uniform over 1..3M elements, per-tensor lr / weight decay),
    # random code states, three steps through the multi-tensor path
    rng = np.random.default_rng(5000 + case)
    kind = _KINDS_LIST[case % 4]
    n_t = int(rng.integers(2, 41))
    sizes = [int(10.0 ** rng.uniform(0, 6.5)) for _ in range(n_t)]
    f = lambda v: float(np.float32(v))
    b1, b2, eps = f(rng.choice([0.9, 0.95, 0.5])), f(rng.choice([0.999, 0.99, 0.95])), f(10.0 ** rng.uniform(-10, -6))
    sts = [_random_state(kind, n, 100 * case + i, seed=91) for i, n in enumerate(sizes)]
    bufs = [upload_state(s) for s in sts]
    hyper = [(f(10.0 ** rng.uniform(-5, -1.5)), f(rng.choice([0.0, 0.01, 0.1]))) for _ in sizes]
    for b, (lr, wd) in zip(bufs, hyper):
        b.lr, b.weight_decay = lr, wd
    tl = fo.TensorList(bufs)
    report = []
    for t in (1, 2, 3):
        gs = [W.grad_bf16(W.ParamSpec("r", (n,), "matrix"), 100 * case + i, t, seed=91, scale=10.0 ** rng.uniform(-5, -2))
              for i, n in enumerate(sizes)]
        for b, g in zip(bufs, gs):
            b.grad.copy_(g.cuda())
        if kind == "adamw":
            adamw_step_fn(mode)(tl, b1, b2, eps, t)
        elif kind == "sgd":
            fo.sgd_step(tl, b1)
        else:
            fo.lion_step(tl, b1, b2)
        for i, (st, g, (lr, wd)) in enumerate(zip(sts, gs, hyper)):
            gb = g.view(torch.int16).numpy().view(np.uint16)
            if kind == "adamw":
                oracle.adamw_step(st, gb, lr, wd, b1, b2, eps, t)
            elif kind == "sgd":
                oracle.sgd_step(st, gb, lr, wd, b1)
            else:
                oracle.lion_step(st, gb, lr, wd, b1, b2)
            compare_state(download(bufs[i]), st, where=f"list case {case} {kind} tensor {i} n={sizes[i]} t={t}", report=report)
    assert_parity(report, mode, f"{(kind, sizes)}")
