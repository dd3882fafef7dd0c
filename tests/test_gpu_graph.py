"""The step calls that enqueue kernels only - flashoptim_adamw_step_noalloc over a list, any step call on a single
tensor (the gradient-release call), and an ordinary multi-tensor call whose tables an earlier call has created and
whose descriptors have not changed since - under HIP stream capture: the captured graph is replayed several
times, with eager work and synchronisations in between, and every replay must leave the same bits as the same
calls made eagerly."""
import pytest
import torch

import paper_2602_23349_amd as fo
import workloads as W

pytestmark = pytest.mark.gpu

B1, B2, EPS = 0.9, 0.999, 1e-8
ARRAYS = ("param", "rho", "m_q", "m_scale", "v_q", "v_scale")


def _raw(t):
    return t.view(torch.int16) if t.element_size() == 2 else t


def _twins(specs, seed):
    a_list, b_list = [], []
    for i, sp in enumerate(specs):
        rs = W.random_state(sp.numel, i, seed=seed, device="cuda")
        g = W.grad_bf16(sp, i, 1, seed=seed, device="cuda", scale=1e-3)
        pair = []
        for _ in range(2):
            b = fo.ParamBuffers(sp.numel, "adamw", with_grad=True)
            b.param.copy_(rs["thp"]); b.rho.copy_(rs["rho"]); b.m_q.copy_(rs["mq"]); b.m_scale.copy_(rs["ms"])
            b.v_q.copy_(rs["vq"]); b.v_scale.copy_(rs["vs"]); b.grad.copy_(g)
            b.lr, b.weight_decay = 1e-3, (0.01 if sp.role == "matrix" else 0.0)
            pair.append(b)
        a_list.append(pair[0]); b_list.append(pair[1])
    return a_list, b_list


def _assert_equal(ref, got, what):
    torch.cuda.synchronize()
    for i, (a, b) in enumerate(zip(ref, got)):
        for k in ARRAYS:
            assert torch.equal(_raw(getattr(a, k)), _raw(getattr(b, k))), (what, i, k)


def test_captured_steps_replay_like_eager_calls():
    specs = W.resnet50()[:30] + W.odd_sizes()[:8]
    ref, got = _twins(specs, seed=41)
    tl_ref, tl_got = fo.TensorList(ref), fo.TensorList(got)
    singles = [tl_got.slice(i) for i in (0, 3, 7)]
    # eager warm-up: the library's per-device set-up (the first AdamW call outside a capture puts the check of the
    # short square root on its stream; the fixed table's address is looked up once) and the tables of tl_got
    fo.adamw_step_exact(tl_ref, B1, B2, EPS, 1)
    fo.adamw_step_noalloc(tl_got, B1, B2, EPS, 1)
    fo.adamw_step_exact(tl_ref, B1, B2, EPS, 1)
    fo.adamw_step_exact(tl_got, B1, B2, EPS, 1)                # creates and uploads this list's tables
    _assert_equal(ref, got, "eager warm-up")
    assert fo.short_sqrt_state() in (1, 2)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fo.adamw_step_noalloc(tl_got, B1, B2, EPS, 2)          # multi-tensor launch, tables from kernel arguments
        for s1 in singles:                                     # single-tensor calls: table-free launches
            fo.adamw_step_exact(s1, B1, B2, EPS, 3)
        fo.adamw_step_exact(tl_got, B1, B2, EPS, 4)            # cached tables, unchanged descriptors: kernels only
    for replay in range(3):
        graph.replay()
        fo.adamw_step_exact(tl_ref, B1, B2, EPS, 2)            # the same calls, eagerly
        for i in (0, 3, 7):
            fo.adamw_step_exact(tl_ref.slice(i), B1, B2, EPS, 3)
        fo.adamw_step_exact(tl_ref, B1, B2, EPS, 4)
        _assert_equal(ref, got, f"replay {replay}")
        # eager work of the program itself between the replays
        for b in got:
            b.grad.mul_(-0.5)
        for b in ref:
            b.grad.mul_(-0.5)
        torch.cuda.synchronize()
