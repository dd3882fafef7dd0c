"""flashoptim_adamw_step_noalloc, the FlashAdamW step for callers that cannot allocate device memory, against
flashoptim_adamw_step_exact on the same inputs: every output array bit for bit, on two calls in a row, the
second over a shorter list of smaller tensors (both calls share the one fixed device array that holds the
launch tables, so the second must not see anything of the first)."""
import pytest
import torch

import paper_2602_23349_amd as fo
import workloads as W

pytestmark = pytest.mark.gpu

HP = dict(beta1=0.9, beta2=0.999, eps=1e-8)
ARRAYS = ("param", "rho", "m_q", "m_scale", "v_q", "v_scale")


def _raw(t):
    return t.view(torch.int16) if t.element_size() == 2 else t


def _twin_lists(specs, seed):
    """Two sets of buffers holding the same valid compressed state and the same gradients."""
    a_list, b_list = [], []
    for i, sp in enumerate(specs):
        rs = W.random_state(sp.numel, i, seed=seed, device="cuda")
        g = W.grad_bf16(sp, i, 1, seed=seed, device="cuda", dist="student3", scale=1e-3)
        pair = []
        for _ in range(2):
            b = fo.ParamBuffers(sp.numel, "adamw", with_grad=True)
            b.param.copy_(rs["thp"]); b.rho.copy_(rs["rho"]); b.m_q.copy_(rs["mq"]); b.m_scale.copy_(rs["ms"])
            b.v_q.copy_(rs["vq"]); b.v_scale.copy_(rs["vs"]); b.grad.copy_(g)
            b.lr, b.weight_decay = 1e-3, (0.01 if sp.role == "matrix" else 0.0)
            pair.append(b)
        a_list.append(pair[0]); b_list.append(pair[1])
    return a_list, b_list


def _assert_equal(a_list, b_list, specs, what):
    torch.cuda.synchronize()
    for sp, a, b in zip(specs, a_list, b_list):
        for k in ARRAYS:
            assert torch.equal(_raw(getattr(a, k)), _raw(getattr(b, k))), (what, sp.name, k)


def test_noalloc_step_equals_exact_step_on_two_calls_in_a_row():
    first = W.resnet50()                      # 161 tensors, 25.6 M elements, one ragged
    second = W.odd_sizes()[:12]               # 12 tiny tensors of 1 ... 1000 elements: shorter and smaller
    for call, specs in enumerate((first, second)):
        t = 3 + call
        ref, got = _twin_lists(specs, seed=11 + call)
        fo.adamw_step_noalloc(got, HP["beta1"], HP["beta2"], HP["eps"], t)
        fo.adamw_step_exact(ref, HP["beta1"], HP["beta2"], HP["eps"], t)
        _assert_equal(ref, got, specs, f"call {call}")
        # and once more on the same buffers (state now produced by the kernels themselves)
        fo.adamw_step_noalloc(got, HP["beta1"], HP["beta2"], HP["eps"], t + 1)
        fo.adamw_step_exact(ref, HP["beta1"], HP["beta2"], HP["eps"], t + 1)
        _assert_equal(ref, got, specs, f"call {call}, second step")


def test_noalloc_step_single_tensor_and_limits():
    specs = [W.ParamSpec("w", (300, 1000), "matrix")]
    ref, got = _twin_lists(specs, seed=5)
    fo.adamw_step_noalloc(got, HP["beta1"], HP["beta2"], HP["eps"], 7)
    fo.adamw_step_exact(ref, HP["beta1"], HP["beta2"], HP["eps"], 7)
    _assert_equal(ref, got, specs, "single tensor")
    # more tensors than the fixed table holds: a clear error, nothing enqueued, nothing changed
    many = [W.ParamSpec(f"t{i}", (32,), "matrix") for i in range(1025)]
    ref, got = _twin_lists(many, seed=6)
    with pytest.raises(fo.FlashOptimError) as err:
        fo.adamw_step_noalloc(got, HP["beta1"], HP["beta2"], HP["eps"], 1)
    assert err.value.status == -7 and "1024" in str(err.value)
    _assert_equal(ref, got, many, "rejected call")
    # exactly at the limit it runs
    fo.adamw_step_noalloc(got[:1024], HP["beta1"], HP["beta2"], HP["eps"], 1)
    fo.adamw_step_exact(ref[:1024], HP["beta1"], HP["beta2"], HP["eps"], 1)
    _assert_equal(ref[:1024], got[:1024], many[:1024], "1024 tensors")
