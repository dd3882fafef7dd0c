"""The other ways of issuing the FlashAdamW step over the Llama-3.1-8B list that the benchmark times give
the same bits as the one fused call (which tests/test_gpu_llama_full.py holds to the oracle on every element):

  * one call per decoder layer - its nine tensors as one list, the layer's gradients in one reused buffer
    (embedding apart; final norm and head together): 34 calls per step, in reverse order;
  * one call per tensor, alternating between two side streams and two gradient buffers.

Every buffer of the three copies of the state is compared on the device after steps 1 and 2.
"""
import types

import pytest
import torch

import paper_2602_23349_amd as fo
import workloads as W

pytestmark = pytest.mark.gpu

HP = dict(lr=1e-3, wd=0.01, beta1=0.9, beta2=0.999, eps=1e-8)
SEED = 11
GRAD_SCALE = 1e-4
ARRAYS = ("param", "rho", "m_q", "m_scale", "v_q", "v_scale")


def _raw(t):
    return t.view(torch.int16) if t.element_size() == 2 else t.view(torch.int8)


def _grad(sp, i, t):
    return W.grad_bf16(sp, i, t, seed=SEED, device="cuda", dist="normal", scale=GRAD_SCALE)


def _layer_groups(specs):
    groups, cur = [], []
    for i, sp in enumerate(specs):
        layer = sp.name.split(".")[1] if sp.name.startswith("layers.") else sp.name.split(".")[0]
        if cur and cur[0][0] != layer and not (cur[0][0] == "norm" and layer == "lm_head"):
            groups.append([j for _, j in cur])
            cur = []
        cur.append((layer, i))
    groups.append([j for _, j in cur])
    return groups


def test_llama_release_by_layer_and_on_two_streams_equal_the_fused_call():
    specs = W.llama31_8b()
    assert len(specs) == 291
    copies = {"fused": [], "by_layer": [], "two_streams": []}
    for i, sp in enumerate(specs):
        th = W.theta0(sp, i, seed=SEED, device="cuda")
        first = None
        for name, lst in copies.items():
            b = fo.ParamBuffers(sp.numel, "adamw", with_grad=(name == "fused"))
            if first is None:
                fo.split_weights(th, b.param, b.rho)
                first = b
            else:
                b.param.copy_(first.param)
                b.rho.copy_(first.rho)
            b.lr, b.weight_decay = HP["lr"], (HP["wd"] if sp.role == "matrix" else 0.0)
            lst.append(b)
        del th
    fused = fo.TensorList(copies["fused"])

    groups = _layer_groups(specs)
    assert len(groups) == 34 and sorted(j for g in groups for j in g) == list(range(291))
    pad = lambda n: (n + 255) // 256 * 256
    glayer = torch.empty(max(sum(pad(specs[j].numel) for j in g) for g in groups), dtype=torch.bfloat16, device="cuda")
    layer_lists = []
    for idx in groups:
        off, lst = 0, []
        for j in idx:
            b = copies["by_layer"][j]
            lst.append(types.SimpleNamespace(param=b.param, rho=b.rho, grad=glayer[off:off + b.numel], m_q=b.m_q,
                                             m_scale=b.m_scale, v_q=b.v_q, v_scale=b.v_scale, numel=b.numel, lr=b.lr,
                                             weight_decay=b.weight_decay))
            off += pad(b.numel)
        layer_lists.append((idx, lst, fo.TensorList(lst)))

    side = [torch.cuda.Stream(), torch.cuda.Stream()]
    gbufs = [torch.empty(max(s.numel for s in specs), dtype=torch.bfloat16, device="cuda") for _ in side]
    singles = fo.TensorList(copies["two_streams"])
    main = torch.cuda.current_stream()

    for t in (1, 2):
        for i, (sp, b) in enumerate(zip(specs, copies["fused"])):
            b.grad.copy_(_grad(sp, i, t))
        fo.adamw_step_exact(fused, HP["beta1"], HP["beta2"], HP["eps"], t)
        # by layer, last layer first: the layer's gradients become ready, then one call steps its tensors
        for idx, lst, tl in reversed(layer_lists):
            for j, d in zip(idx, lst):
                d.grad.copy_(copies["fused"][j].grad)
            fo.adamw_step_exact(tl, HP["beta1"], HP["beta2"], HP["eps"], t)
        # per tensor on two streams: gradient k goes into buffer k % 2 on stream k % 2, in that stream's order
        for sd in side:
            sd.wait_stream(main)
        for k, i in enumerate(reversed(range(len(specs)))):
            sd, g = side[k % 2], gbufs[k % 2][:specs[i].numel]
            with torch.cuda.stream(sd):
                g.copy_(copies["fused"][i].grad, non_blocking=True)
            singles.set_grad(i, g)
            fo.adamw_step_exact(singles.slice(i), HP["beta1"], HP["beta2"], HP["eps"], t, stream=sd)
        for sd in side:
            main.wait_stream(sd)
        torch.cuda.synchronize()
        for i, sp in enumerate(specs):
            for k in ARRAYS:
                want = _raw(getattr(copies["fused"][i], k))
                for name in ("by_layer", "two_streams"):
                    assert torch.equal(want, _raw(getattr(copies[name][i], k))), (name, t, sp.name, k)
    assert all(bool(b.v_q.any()) for b in copies["fused"][:12])
    del copies, fused, layer_lists, singles, gbufs, glayer
    fo.release_cache()
    torch.cuda.empty_cache()
