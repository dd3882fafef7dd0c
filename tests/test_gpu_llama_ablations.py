"""GPU parity of the AdamW ablation and reference steps (Section 4.3: split weights with FP32 states, FP32
weights with 8-bit states, plain FP32 AdamW with BF16 gradients) at full size: the Llama-3.1-8B parameter
list in one fused call per step, the configuration of the benchmark's ablation lines.

The oracle runs the same two steps with the same flags on SAMPLED groups of 32 elements of every tensor (first
and last group, both sides of the first tile boundaries and of every boundary between two kernel launches of
the call, random groups), fed with copies of the inputs the GPU used.  Every array of the sampled groups is
compared bit for bit, FP32 arrays included.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_23349_amd as fo
import workloads as W
from helpers import bits16

pytestmark = pytest.mark.gpu

HP = dict(lr=1e-3, wd=0.01, beta1=0.9, beta2=0.999, eps=1e-8)
SEED = 7
GRAD_SCALE = 1e-4
N_RANDOM_GROUPS = 12
TILE = 2048                       # elements per workgroup of the AdamW steps
LAUNCH_TILES = (1 << 28) // TILE  # workgroups per kernel launch of a fused call


def _sample_groups(numel, rng, first_tile):
    ng = (numel + 31) // 32
    pick = {0, ng - 1}
    edges = [TILE // 32, 2 * TILE // 32]
    n_tiles = (numel + TILE - 1) // TILE
    k = (first_tile + LAUNCH_TILES - 1) // LAUNCH_TILES
    while k * LAUNCH_TILES < first_tile + n_tiles:
        if k * LAUNCH_TILES > first_tile:
            edges.append((k * LAUNCH_TILES - first_tile) * TILE // 32)
        k += 1
    for edge in edges:
        for g in (edge - 1, edge):
            if 0 <= g < ng:
                pick.add(g)
    pick.update(int(x) for x in rng.integers(0, ng, size=min(N_RANDOM_GROUPS, ng)))
    return np.array(sorted(pick), dtype=np.int64)


def _compare(b, st, e, g, where):
    f32 = lambda t: t[e].cpu().numpy().view(np.uint32)
    if st.split_weights:
        assert np.array_equal(bits16(b.param[e]), st.thp) and np.array_equal(b.rho[e].cpu().numpy(), st.rho), where
    else:
        assert np.array_equal(f32(b.theta), st.theta32.view(np.uint32)), where
    if st.quantize_states:
        assert np.array_equal(b.m_q[e].cpu().numpy(), st.mq) and np.array_equal(bits16(b.m_scale[g]), st.ms), where
        assert np.array_equal(b.v_q[e].cpu().numpy(), st.vq) and np.array_equal(bits16(b.v_scale[g]), st.vs), where
    else:
        assert np.array_equal(f32(b.m), st.m32.view(np.uint32)), where
        assert np.array_equal(f32(b.v), st.v32.view(np.uint32)), where


@pytest.mark.parametrize("split,quant", [(True, False), (False, True), (False, False)])
def test_llama_adamw_ablation_steps_sampled_parity(split, quant):
    specs = W.llama31_8b()
    assert sum(s.numel for s in specs) == 8_030_261_248 and len(specs) == 291
    rng = np.random.default_rng(77)
    bufs, states, eidx, gidx = [], [], [], []
    first = 0
    for i, sp in enumerate(specs):
        groups = _sample_groups(sp.numel, rng, first)
        first += (sp.numel + TILE - 1) // TILE
        gi = torch.from_numpy(groups).cuda()
        e = (gi[:, None] * 32 + torch.arange(32, device="cuda")[None, :]).reshape(-1)
        assert int(e.max()) < sp.numel                                 # every tensor of the list is a multiple of 32
        eidx.append(e)
        gidx.append(gi)
        b = fo.ParamBuffers(sp.numel, "adamw", with_grad=True, split_weights=split, quantize_states=quant)
        th = W.theta0(sp, i, seed=SEED, device="cuda")
        if split:
            fo.split_weights(th, b.param, b.rho)
        else:
            b.theta.copy_(th)
        states.append(oracle.TensorState(th[e].cpu().numpy(), "adamw", split_weights=split, quantize_states=quant))
        del th
        b.lr, b.weight_decay = HP["lr"], (HP["wd"] if sp.role == "matrix" else 0.0)
        bufs.append(b)
    assert (first + LAUNCH_TILES - 1) // LAUNCH_TILES == 30
    tl = fo.TensorListEx(bufs)
    for t in (1, 2):
        for i, (sp, b) in enumerate(zip(specs, bufs)):
            b.grad.copy_(W.grad_bf16(sp, i, t, seed=SEED, device="cuda", dist="normal", scale=GRAD_SCALE))
            oracle.adamw_step(states[i], bits16(b.grad[eidx[i]]), HP["lr"], b.weight_decay, HP["beta1"], HP["beta2"],
                              HP["eps"], t)
        fo.adamw_step_ex(tl, HP["beta1"], HP["beta2"], HP["eps"], t)           # ONE call, 291 tensors, 30 launches
        torch.cuda.synchronize()
        for i, (sp, b) in enumerate(zip(specs, bufs)):
            _compare(b, states[i], eidx[i], gidx[i], f"split={split} quant={quant} t={t} {sp.name}")
    n = sum(int(e.numel()) for e in eidx)
    print(f"split={split} quant={quant}: {n} sampled elements of 291 tensors, steps 1-2: no difference")
    del bufs, tl
    fo.release_cache()
    torch.cuda.empty_cache()
